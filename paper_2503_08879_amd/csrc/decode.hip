// Decoding over the reduced cache (paper Sec. 2 Step 4): the new token's (k, v) replaces the
// oldest entry of the recent window, then every query head attends over the reduced row.
//
// decode_kernel: grid (splits, rows).  A workgroup streams its slice of Kc and Vc once for all
// G heads of the row (16-byte loads, LPT lanes per token), keeps an online softmax per lane
// group and merges lane groups -> waves -> workgroup.  With one split per row (many rows: all
// layers of a step in one launch) a 16-wave workgroup owns the whole row and writes `out`
// itself; with few rows the row is split, partials (max, sum, acc[G][d]) go to scratch and
// combine_kernel merges them.  (A last-workgroup-done merge inside one kernel needs a device
// scope fence in every workgroup, which on this multi-XCD part writes back and invalidates
// L2: measured ~8x slower than two launches.)  The appended token is read from k_new / v_new
// directly and stored to its slot by the workgroup that owns it, so append and attention are
// one launch.
#include "device_utils.h"
#include "kernels.h"

namespace sagekv {

namespace {

template <int DT, int D, int GB, int NW>
__global__ __launch_bounds__(NW * 64) void decode_kernel(DecodeParams p, int g0) {
  constexpr int EPL = Elem<DT>::per_lane;
  constexpr int EB = Elem<DT>::bytes;
  constexpr int LPT = D / EPL;
  constexpr int TPL = 64 / LPT;
  constexpr int SB = (GB > 4 || NW > 4) ? 4 : 8;  // loads per batch
  constexpr int ROWB = D * EB;
  constexpr int kDecWaves = NW, kDecThreads = NW * 64;

  __shared__ float s_acc[kDecWaves][GB][D];
  __shared__ float2 s_ml[kDecWaves][GB];

  const int row = blockIdx.y, split = blockIdx.x;
  const int prob = row / p.Hkv, c = row % p.Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tq = lane / LPT, cl = lane % LPT;

  char* Kr = (char*)p.Kc + (int64_t)row * p.cap * ROWB;
  char* Vr = (char*)p.Vc + (int64_t)row * p.cap * ROWB;
  const char* kn = p.k_new ? (const char*)p.k_new + (int64_t)row * ROWB : nullptr;
  const char* vn = p.v_new ? (const char*)p.v_new + (int64_t)row * ROWB : nullptr;
  const int slot = kn ? p.slot : -1;

  const int t_begin = split * p.tokens_per_split;
  const int t_end = min(p.len, t_begin + p.tokens_per_split);

  if (slot >= t_begin && slot < t_end && tid < LPT) {  // Step 4: the new token enters the window
    st16(Kr + (int64_t)slot * ROWB + tid * 16, ld16(kn + tid * 16));
    st16(Vr + (int64_t)slot * ROWB + tid * 16, ld16(vn + tid * 16));
  }

  uint4 q[GB];
#pragma unroll
  for (int g = 0; g < GB; ++g) {
    const int h = c * p.G + g0 + g;
    q[g] = ld16((const char*)p.q + (((int64_t)prob * p.Hq + h) * D + cl * EPL) * EB);
  }
  float m[GB], l[GB], acc[GB][EPL];
#pragma unroll
  for (int g = 0; g < GB; ++g) {
    m[g] = -INFINITY;
    l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
  }

  for (int t0 = t_begin + wave * SB * TPL; t0 < t_end; t0 += kDecWaves * SB * TPL) {
    uint4 kv[SB], vv[SB];
    bool valid[SB];
#pragma unroll
    for (int i = 0; i < SB; ++i) {
      const int tok = t0 + i * TPL + tq;
      valid[i] = tok < t_end;
      const int tc = valid[i] ? tok : t_begin;
      const char* ks = (tc == slot) ? kn : Kr + (int64_t)tc * ROWB;
      const char* vs = (tc == slot) ? vn : Vr + (int64_t)tc * ROWB;
      kv[i] = p.stream_loads ? ld16_stream(ks + cl * 16) : ld16(ks + cl * 16);
      vv[i] = p.stream_loads ? ld16_stream(vs + cl * 16) : ld16(vs + cl * 16);
    }
    float x[SB][GB];
#pragma unroll
    for (int i = 0; i < SB; ++i)
#pragma unroll
      for (int g = 0; g < GB; ++g) {
        const float v = group_sum<LPT>(dot16<DT>(kv[i], q[g], 0.f)) * p.scale;
        x[i][g] = valid[i] ? v : -INFINITY;
      }
    float mn[GB];
    bool any = false;
#pragma unroll
    for (int g = 0; g < GB; ++g) {
      float bm = x[0][g];
#pragma unroll
      for (int i = 1; i < SB; ++i) bm = fmaxf(bm, x[i][g]);
      mn[g] = fmaxf(m[g], bm);
      any = any || (mn[g] != -INFINITY);
    }
    if (any) {  // lanes of one token group agree
#pragma unroll
      for (int g = 0; g < GB; ++g) {
        const float corr = exp_fast(m[g] - mn[g]);
        l[g] *= corr;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] *= corr;
        m[g] = mn[g];
      }
#pragma unroll
      for (int i = 0; i < SB; ++i) {
        float vf[EPL];
        unpack16<DT>(vv[i], vf);
#pragma unroll
        for (int g = 0; g < GB; ++g) {
          const float pw = exp_fast(x[i][g] - mn[g]);
          l[g] += pw;
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(pw, vf[e], acc[g][e]);
        }
      }
    }
  }

  // merge the TPL token groups of the wave (same cl, different tq)
#pragma unroll
  for (int g = 0; g < GB; ++g) {
    float M = m[g];
#pragma unroll
    for (int o = LPT; o < 64; o <<= 1) M = fmaxf(M, __shfl_xor(M, o));
    const float f = (m[g] == -INFINITY) ? 0.f : exp_fast(m[g] - M);
    float ls = l[g] * f;
#pragma unroll
    for (int o = LPT; o < 64; o <<= 1) ls += __shfl_xor(ls, o);
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      float a = acc[g][e] * f;
#pragma unroll
      for (int o = LPT; o < 64; o <<= 1) a += __shfl_xor(a, o);
      if (tq == 0) s_acc[wave][g][cl * EPL + e] = a;
    }
    if (lane == 0) s_ml[wave][g] = make_float2(M, ls);
  }
  __syncthreads();

  // merge the waves; one split: finish here, else write this split's partial
  const bool single = p.n_splits == 1;
  float* pa = p.part_acc + (((int64_t)row * p.n_splits + split) * p.G + g0) * D;
  float2* pml = p.part_ml + ((int64_t)row * p.n_splits + split) * p.G + g0;
  for (int it = tid; it < GB * D; it += kDecThreads) {
    const int g = it / D, j = it % D;
    float M = s_ml[0][g].x;
#pragma unroll
    for (int w = 1; w < kDecWaves; ++w) M = fmaxf(M, s_ml[w][g].x);
    float a = 0.f, ls = 0.f;
#pragma unroll
    for (int w = 0; w < kDecWaves; ++w) {
      const float2 ml = s_ml[w][g];
      const float f = (ml.x == -INFINITY) ? 0.f : exp_fast(ml.x - M);
      a += s_acc[w][g][j] * f;
      ls += ml.y * f;
    }
    if (single) {
      p.out[((int64_t)prob * p.Hq + c * p.G + g0 + g) * D + j] = a / ls;
    } else {
      pa[(int64_t)g * D + j] = a;
      if (j == 0) pml[g] = make_float2(M, ls);
    }
  }
}

// Merges the splits of a row: out = sum_s acc_s e^{m_s - M} / sum_s l_s e^{m_s - M}.
__global__ __launch_bounds__(256) void combine_kernel(DecodeParams p) {
  const int row = blockIdx.x, tid = threadIdx.x;
  const int prob = row / p.Hkv, c = row % p.Hkv;
  const int D = p.D;
  for (int it = tid; it < p.G * D; it += 256) {
    const int g = it / D, j = it % D;
    const float2* ml = p.part_ml + (int64_t)row * p.n_splits * p.G + g;
    const float* a = p.part_acc + ((int64_t)row * p.n_splits * p.G + g) * D + j;
    float M = -INFINITY;
    for (int s = 0; s < p.n_splits; ++s) M = fmaxf(M, ml[(int64_t)s * p.G].x);
    float num = 0.f, den = 0.f;
    for (int s = 0; s < p.n_splits; ++s) {
      const float2 v = ml[(int64_t)s * p.G];
      const float f = (v.x == -INFINITY) ? 0.f : exp_fast(v.x - M);
      num += a[(int64_t)s * p.G * D] * f;
      den += v.y * f;
    }
    p.out[((int64_t)prob * p.Hq + c * p.G + g) * D + j] = num / den;
  }
}

template <int LPT>
__global__ __launch_bounds__(64) void append_kernel(DecodeParams p, int row_bytes) {
  const int row = blockIdx.x, tid = threadIdx.x;
  if (tid >= LPT) return;
  char* Kr = (char*)p.Kc + ((int64_t)row * p.cap + p.slot) * row_bytes;
  char* Vr = (char*)p.Vc + ((int64_t)row * p.cap + p.slot) * row_bytes;
  st16(Kr + tid * 16, ld16((const char*)p.k_new + (int64_t)row * row_bytes + tid * 16));
  st16(Vr + tid * 16, ld16((const char*)p.v_new + (int64_t)row * row_bytes + tid * 16));
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t* p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = 0u;
}

template <int DT, int D>
hipError_t launch_decode_g(const DecodeParams& p, int g0, int gb, dim3 grid, hipStream_t s) {
  const bool single = p.n_splits == 1;  // one workgroup per row: use a big one
  switch (gb) {
#define SAGEKV_CASE(N)                                                                               \
  case N:                                                                                            \
    if (!single)                                                                                     \
      hipLaunchKernelGGL((decode_kernel<DT, D, N, 4>), grid, dim3(256), 0, s, p, g0);                \
    else if (N <= 4)                                                                                 \
      hipLaunchKernelGGL((decode_kernel<DT, D, N, 16>), grid, dim3(1024), 0, s, p, g0);              \
    else                                                                                             \
      hipLaunchKernelGGL((decode_kernel<DT, D, N, 8>), grid, dim3(512), 0, s, p, g0);                \
    break;
    SAGEKV_CASE(1) SAGEKV_CASE(2) SAGEKV_CASE(3) SAGEKV_CASE(4)
    SAGEKV_CASE(5) SAGEKV_CASE(6) SAGEKV_CASE(7) SAGEKV_CASE(8)
#undef SAGEKV_CASE
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_decode(const DecodeParams& p, hipStream_t s) {
  const int rows = p.n_problems * p.Hkv;
  dim3 grid((unsigned)p.n_splits, (unsigned)rows);
  for (int g0 = 0; g0 < p.G; g0 += max_group_per_launch()) {
    const int gb = p.G - g0 < max_group_per_launch() ? p.G - g0 : max_group_per_launch();
    DecodeParams q = p;
    if (g0 > 0) q.k_new = nullptr;  // the first launch already stored the new token
    hipError_t e;
    if (p.dtype == DT_BF16)
      e = p.D == 128 ? launch_decode_g<DT_BF16, 128>(q, g0, gb, grid, s) : launch_decode_g<DT_BF16, 64>(q, g0, gb, grid, s);
    else
      e = p.D == 128 ? launch_decode_g<DT_F32, 128>(q, g0, gb, grid, s) : launch_decode_g<DT_F32, 64>(q, g0, gb, grid, s);
    if (e != hipSuccess) return e;
  }
  if (p.n_splits > 1) {
    hipLaunchKernelGGL(combine_kernel, dim3((unsigned)rows), dim3(256), 0, s, p);
    return hipGetLastError();
  }
  return hipSuccess;
}

hipError_t launch_append(const DecodeParams& p, hipStream_t s) {
  const int rows = p.n_problems * p.Hkv;
  const int eb = p.dtype == DT_BF16 ? 2 : 4;
  const int row_bytes = p.D * eb;
  switch (row_bytes / 16) {
    case 8: hipLaunchKernelGGL(append_kernel<8>, dim3((unsigned)rows), dim3(64), 0, s, p, row_bytes); break;
    case 16: hipLaunchKernelGGL(append_kernel<16>, dim3((unsigned)rows), dim3(64), 0, s, p, row_bytes); break;
    case 32: hipLaunchKernelGGL(append_kernel<32>, dim3((unsigned)rows), dim3(64), 0, s, p, row_bytes); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_fill_zero(void* ptr, size_t bytes, hipStream_t s) {
  const size_t n = bytes / 4;
  if (n == 0) return hipSuccess;
  size_t want = (n + 255) / 256;
  unsigned grid = (unsigned)(want < 4096 ? want : 4096);
  hipLaunchKernelGGL(fill_zero_kernel, dim3(grid), dim3(256), 0, s, (uint32_t*)ptr, n);
  return hipGetLastError();
}

}  // namespace sagekv
