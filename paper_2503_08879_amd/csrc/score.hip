// Eviction pass, scoring stage (paper Sec. 2 Step 2: attention scores of the last token's
// query against the cached keys).
//
//   score_kernel    streams K once: logit[g][i] = q[g].K[i]/sqrt(d) for the G heads of a row,
//                   fp32 logits to scratch, per-chunk softmax partials (max, sum exp).
//   stats_kernel    merges the partials of a row into (M, Z) per head, in fp64.
//   combine_kernel  score[i] = sum_g exp(logit[g][i] - M_g) / Z_g  (fp32) and the first radix
//                   histogram of the candidates' scores, merged across workgroups with atomics.
#include "device_utils.h"
#include "kernels.h"

namespace sagekv {

namespace {

constexpr int kScoreThreads = 256;
constexpr int kScoreWaves = kScoreThreads / kWave;
constexpr int kBlocksPerWave = kScoreChunk / (kScoreWaves * 64);  // 64-token blocks per wave

// One wave handles 64 tokens per block: LPT lanes share a token (16 bytes each), so one
// 16-byte load instruction covers TPL = 64/LPT whole tokens, fully coalesced; LPT such loads
// make a block.  After load i the lane with (lane % LPT) == i keeps the reduced dot product,
// so each lane ends a block owning exactly one token's logits for all heads.
template <int DT, int D, int GB>
__global__ __launch_bounds__(kScoreThreads) void score_kernel(ScoreParams p) {
  constexpr int EPL = Elem<DT>::per_lane;
  constexpr int EB = Elem<DT>::bytes;
  constexpr int LPT = D / EPL;
  constexpr int TPL = 64 / LPT;
  constexpr int SB = LPT < 8 ? LPT : 8;  // loads in flight per batch

  const int row = blockIdx.y;
  const int prob = row / p.geo.Hkv, c = row % p.geo.Hkv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int tq = lane / LPT, cl = lane % LPT;
  const int64_t L = p.geo.L;

  const char* Krow = (const char*)p.K + ((int64_t)prob * p.ks_problem + (int64_t)c * p.ks_head) * EB;
  const int64_t tok_bytes = p.ks_token * EB;

  uint4 q[GB];
#pragma unroll
  for (int g = 0; g < GB; ++g) {
    int h = c * p.geo.G + p.g0 + g;
    q[g] = ld16((const char*)p.q_last + (((int64_t)prob * p.geo.Hq + h) * D + cl * EPL) * EB);
  }

  float m[GB], sum[GB];
#pragma unroll
  for (int g = 0; g < GB; ++g) {
    m[g] = -INFINITY;
    sum[g] = 0.f;
  }

  const int64_t chunk_base = (int64_t)blockIdx.x * kScoreChunk;
  for (int blk = 0; blk < kBlocksPerWave; ++blk) {
    const int64_t tok_base = chunk_base + (int64_t)(wave * kBlocksPerWave + blk) * 64;
    if (tok_base >= L) break;  // wave-uniform
    float keep[GB];
#pragma unroll
    for (int g = 0; g < GB; ++g) keep[g] = 0.f;
#pragma unroll
    for (int i0 = 0; i0 < LPT; i0 += SB) {
      uint4 kv[SB];
#pragma unroll
      for (int i = 0; i < SB; ++i) {
        int64_t tok = tok_base + (i0 + i) * TPL + tq;
        tok = tok < L ? tok : L - 1;  // tail: re-read the last token, masked below
        kv[i] = ld16(Krow + tok * tok_bytes + cl * 16);
      }
#pragma unroll
      for (int i = 0; i < SB; ++i) {
#pragma unroll
        for (int g = 0; g < GB; ++g) {
          float v = group_sum<LPT>(dot16<DT>(kv[i], q[g], 0.f));
          keep[g] = (cl == i0 + i) ? v : keep[g];
        }
      }
    }
    const int64_t tok = tok_base + cl * TPL + tq;
    if (tok < L) {
#pragma unroll
      for (int g = 0; g < GB; ++g) {
        float x = keep[g] * p.scale;
        p.logits[((int64_t)row * p.geo.G + p.g0 + g) * p.geo.Lp + tok] = x;
        float mn = fmaxf(m[g], x);
        sum[g] = sum[g] * exp_fast(m[g] - mn) + exp_fast(x - mn);
        m[g] = mn;
      }
    }
  }

  // (max, sum) of the chunk: lanes -> wave -> workgroup
  __shared__ float2 part[kScoreWaves][GB];
#pragma unroll
  for (int g = 0; g < GB; ++g) {
    float M = wave_max(m[g]);
    float s = (m[g] == -INFINITY) ? 0.f : sum[g] * exp_fast(m[g] - M);
    s = group_sum<64>(s);
    if (lane == 0) part[wave][g] = make_float2(M, s);
  }
  __syncthreads();
  if (threadIdx.x < GB) {
    const int g = threadIdx.x;
    float M = part[0][g].x;
#pragma unroll
    for (int w = 1; w < kScoreWaves; ++w) M = fmaxf(M, part[w][g].x);
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < kScoreWaves; ++w) {
      float2 pw = part[w][g];
      s += (pw.x == -INFINITY) ? 0.f : pw.y * exp_fast(pw.x - M);
    }
    p.partials[((int64_t)row * p.geo.G + p.g0 + g) * p.n_chunks + blockIdx.x] = make_float2(M, s);
  }
}

__global__ __launch_bounds__(64) void stats_kernel(StatsParams p) {
  const int row = blockIdx.x, lane = threadIdx.x;
  for (int b = lane; b < kHistBins; b += 64) p.ghist[(int64_t)row * kHistBins + b] = 0;
  for (int g = 0; g < p.G; ++g) {
    const float2* pr = p.partials + ((int64_t)row * p.G + g) * p.n_chunks;
    float M = -INFINITY;
    for (int i = lane; i < p.n_chunks; i += 64) M = fmaxf(M, pr[i].x);
    M = wave_max(M);
    double z = 0.0;
    for (int i = lane; i < p.n_chunks; i += 64) {
      float2 v = pr[i];
      z += (double)v.y * exp((double)v.x - (double)M);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) z += __shfl_xor(z, o);
    if (lane == 0) {
      RowStat st;
      st.M = M;
      st.Z = z;
      st.invZ = (float)(1.0 / z);
      p.stats[(int64_t)row * p.G + g] = st;
    }
  }
}

constexpr int kCombineThreads = 256;
constexpr int kMaxG = 64;

__global__ __launch_bounds__(kCombineThreads) void combine_kernel(CombineParams p) {
  __shared__ int hist[kHistBins];
  __shared__ float sM[kMaxG], sInv[kMaxG];
  const int row = blockIdx.y, tid = threadIdx.x;
  const int G = p.geo.G;
  const int64_t L = p.geo.L, Lp = p.geo.Lp;
  for (int b = tid; b < kHistBins; b += kCombineThreads) hist[b] = 0;
  if (tid < G) {
    RowStat st = p.stats[(int64_t)row * G + tid];
    sM[tid] = st.M;
    sInv[tid] = st.invZ;
  }
  __syncthreads();
  const float* lg = p.logits + (int64_t)row * G * Lp;
  float* out = p.scores + (int64_t)row * p.pitch;
  const int64_t cand_lo = p.S, cand_hi = L - p.W;
  const bool vec_out = (p.pitch & 3) == 0;
  const int64_t base = (int64_t)blockIdx.x * kCombineChunk;
#pragma unroll
  for (int it = 0; it < kCombineChunk / (kCombineThreads * 4); ++it) {
    const int64_t tok = base + (int64_t)it * kCombineThreads * 4 + tid * 4;
    if (tok >= L) break;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int g = 0; g < G; ++g) {
      const float4 x = *reinterpret_cast<const float4*>(lg + (int64_t)g * Lp + tok);
      const float M = sM[g], inv = sInv[g];
      acc[0] += exp_accurate(x.x - M) * inv;
      acc[1] += exp_accurate(x.y - M) * inv;
      acc[2] += exp_accurate(x.z - M) * inv;
      acc[3] += exp_accurate(x.w - M) * inv;
    }
    if (vec_out && tok + 3 < L) {
      *reinterpret_cast<float4*>(out + tok) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (tok + j < L) out[tok + j] = acc[j];
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t t = tok + j;
      if (t >= cand_lo && t < cand_hi) atomicAdd(&hist[(__float_as_uint(acc[j]) >> 20) & (kHistBins - 1)], 1);
    }
  }
  __syncthreads();
  int* gh = p.ghist + (int64_t)row * kHistBins;
  for (int b = tid; b < kHistBins; b += kCombineThreads) {
    int v = hist[b];
    if (v) atomicAdd(&gh[b], v);
  }
}

template <int DT, int D>
hipError_t launch_score_g(const ScoreParams& p, int gb, dim3 grid, hipStream_t s) {
  switch (gb) {
#define SAGEKV_CASE(N) \
  case N:              \
    hipLaunchKernelGGL((score_kernel<DT, D, N>), grid, dim3(kScoreThreads), 0, s, p); \
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

int max_group_per_launch() { return 8; }

hipError_t launch_score(const ScoreParams& p0, hipStream_t s) {
  const int rows = p0.geo.n_problems * p0.geo.Hkv;
  dim3 grid((unsigned)p0.n_chunks, (unsigned)rows);
  for (int g0 = 0; g0 < p0.geo.G; g0 += max_group_per_launch()) {
    ScoreParams p = p0;
    p.g0 = g0;
    const int gb = p0.geo.G - g0 < max_group_per_launch() ? p0.geo.G - g0 : max_group_per_launch();
    hipError_t e;
    if (p.geo.dtype == DT_BF16)
      e = p.geo.D == 128 ? launch_score_g<DT_BF16, 128>(p, gb, grid, s) : launch_score_g<DT_BF16, 64>(p, gb, grid, s);
    else
      e = p.geo.D == 128 ? launch_score_g<DT_F32, 128>(p, gb, grid, s) : launch_score_g<DT_F32, 64>(p, gb, grid, s);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_stats(const StatsParams& p, int rows, hipStream_t s) {
  hipLaunchKernelGGL(stats_kernel, dim3((unsigned)rows), dim3(64), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_combine(const CombineParams& p, hipStream_t s) {
  const int rows = p.geo.n_problems * p.geo.Hkv;
  const unsigned nx = (unsigned)((p.geo.L + kCombineChunk - 1) / kCombineChunk);
  hipLaunchKernelGGL(combine_kernel, dim3(nx, (unsigned)rows), dim3(kCombineThreads), 0, s, p);
  return hipGetLastError();
}

}  // namespace sagekv
