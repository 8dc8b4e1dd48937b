// Decoding over the reduced cache (paper Sec. 2 Step 4): the new token's (k, v) replaces the
// oldest entry of the recent window, then every query head attends over the reduced row.
//
// decode_kernel: grid (splits, rows).  A workgroup streams its slice of Kc and Vc once for all
// G heads of the row (16-byte loads, LPT lanes per token), keeps an online softmax per lane
// group and merges lane groups -> waves -> workgroup.  With one split per row (many rows: all
// layers of a step in one launch) one workgroup (8 waves bf16, up to 16 fp32) owns the whole row and
// writes `out` itself; with few rows the row is split, partials (max, sum, acc[G][d]) go to scratch and
// combine_kernel merges them.  (A last-workgroup-done merge inside one kernel needs a device
// scope fence in every workgroup, which on this multi-XCD part writes back and invalidates
// L2: measured ~8x slower than two launches.)  The appended token is read from k_new / v_new
// directly and stored to its slot by the workgroup that owns it, so append and attention are
// one launch.
#include "device_utils.h"
#include "kernels.h"

namespace sagekv {

namespace {

// Slot of the new token, attended length and slice size of this launch: the host's values, or
// derived from the device-side count of appended tokens.
struct StepGeom {
  int slot, len, tokens_per_split, n_appended;
};
__device__ __forceinline__ StepGeom step_geom(const DecodeParams& p) {
  StepGeom s = {p.k_new ? p.slot : -1, p.len, p.tokens_per_split, 0};
  if (p.ring) {
    s.n_appended = p.ring[0];
    const RingPos r = ring_position(p.ring_base, p.ring_W, p.ring_grow, p.cap, s.n_appended < 0 ? 0 : s.n_appended);
    s.slot = p.k_new ? r.slot : -1;
    s.len = r.len;
    s.tokens_per_split = split_tokens(r.len, p.n_splits);
  }
  return s;
}

// Called once per row of a launch whose workgroups own whole rows: the last row to finish advances
// the device-side count (for sliced rows the merge launch does).  Every workgroup has read ring[0] before it gets here (the
// value went into its addresses), so the store cannot overtake a reader; the next launch on the
// stream sees it.  Only the counter itself is exchanged between workgroups: relaxed atomics, no
// cache-wide fence.
__device__ __forceinline__ void row_done(const DecodeParams& p, const StepGeom& sg) {
  if (!p.ring || !p.ring_advance) return;
  const int rows = (int)gridDim.y;
  const int ticket = __hip_atomic_fetch_add(&p.ring[1], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (ticket == rows - 1) {
    __hip_atomic_store(&p.ring[1], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&p.ring[0], sg.n_appended + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// out[head g][dim j] of a row from its slices: sum_s acc_s e^{m_s - M} / sum_s l_s e^{m_s - M}.
// One pass; the loads of up to 32 slices are all issued before the first is used (one memory round
// trip), the arithmetic then goes through them eight at a time.
__device__ __forceinline__ float merge_slices(const DecodeParams& p, int row, int g, int j) {
  const float* ml = reinterpret_cast<const float*>(p.part_ml + (int64_t)row * p.n_splits * p.G + g);
  const float* a = p.part_acc + ((int64_t)row * p.n_splits * p.G + g) * p.D + j;
  float M = -INFINITY, num = 0.f, den = 0.f;
  for (int s0 = 0; s0 < p.n_splits; s0 += 32) {
    float vm[32], vl[32], av[32];
#pragma unroll
    for (int u = 0; u < 32; ++u) {
      const int s = s0 + u < p.n_splits ? s0 + u : p.n_splits - 1;
      vm[u] = ml[(int64_t)s * p.G * 2];
      vl[u] = ml[(int64_t)s * p.G * 2 + 1];
      av[u] = a[(int64_t)s * p.G * p.D];
    }
#pragma unroll
    for (int u0 = 0; u0 < 32; u0 += 8) {
      if (s0 + u0 >= p.n_splits) break;
      float Mn = M;
#pragma unroll
      for (int u = u0; u < u0 + 8; ++u) {
        if (s0 + u >= p.n_splits) vm[u] = -INFINITY;
        Mn = fmaxf(Mn, vm[u]);
      }
      if (Mn == -INFINITY) continue;  // nothing attended in these slices (uniform over the workgroup)
      const float f0 = (M == -INFINITY) ? 0.f : exp_fast(M - Mn);
      num *= f0;
      den *= f0;
#pragma unroll
      for (int u = u0; u < u0 + 8; ++u) {
        const float f = (vm[u] == -INFINITY) ? 0.f : exp_fast(vm[u] - Mn);
        num = fmaf(av[u], f, num);
        den = fmaf(vl[u], f, den);
      }
      M = Mn;
    }
  }
  return num / den;
}

// End of a decode workgroup that owns its whole row: the row is done.  (Sliced rows are completed
// by the merge launch.)
__device__ __forceinline__ void finish_row(const DecodeParams& p, const StepGeom& sg) {
  if (p.n_splits == 1 && threadIdx.x == 0) row_done(p, sg);
}

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

  const CacheRow Kr = cache_row(p.Kc, p.cpm, false, prob, c, row, p.cap, ROWB, EB);
  const CacheRow Vr = cache_row(p.Vc, p.cpm, true, prob, c, row, p.cap, ROWB, EB);
  const char* kn = p.k_new ? (const char*)p.k_new + (int64_t)row * ROWB : nullptr;
  const char* vn = p.v_new ? (const char*)p.v_new + (int64_t)row * ROWB : nullptr;
  const StepGeom sg = step_geom(p);
  const int slot = sg.slot;

  const int t_begin = split * sg.tokens_per_split;
  const int t_end = min(sg.len, t_begin + sg.tokens_per_split);

  if (slot >= t_begin && slot < t_end && tid < LPT) {  // Step 4: the new token enters the window
    st16(Kr.at(slot) + tid * 16, ld16(kn + tid * 16));
    st16(Vr.at(slot) + tid * 16, ld16(vn + tid * 16));
  }

  uint4 q[GB], q2[GB];  // q2: the sink tokens' query (window-relative positions), else = q
#pragma unroll
  for (int g = 0; g < GB; ++g) {
    const int h = c * p.G + g0 + g;
    q[g] = ld16((const char*)p.q + (((int64_t)prob * p.Hq + h) * D + cl * EPL) * EB);
    q2[g] = p.q_sink ? ld16((const char*)p.q_sink + (((int64_t)prob * p.Hq + h) * D + cl * EPL) * EB) : q[g];
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
      const char* ks = (tc == slot) ? kn : Kr.at(tc);
      const char* vs = (tc == slot) ? vn : Vr.at(tc);
      kv[i] = ld16(ks + cl * 16);
      vv[i] = ld16(vs + cl * 16);
    }
    // fp32 caches: the logit in fp64 (exact products), and below the exponent's argument from the fp64
    // logit: an fp32 logit of magnitude 100 would be off by 2.5e-5, and so would its softmax weight
    constexpr bool F64 = DT == DT_F32;
    float x[SB][GB];
    double xd[F64 ? SB : 1][F64 ? GB : 1];
#pragma unroll
    for (int i = 0; i < SB; ++i)
#pragma unroll
      for (int g = 0; g < GB; ++g) {
        const int tok = t0 + i * TPL + tq;
        const uint4& qq = tok < p.qs_S ? q2[g] : q[g];
        float v;
        if constexpr (F64) {
          double a = (double)__uint_as_float(kv[i].x) * (double)__uint_as_float(qq.x) +
                     (double)__uint_as_float(kv[i].y) * (double)__uint_as_float(qq.y) +
                     (double)__uint_as_float(kv[i].z) * (double)__uint_as_float(qq.z) +
                     (double)__uint_as_float(kv[i].w) * (double)__uint_as_float(qq.w);
#pragma unroll
          for (int o = 1; o < LPT; o <<= 1) a += __shfl_xor(a, o);
          a *= 1.0 / sqrt((double)D);
          xd[i][g] = a;
          v = (float)a;
        } else {
          v = group_sum<LPT>(dot16<DT>(kv[i], qq, 0.f)) * p.scale;
        }
        x[i][g] = valid[i] && head_attends(p.pq_S, p.pq_k, p.G, g0 + g, tok) ? v : -INFINITY;
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
        const float corr = (mn[g] == -INFINITY) ? 1.f : exp_fast(m[g] - mn[g]);  // head with nothing to attend yet
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
          float arg = x[i][g] - mn[g];
          if constexpr (F64) arg = (float)(xd[i][g] - (double)mn[g]);
          const float pw = (x[i][g] == -INFINITY) ? 0.f : exp_fast(arg);
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
  finish_row(p, sg);
}

// bf16 decode with the q.K products on the matrix cores.  Per 32-token block a wave stages K
// through XOR-swizzled LDS into v_mfma_f32_16x16x32_bf16 (A = queries, zero padded to GPAD heads),
// so a lane ends with the 4 logits of one token: the softmax weights are computed once per
// (token, head) instead of once per lane, then handed through LDS to the lanes that hold the V
// chunks (16 lanes per token, fp32 FMA accumulation).  K and V of block b+1 are both in flight
// while block b is processed (two 8-load register buffers per wave).  STREAM: the reduced cache
// does not fit the on-chip caches between steps, read it with streaming loads.
template <int D, int GPAD, int NW, bool STREAM, bool PG>
__global__ __launch_bounds__(NW * 64) void decode_mfma_kernel(DecodeParams p, int g0, int gb) {
  constexpr int BT = GPAD > 4 ? 16 : 32;                   // tokens per block (registers: acc is GPAD x 8)
  constexpr int CH = D / 8, TPL = 64 / CH, NLOAD = BT / TPL, KSTEPS = D / 32;
  constexpr int TILES = 16 / GPAD;                         // 16-token tiles sharing the accumulator rows
  constexpr int NT = BT / 16;                              // tiles per block (<= TILES for GPAD <= 8)
  constexpr int ROWB = D * 2, EPL = 8;
  constexpr int kThreads = NW * 64;
  static_assert(NT <= TILES, "one accumulator per block");

  __shared__ uint4 kbuf[NW][BT * CH];
  __shared__ float pbuf[NW][BT][GPAD];
  __shared__ float cbuf[NW][GPAD];
  __shared__ float2 s_ml[NW][GPAD];

  const int row = blockIdx.y, split = blockIdx.x;
  const int prob = row / p.Hkv, c = row % p.Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tq = lane / CH, cl = lane % CH;  // load / PV role: token sub-index, 16-byte chunk
  const int n = lane & 15, j = lane >> 4;    // MFMA role: column (token), row block

  const CacheRowT<PG, ROWB> Kr = {cache_row(p.Kc, p.cpm, false, prob, c, row, p.cap, ROWB, 2)};
  const CacheRowT<PG, ROWB> Vr = {cache_row(p.Vc, p.cpm, true, prob, c, row, p.cap, ROWB, 2)};
  const char* kn = p.k_new ? (const char*)p.k_new + (int64_t)row * ROWB : nullptr;
  const char* vn = p.v_new ? (const char*)p.v_new + (int64_t)row * ROWB : nullptr;
  const StepGeom sg = step_geom(p);
  const int slot = sg.slot;
  const int t_begin = split * sg.tokens_per_split;
  const int t_end = min(sg.len, t_begin + sg.tokens_per_split);
  if (slot >= t_begin && slot < t_end && tid < CH) {  // Step 4: the new token enters the window
    st16(Kr.at(slot) + tid * 16, ld16(kn + tid * 16));
    st16(Vr.at(slot) + tid * 16, ld16(vn + tid * 16));
  }

  // accumulator rows 4j..4j+3 = (tile slot, heads hbase..hbase+3); slots >= NT stay empty
  const int hbase = (4 * j) % GPAD, tile = (4 * j) / GPAD;
  const int t_mine = tile * 16 + n;  // this lane's token within the block (MFMA role)
  float m_run[4], l_part[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    m_run[r] = -INFINITY;
    l_part[r] = 0.f;
  }
  float acc[GPAD][EPL];
#pragma unroll
  for (int g = 0; g < GPAD; ++g)
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;

  uint4* buf = kbuf[wave];
  const int nblk = (t_end - t_begin + BT - 1) / BT;
  uint4 kv[NLOAD], vv[NLOAD];
  auto load_block = [&](int b, uint4* dst, const CacheRowT<PG, ROWB>& base, const char* fresh) {
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
      const int tok = t_begin + b * BT + i * TPL + tq;
      const int tc = tok < t_end ? tok : t_begin;
      const char* src = (tc == slot) ? fresh : base.at(tc);
      dst[i] = STREAM ? ld16_stream(src + cl * 16) : ld16(src + cl * 16);
    }
  };
  if (wave < nblk) {  // first blocks in flight before anything else is waited for
    load_block(wave, kv, Kr, kn);
    load_block(wave, vv, Vr, vn);
  }
  // A operand of tile slot ts, k-step kc, kept in LDS (registers are short here): lane (row m = n,
  // k-group j) reads q[head m % GPAD][8*(4*kc + j) ..+8] if m / GPAD == ts, zeros otherwise
  // Set 1 holds the query the sink tokens are scored with, when the caller gives one.
  __shared__ uint4 qbuf[2][NT][KSTEPS][64];
  for (int it = tid; it < (p.q_sink ? 2 : 1) * NT * KSTEPS * 64; it += kThreads) {
    const int l = it & 63, kc = (it >> 6) % KSTEPS, ts = (it / (64 * KSTEPS)) % NT, set = it / (64 * KSTEPS * NT);
    const int m = l & 15, jj = l >> 4;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (m % GPAD < gb && m / GPAD == ts) {
      const int h = c * p.G + g0 + m % GPAD;
      v = ld16((const char*)(set ? p.q_sink : p.q) + (((int64_t)prob * p.Hq + h) * D + (4 * kc + jj) * 8) * 2);
    }
    qbuf[set][ts][kc][l] = v;
  }
  __syncthreads();
  for (int b = wave; b < nblk; b += NW) {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");  // last block's LDS reads are done
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
      const int t = i * TPL + tq;
      buf[t * CH + (cl ^ (t & (CH - 1)))] = kv[i];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    const bool more = b + NW < nblk;
    if (more) load_block(b + NW, kv, Kr, kn);

    // logits of the block
    f32x4_t d = f32x4_t{0.f, 0.f, 0.f, 0.f}, ds = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const bool sink_blk = p.q_sink && t_begin + b * BT < p.qs_S;  // wave-uniform: the block holds sink tokens
#pragma unroll
    for (int ts = 0; ts < NT; ++ts) {
      const int t = ts * 16 + n;
#pragma unroll
      for (int kc = 0; kc < KSTEPS; ++kc) {
        const uint4 bb = buf[t * CH + ((4 * kc + j) ^ (n & (CH - 1)))];
        const uint4 qv = qbuf[0][ts][kc][lane];
        d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, qv), __builtin_bit_cast(bf16x8_t, bb), d,
                                                    0, 0, 0);
        if (sink_blk) {
          const uint4 qs = qbuf[1][ts][kc][lane];
          ds = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, qs), __builtin_bit_cast(bf16x8_t, bb),
                                                       ds, 0, 0, 0);
        }
      }
    }
    const int tok = t_begin + b * BT + t_mine;
    float x[4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
      x[r] = (tile < NT && tok < t_end && hbase + r < gb && head_attends(p.pq_S, p.pq_k, p.G, g0 + hbase + r, tok))
                 ? (sink_blk && tok < p.qs_S ? ds[r] : d[r]) * p.scale
                 : -INFINITY;

    // online softmax, once per (token, head); lanes with the same heads agree on the maximum
    float corr[4], pw[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float bm = x[r];
#pragma unroll
      for (int o = 1; o < 16; o <<= 1) bm = fmaxf(bm, __shfl_xor(bm, o));
#pragma unroll
      for (int o = 16 * (GPAD / 4); o < 64; o <<= 1) bm = fmaxf(bm, __shfl_xor(bm, o));
      const float mn = fmaxf(m_run[r], bm);
      corr[r] = (mn == -INFINITY) ? 1.f : exp_fast(m_run[r] - mn);
      pw[r] = (x[r] == -INFINITY) ? 0.f : exp_fast(x[r] - mn);
      l_part[r] = l_part[r] * corr[r] + pw[r];
      m_run[r] = mn;
    }
    if (tile < NT) *reinterpret_cast<float4*>(&pbuf[wave][t_mine][hbase]) = make_float4(pw[0], pw[1], pw[2], pw[3]);
    if (n == 0 && j < GPAD / 4)
      *reinterpret_cast<float4*>(&cbuf[wave][hbase]) = make_float4(corr[0], corr[1], corr[2], corr[3]);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");

    // P.V on the lanes that hold the V chunks
#pragma unroll
    for (int g4 = 0; g4 < GPAD / 4; ++g4) {
      const float4 c4 = *reinterpret_cast<const float4*>(&cbuf[wave][g4 * 4]);
      const float cr[4] = {c4.x, c4.y, c4.z, c4.w};
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g4 * 4 + r][e] *= cr[r];
    }
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
      if (GPAD > 4) __builtin_amdgcn_sched_barrier(0);  // keep the unrolled steps apart: registers
      const int t_local = i * TPL + tq;
      float vf[EPL];
      unpack16<DT_BF16>(vv[i], vf);
      if (more) {  // the register is free: V of the next block, as early as possible
        const int tokn = t_begin + (b + NW) * BT + i * TPL + tq;
        const int tcn = tokn < t_end ? tokn : t_begin;
        const char* src = (tcn == slot) ? vn : Vr.at(tcn);
        vv[i] = STREAM ? ld16_stream(src + cl * 16) : ld16(src + cl * 16);
      }
#pragma unroll
      for (int g4 = 0; g4 < GPAD / 4; ++g4) {
        const float4 p4 = *reinterpret_cast<const float4*>(&pbuf[wave][t_local][g4 * 4]);
        const float pp[4] = {p4.x, p4.y, p4.z, p4.w};
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc[g4 * 4 + r][e] = fmaf(pp[r], vf[e], acc[g4 * 4 + r][e]);
      }
    }
  }

  // wave totals: sum of weights per head, accumulators over the TPL token groups
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    float ls = l_part[r];
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) ls += __shfl_xor(ls, o);
#pragma unroll
    for (int o = 16 * (GPAD / 4); o < 64; o <<= 1) ls += __shfl_xor(ls, o);
    if (n == 0 && j < GPAD / 4) s_ml[wave][hbase + r] = make_float2(m_run[r], ls);
  }
  __syncthreads();  // every wave is done with its K buffer: reuse it for the accumulators
  float* s_acc = reinterpret_cast<float*>(&kbuf[0][0]);  // [NW][GPAD][D]
  static_assert(GPAD * D * 4 <= BT * CH * 16 + 0 * NW, "accumulators fit the K buffers");
#pragma unroll
  for (int g = 0; g < GPAD; ++g)
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      float a = acc[g][e];
#pragma unroll
      for (int o = CH; o < 64; o <<= 1) a += __shfl_xor(a, o);
      if (tq == 0) s_acc[((wave * GPAD) + g) * D + cl * EPL + e] = a;
    }
  __syncthreads();

  const bool single = p.n_splits == 1;
  float* pa = p.part_acc + (((int64_t)row * p.n_splits + split) * p.G + g0) * D;
  float2* pml = p.part_ml + ((int64_t)row * p.n_splits + split) * p.G + g0;
  for (int it = tid; it < gb * D; it += kThreads) {
    const int g = it / D, jj = it % D;
    float M = s_ml[0][g].x;
#pragma unroll
    for (int w = 1; w < NW; ++w) M = fmaxf(M, s_ml[w][g].x);
    float a = 0.f, ls = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float2 ml = s_ml[w][g];
      const float f = (ml.x == -INFINITY) ? 0.f : exp_fast(ml.x - M);
      a += s_acc[((w * GPAD) + g) * D + jj] * f;
      ls += ml.y * f;
    }
    if (single) {
      p.out[((int64_t)prob * p.Hq + c * p.G + g0 + g) * D + jj] = a / ls;
    } else {
      pa[(int64_t)g * D + jj] = a;
      if (jj == 0) pml[g] = make_float2(M, ls);
    }
  }
  finish_row(p, sg);
}

// bf16 decode with BOTH products on the matrix cores.  q.K as in decode_mfma_kernel.  The softmax
// weights of a 32-token block are rounded to bf16 (as the values are) and written to LDS as
// P[head][token]; V goes through the wave's staging buffer like K, and a lane gets the MFMA B operand
// V[8 tokens][its dim] with two transposed LDS reads (ds_read_b64_tr_b16: lane s of a 16-lane group
// addresses 4 dims of token s / 4 and receives dim s of 4 tokens).
// out[head][dim] accumulates in one 16x16 tile per 16 dims, rows = heads, so the accumulator does not
// grow with the group size and the vector ALU no longer does G x head_dim multiply-adds per token.
__device__ __forceinline__ uint32_t bf16_rne(float f) {  // finite, non-negative input
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

template <int D, int GPAD, int NW, bool STREAM, bool PG>
__global__ __launch_bounds__(NW * 64) void decode_pv_mfma_kernel(DecodeParams p, int g0, int gb) {
  constexpr int BT = 32;
  constexpr int CH = D / 8, TPL = 64 / CH, NLOAD = BT / TPL, KSTEPS = D / 32;
  constexpr int TILES = 16 / GPAD;                       // 16-token tiles sharing a q.K accumulator
  constexpr int NT = BT / 16;                            // token tiles per block
  constexpr int NACC = NT > TILES ? NT / TILES : 1;      // q.K accumulators per block
  constexpr int NDT = D / 16;                            // output tiles (16 dims each)
  constexpr int ROWB = D * 2;
  constexpr int kThreads = NW * 64;
  static_assert(GPAD * D * 4 <= BT * CH * 16, "accumulators fit the staging buffers");

  __shared__ uint4 kbuf[NW][BT * CH];  // K staging, then V staging, at the end the waves' accumulators
  __shared__ __attribute__((aligned(16))) unsigned short pT[NW][16][BT];  // weights, bf16, [head][token]
  __shared__ float2 s_ml[NW][GPAD];
  __shared__ uint4 qbuf[2][NT][KSTEPS][64];

  const int row = blockIdx.y, split = blockIdx.x;
  const int prob = row / p.Hkv, c = row % p.Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tq = lane / CH, cl = lane % CH;  // load role: token sub-index, 16-byte chunk
  const int n = lane & 15, j = lane >> 4;    // MFMA role: column, row block / k-group

  const CacheRowT<PG, ROWB> Kr = {cache_row(p.Kc, p.cpm, false, prob, c, row, p.cap, ROWB, 2)};
  const CacheRowT<PG, ROWB> Vr = {cache_row(p.Vc, p.cpm, true, prob, c, row, p.cap, ROWB, 2)};
  const char* kn = p.k_new ? (const char*)p.k_new + (int64_t)row * ROWB : nullptr;
  const char* vn = p.v_new ? (const char*)p.v_new + (int64_t)row * ROWB : nullptr;
  const StepGeom sg = step_geom(p);
  const int slot = sg.slot;
  const int t_begin = split * sg.tokens_per_split;
  const int t_end = min(sg.len, t_begin + sg.tokens_per_split);
  if (slot >= t_begin && slot < t_end && tid < CH) {  // Step 4: the new token enters the window
    st16(Kr.at(slot) + tid * 16, ld16(kn + tid * 16));
    st16(Vr.at(slot) + tid * 16, ld16(vn + tid * 16));
  }

  // q.K accumulator a, register r of lane (j, n): head hbase + r, token tile a * TILES + tslot, column n
  const int hbase = (4 * j) % GPAD, tslot = (4 * j) / GPAD;
  float m_run[4], l_part[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    m_run[r] = -INFINITY;
    l_part[r] = 0.f;
  }
  f32x4_t acc[NDT];  // out[head 4j + r][dim 16 * nd + n]
#pragma unroll
  for (int nd = 0; nd < NDT; ++nd) acc[nd] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  uint4* buf = kbuf[wave];
  reinterpret_cast<uint4*>(&pT[wave][0][0])[lane] = make_uint4(0u, 0u, 0u, 0u);  // rows of absent heads stay 0
  const int nblk = (t_end - t_begin + BT - 1) / BT;
  uint4 kv[NLOAD], vv[NLOAD];
  auto load_block = [&](int b, uint4* dst, const CacheRowT<PG, ROWB>& base, const char* fresh) {
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
      const int tok = t_begin + b * BT + i * TPL + tq;
      const int tc = tok < t_end ? tok : t_begin;
      const char* src = (tc == slot) ? fresh : base.at(tc);
      dst[i] = STREAM ? ld16_stream(src + cl * 16) : ld16(src + cl * 16);
    }
  };
  if (wave < nblk) {
    load_block(wave, kv, Kr, kn);
    load_block(wave, vv, Vr, vn);
  }
  for (int it = tid; it < (p.q_sink ? 2 : 1) * NT * KSTEPS * 64; it += kThreads) {
    const int l = it & 63, kc = (it >> 6) % KSTEPS, ts = (it / (64 * KSTEPS)) % NT, set = it / (64 * KSTEPS * NT);
    const int m = l & 15, jj = l >> 4;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (m % GPAD < gb && m / GPAD == ts % TILES) {
      const int h = c * p.G + g0 + m % GPAD;
      v = ld16((const char*)(set ? p.q_sink : p.q) + (((int64_t)prob * p.Hq + h) * D + (4 * kc + jj) * 8) * 2);
    }
    qbuf[set][ts][kc][l] = v;
  }
  __syncthreads();

  // V staging swizzle (16-byte chunk ^= vswz(token)): the four tokens a 16-lane group reads together
  // land in different banks
  auto vswz = [](int t) { return CH == 16 ? (((t & 3) << 1) | (((t >> 3) & 1) << 3)) : ((t & 3) << 1); };

  for (int b = wave; b < nblk; b += NW) {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");  // last block's reads of the buffer are done
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
      const int t = i * TPL + tq;
      buf[t * CH + (cl ^ (t & (CH - 1)))] = kv[i];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    const bool more = b + NW < nblk;
    if (more) load_block(b + NW, kv, Kr, kn);

    f32x4_t d[NACC], ds[NACC];
#pragma unroll
    for (int a = 0; a < NACC; ++a) d[a] = ds[a] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const bool sink_blk = p.q_sink && t_begin + b * BT < p.qs_S;  // wave-uniform: the block holds sink tokens
#pragma unroll
    for (int ts = 0; ts < NT; ++ts) {
      const int t = ts * 16 + n, a = ts / TILES;
#pragma unroll
      for (int kc = 0; kc < KSTEPS; ++kc) {
        const uint4 bb = buf[t * CH + ((4 * kc + j) ^ (n & (CH - 1)))];
        d[a] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, qbuf[0][ts][kc][lane]),
                                                       __builtin_bit_cast(bf16x8_t, bb), d[a], 0, 0, 0);
        if (sink_blk)
          ds[a] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, qbuf[1][ts][kc][lane]),
                                                          __builtin_bit_cast(bf16x8_t, bb), ds[a], 0, 0, 0);
      }
    }
    float x[NACC][4];
#pragma unroll
    for (int a = 0; a < NACC; ++a) {
      const int tile = a * TILES + tslot;
      const int tok = t_begin + b * BT + tile * 16 + n;
#pragma unroll
      for (int r = 0; r < 4; ++r)
        x[a][r] = (tile < NT && tok < t_end && hbase + r < gb && head_attends(p.pq_S, p.pq_k, p.G, g0 + hbase + r, tok))
                      ? (sink_blk && tok < p.qs_S ? ds[a][r] : d[a][r]) * p.scale
                      : -INFINITY;
    }
    // online softmax, once per (token, head); lanes with the same heads agree on the maximum
    float corr[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float bm = x[0][r];
#pragma unroll
      for (int a = 1; a < NACC; ++a) bm = fmaxf(bm, x[a][r]);
#pragma unroll
      for (int o = 1; o < 16; o <<= 1) bm = fmaxf(bm, __shfl_xor(bm, o));
#pragma unroll
      for (int o = 16 * (GPAD / 4); o < 64; o <<= 1) bm = fmaxf(bm, __shfl_xor(bm, o));
      const float mn = fmaxf(m_run[r], bm);
      corr[r] = (mn == -INFINITY) ? 1.f : exp_fast(m_run[r] - mn);
      float lsum = 0.f;
#pragma unroll
      for (int a = 0; a < NACC; ++a) {
        const uint32_t pb = (x[a][r] == -INFINITY) ? 0u : bf16_rne(exp_fast(x[a][r] - mn));
        lsum += __uint_as_float(pb << 16);  // the denominator sums the weights the numerator uses
        const int tile = a * TILES + tslot;
        if (tile < NT) pT[wave][hbase + r][tile * 16 + n] = (unsigned short)pb;
      }
      l_part[r] = l_part[r] * corr[r] + lsum;
      m_run[r] = mn;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");  // weights visible; q.K reads of the buffer done

    // V of the block into the staging buffer, V of the next block into the registers
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
      const int t = i * TPL + tq;
      buf[t * CH + (cl ^ vswz(t))] = vv[i];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    if (more) load_block(b + NW, vv, Vr, vn);

    // out += P.V: A = weights [head n][tokens 8j..8j+7], B = values [tokens 8j..8j+7][dim 16 nd + n]
    const uint4 pa = *reinterpret_cast<const uint4*>(&pT[wave][n][8 * j]);
#pragma unroll
    for (int nd = 0; nd < NDT; ++nd) {
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[nd][r] *= corr[r];  // rows 4j + r are heads hbase + r for every j in use
      // transposed LDS read: lane s of a 16-lane group gives the address of 4 dims of token s / 4
      // and receives its own dim of 4 tokens
      typedef short v4s_t __attribute__((ext_vector_type(4)));
      const int tu = 8 * j + (n >> 2);                       // first token this lane addresses
      const int cch = (2 * nd + ((n & 3) >> 1)) ^ vswz(tu);  // vswz(tu) = vswz(tu + 4)
      const unsigned short* b16 = reinterpret_cast<const unsigned short*>(buf);
      const v4s_t x0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) v4s_t*)(b16 + (tu * CH + cch) * 8 + (n & 1) * 4));
      const v4s_t x1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) v4s_t*)(b16 + ((tu + 4) * CH + cch) * 8 + (n & 1) * 4));
      struct { v4s_t a, b; } pair = {x0, x1};
      const uint4 vb = __builtin_bit_cast(uint4, pair);
      acc[nd] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, pa), __builtin_bit_cast(bf16x8_t, vb),
                                                        acc[nd], 0, 0, 0);
    }
  }

  // wave totals: sum of weights per head over the lanes that share it
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    float ls = l_part[r];
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) ls += __shfl_xor(ls, o);
#pragma unroll
    for (int o = 16 * (GPAD / 4); o < 64; o <<= 1) ls += __shfl_xor(ls, o);
    if (n == 0 && j < GPAD / 4) s_ml[wave][hbase + r] = make_float2(m_run[r], ls);
  }
  __syncthreads();  // every wave is done with its staging buffer: reuse it for the accumulators
  float* s_acc = reinterpret_cast<float*>(&kbuf[0][0]);  // [NW][GPAD][D]
#pragma unroll
  for (int nd = 0; nd < NDT; ++nd)
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (4 * j + r < GPAD) s_acc[((wave * GPAD) + 4 * j + r) * D + nd * 16 + n] = acc[nd][r];
  __syncthreads();

  const bool single = p.n_splits == 1;
  float* pa_out = p.part_acc + (((int64_t)row * p.n_splits + split) * p.G + g0) * D;
  float2* pml = p.part_ml + ((int64_t)row * p.n_splits + split) * p.G + g0;
  for (int it = tid; it < gb * D; it += kThreads) {
    const int g = it / D, jj = it % D;
    float M = s_ml[0][g].x;
#pragma unroll
    for (int w = 1; w < NW; ++w) M = fmaxf(M, s_ml[w][g].x);
    float a = 0.f, ls = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float2 ml = s_ml[w][g];
      const float f = (ml.x == -INFINITY) ? 0.f : exp_fast(ml.x - M);
      a += s_acc[((w * GPAD) + g) * D + jj] * f;
      ls += ml.y * f;
    }
    if (single) {
      p.out[((int64_t)prob * p.Hq + c * p.G + g0 + g) * D + jj] = a / ls;
    } else {
      pa_out[(int64_t)g * D + jj] = a;
      if (jj == 0) pml[g] = make_float2(M, ls);
    }
  }
  finish_row(p, sg);
}

// Merge launch: the slices of a row -> out (see merge_slices).
__global__ __launch_bounds__(128) void combine_kernel(DecodeParams p) {
  const int row = blockIdx.x, g = blockIdx.y, j = threadIdx.x;  // one thread per output element
  const int prob = row / p.Hkv, c = row % p.Hkv;
  // every slice kernel of the step has finished: the device-side count of appended tokens moves on
  if (p.ring && p.ring_advance && row == 0 && g == 0 && j == 0) p.ring[0] = p.ring[0] + 1;
  if (j >= p.D) return;
  p.out[((int64_t)prob * p.Hq + c * p.G + g) * p.D + j] = merge_slices(p, row, g, j);
}

template <int LPT>
__global__ __launch_bounds__(64) void append_kernel(DecodeParams p, int row_bytes) {
  const int row = blockIdx.x, tid = threadIdx.x;
  if (tid >= LPT) return;
  const int prob = row / p.Hkv, c = row % p.Hkv, eb = row_bytes / p.D;
  const CacheRow Kr = cache_row(p.Kc, p.cpm, false, prob, c, row, p.cap, row_bytes, eb);
  const CacheRow Vr = cache_row(p.Vc, p.cpm, true, prob, c, row, p.cap, row_bytes, eb);
  st16(Kr.at(p.slot) + tid * 16, ld16((const char*)p.k_new + (int64_t)row * row_bytes + tid * 16));
  st16(Vr.at(p.slot) + tid * 16, ld16((const char*)p.v_new + (int64_t)row * row_bytes + tid * 16));
}

__global__ __launch_bounds__(256) void fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = v;
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

template <int D, bool STREAM, bool PG>
hipError_t launch_decode_mfma_s(const DecodeParams& p, int g0, int gb, dim3 grid, hipStream_t s) {
  // One workgroup per row (many rows): 8 waves, one workgroup per CU; a row split over several
  // workgroups: 4 waves.  (For 256 < rows <= 512, 4-wave workgroups that are all resident at once
  // were measured no faster than two rounds of 8-wave ones.)
  // Up to 4 heads with whole rows, P.V on the vector ALU is a little faster (measured 86 vs 89 us
  // per step at 256 rows x 4096 tokens); with more heads, or short slices, P.V on the matrix cores
  // wins clearly (448 rows x 1024 tokens x 7 heads: 47 vs 68 us).
  const bool big = p.n_splits == 1;
  // more rows than CUs: 4-wave workgroups, two resident per CU, beat two rounds of 8-wave ones
  // (measured 43 vs 47 us at 448 rows x 1024 tokens x 7 heads)
  const bool wide = big && grid.y <= 256;
  if (gb <= 4) {
    if (big) hipLaunchKernelGGL((decode_mfma_kernel<D, 4, 8, STREAM, PG>), grid, dim3(512), 0, s, p, g0, gb);
    else hipLaunchKernelGGL((decode_pv_mfma_kernel<D, 4, 4, STREAM, PG>), grid, dim3(256), 0, s, p, g0, gb);
  } else if (gb <= 8) {
    if (wide) hipLaunchKernelGGL((decode_pv_mfma_kernel<D, 8, 8, STREAM, PG>), grid, dim3(512), 0, s, p, g0, gb);
    else hipLaunchKernelGGL((decode_pv_mfma_kernel<D, 8, 4, STREAM, PG>), grid, dim3(256), 0, s, p, g0, gb);
  } else {
    if (wide) hipLaunchKernelGGL((decode_pv_mfma_kernel<D, 16, 8, STREAM, PG>), grid, dim3(512), 0, s, p, g0, gb);
    else hipLaunchKernelGGL((decode_pv_mfma_kernel<D, 16, 4, STREAM, PG>), grid, dim3(256), 0, s, p, g0, gb);
  }
  return hipGetLastError();
}

template <int D>
hipError_t launch_decode_mfma(const DecodeParams& p, int g0, int gb, dim3 grid, hipStream_t s) {
  if (p.cpm.table)
    return p.stream_loads ? launch_decode_mfma_s<D, true, true>(p, g0, gb, grid, s)
                          : launch_decode_mfma_s<D, false, true>(p, g0, gb, grid, s);
  return p.stream_loads ? launch_decode_mfma_s<D, true, false>(p, g0, gb, grid, s)
                        : launch_decode_mfma_s<D, false, false>(p, g0, gb, grid, s);
}

}  // namespace

hipError_t launch_decode(const DecodeParams& p, hipStream_t s) {
  const int rows = p.n_problems * p.Hkv;
  dim3 grid((unsigned)p.n_splits, (unsigned)rows);
  const int per_launch = p.dtype == DT_BF16 ? 16 : max_group_per_launch();  // heads one launch handles
  for (int g0 = 0; g0 < p.G; g0 += per_launch) {
    const int gb = p.G - g0 < per_launch ? p.G - g0 : per_launch;
    DecodeParams q = p;
    if (g0 > 0) q.k_new = nullptr;  // the first launch already stored the new token
    if (g0 + per_launch < p.G) q.ring_advance = 0;  // the last launch of the step moves the ring on
    hipError_t e;
    if (p.dtype == DT_BF16)
      e = p.D == 128 ? launch_decode_mfma<128>(q, g0, gb, grid, s) : launch_decode_mfma<64>(q, g0, gb, grid, s);
    else
      e = p.D == 128 ? launch_decode_g<DT_F32, 128>(q, g0, gb, grid, s) : launch_decode_g<DT_F32, 64>(q, g0, gb, grid, s);
    if (e != hipSuccess) return e;
  }
  if (p.n_splits > 1) {
    hipLaunchKernelGGL(combine_kernel, dim3((unsigned)rows, (unsigned)p.G), dim3(128), 0, s, p);
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

// A fill kernel instead of a memset: the calls may be recorded into a HIP graph.
hipError_t launch_fill_u32(void* ptr, size_t n, uint32_t value, hipStream_t s) {
  if (n == 0) return hipSuccess;
  size_t want = (n + 255) / 256;
  unsigned grid = (unsigned)(want < 4096 ? want : 4096);
  hipLaunchKernelGGL(fill_u32_kernel, dim3(grid), dim3(256), 0, s, (uint32_t*)ptr, n, value);
  return hipGetLastError();
}

}  // namespace sagekv
