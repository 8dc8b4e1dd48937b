// Eviction pass, selection stage (paper Sec. 2 Step 2 "top-k", Step 3 "Concat"):
// per row, the k candidates with the largest score, ties to the lower index, written in
// ascending position between the sink and the recent window; then the gather of K and V.
//
// topk_kernel: one 1024-thread workgroup per row; two passes over the row's scores (steps 1 and
// 2) on the usual route, all with aligned 16-byte loads.
//   1. coarse bracket of the k-th score: the first two digits (11 + 11 bits) of a radix select on
//      the fp32 bit patterns of the scores (all positive, so the unsigned order is the float
//      order).  The first digit's histogram was built by many workgroups in the combine stage; the
//      second is an LDS histogram over the row.  The k-th score is then known to 2^-13 relative.
//   2. one scan counts the scores above a relative band around that bracket and lists the band's
//      members; those are re-evaluated in fp64 (dot products, exp, fp64-combined normalisers),
//      patched into the score row and ranked exactly among themselves (score descending, index
//      ascending), so the decision near the threshold does not depend on fp32 summation order.
//      The exact threshold is the (k - #above)-th of them.
//   3. only if the band holds more than kDenseBand members (a row of near-ties) or the refined
//      threshold sits on the band's edge: patch the band, exact radix select of the whole row.
//   4. ordered output.  Usual route: the band scan has marked every score above the band in an LDS
//      bitmap (one bit per candidate, rows of up to 512K candidates), the selected band members
//      are added, and a prefix sum over the bitmap's population counts gives the positions: the
//      row is read twice in all.  General route or longer rows: every wave counts and then writes
//      a contiguous part of the row.  Both keep the output ascending and give ties to the lowest
//      indices.
#include "device_utils.h"
#include "kernels.h"
#include "radix_select.h"

namespace sagekv {

namespace {

constexpr int kDenseBand = 1024;  // band members whose exact ranking is done among themselves

// A row of fp32 scores read with aligned 16-byte loads.  "Quad" q holds row elements 4q - head ..
// 4q - head + 3; quads q_lo .. q_hi-1 lie fully inside the row and are read with one vector load
// each, several in flight per thread.  The at most six elements before and after them are the
// row's edge elements: first edge = elements 0 .. n_first-1, last edge = elements last0 .. E-1.
// One workgroup (one CU) owns a row, so the passes below are bound by instruction issue as much
// as by the CU's load path: per element they spend two to four vector instructions, counts go
// through wave ballots into scalar registers.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) u32x4* GlobalQuads;  // global memory: 16-byte vector loads

struct QuadRow {
  const float* cand;
  GlobalQuads quads;  // quads[q] for q_lo <= q < q_hi
  int head;           // floats between the 16-byte boundary below cand and cand
  int q_lo, q_hi;
  int n_first, last0, E;
};

__device__ inline QuadRow quad_row(const float* cand, int E) {
  QuadRow r;
  r.cand = cand;
  r.head = (int)((reinterpret_cast<uintptr_t>(cand) >> 2) & 3);
  r.quads = (GlobalQuads)(cand - r.head);
  r.q_lo = r.head ? 1 : 0;
  r.q_hi = (r.head + E) >> 2;
  if (r.q_hi < r.q_lo) r.q_hi = r.q_lo;
  r.n_first = 4 * r.q_lo - r.head < E ? 4 * r.q_lo - r.head : E;
  r.last0 = 4 * r.q_hi - r.head > r.n_first ? 4 * r.q_hi - r.head : r.n_first;
  r.E = E;
  return r;
}

// Row index of the edge element that thread `t` (0..7) looks after, or -1: threads 0..3 the first
// edge, 4..7 the last one.
__device__ inline int edge_index(const QuadRow& r, int t) {
  if (t < 4) return t < r.n_first ? t : -1;
  return r.last0 + (t - 4) < r.E ? r.last0 + (t - 4) : -1;
}

constexpr int kQuadUnroll = 8;  // quads in flight per thread: 32 scores

// LDS histogram of digit (key >> shift) & (2^nbits - 1) over the keys that match `prefix` under `mask`.
__device__ inline void hist_pass_quads(TopkShared& sh, const QuadRow& r, uint32_t prefix, uint32_t mask, int shift,
                                       int nbits) {
  for (int b = threadIdx.x; b < kHistBins; b += kTopkThreads) sh.hist[b] = 0;
  __syncthreads();
  const uint32_t dm = (1u << nbits) - 1u;
  const int ei = threadIdx.x < 8 ? edge_index(r, threadIdx.x) : -1;
  uint32_t ekey = ~prefix;
  if (ei >= 0) ekey = __float_as_uint(r.cand[ei]);
  for (int q0 = r.q_lo + threadIdx.x; q0 < r.q_hi; q0 += kQuadUnroll * kTopkThreads) {
    u32x4 v[kQuadUnroll];
#pragma unroll
    for (int u = 0; u < kQuadUnroll; ++u) {
      const int q = q0 + u * kTopkThreads;
      v[u] = r.quads[q < r.q_hi ? q : r.q_hi - 1];
    }
#pragma unroll
    for (int u = 0; u < kQuadUnroll; ++u) {
      const bool valid = q0 + u * kTopkThreads < r.q_hi;
      const uint32_t key[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (valid && (key[e] & mask) == prefix) atomicAdd(&sh.hist[(key[e] >> shift) & dm], 1);
    }
  }
  if (ei >= 0 && (ekey & mask) == prefix) atomicAdd(&sh.hist[(ekey >> shift) & dm], 1);
  __syncthreads();
}

__device__ inline int lanes_below(unsigned long long ballot) {  // set bits of `ballot` in lanes below this one
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(ballot >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)ballot, 0u));
}

template <int DT>
__global__ __launch_bounds__(kTopkThreads) void topk_kernel(TopkParams p) {
  __shared__ TopkShared sh;
  extern __shared__ __align__(16) uint32_t bitmap[];  // bit i + head: candidate i is selected (head: see QuadRow)
  const int tid = threadIdx.x;
  const int list = blockIdx.x;  // selection list: one per row (group-sum) or one per (row, query head)
  const int row = list / p.n_lists, gl = list % p.n_lists;
  if (p.gate.row_flag && (*p.gate.n_flagged == 0 || p.gate.row_flag[row] == 0)) return;  // gated launch: only the flagged rows
  const int g_lo = p.n_lists > 1 ? gl : 0, g_hi = p.n_lists > 1 ? gl + 1 : p.geo.G;
  const int prob = row / p.geo.Hkv, c = row % p.geo.Hkv;
  const int S = p.S, W = p.W, k = p.k;
  const int64_t L = p.geo.L;
  const int E = (int)(L - S - W);
  const int n_kept = S + p.n_lists * k + W;
  int32_t* kept_row = p.kept_idx + (int64_t)row * n_kept;
  int32_t* kept = kept_row + gl * k;  // this list's k slots start at kept[S]
  float* cand = p.scores + (int64_t)list * p.pitch + S;
  const RowStat* row_stats = p.stats + (int64_t)row * p.geo.G;

  if (gl == 0) {
    for (int t = tid; t < S; t += kTopkThreads) kept_row[t] = t;
    for (int t = tid; t < W; t += kTopkThreads) kept_row[S + p.n_lists * k + t] = (int32_t)(L - W + t);
  }
  if (k == 0) return;
  const QuadRow qr = quad_row(cand, E);
  const int edge_i = tid < 8 ? edge_index(qr, tid) : -1;  // this thread's edge element, if any

  // 1. bracket of the k-th fp32 score: its first 22 bits
  for (int b = tid; b < kHistBins; b += kTopkThreads) sh.hist[b] = p.ghist[(int64_t)list * kHistBins + b];
  __syncthreads();
  uint32_t tau;
  int quota;
  {
    int bin, rem;
    pick_digit(sh, 1 << 11, k, &bin, &rem);
    tau = (uint32_t)bin << 20;
    hist_pass_quads(sh, qr, tau, 0xFFF00000u, 9, 11);
    pick_digit(sh, 1 << 11, rem, &bin, &rem);
    tau |= (uint32_t)bin << 9;
    quota = rem;
  }

  // 2. the band around it.  Scores above the band are selected whatever their exact value; the
  //    members of the band are re-evaluated in fp64 (and patched into the score row).  With a band
  //    of at most kDenseBand members the exact threshold is found among them alone: it is the
  //    (k - #above)-th largest refined value, provided it still lies strictly inside the band
  //    (then no score outside the band can compare differently).  Anything else (a huge band of
  //    near-ties, a refined value on the band's edge) takes the general route: patch, then a full
  //    radix select of the patched row.
  // (below 2^-126 the scores sit on the 2^-149 grid: the band is at least kDenormSlack wide each way)
  const float lo = __uint_as_float(tau) * (1.0f - p.band) - kDenormSlack,
              hi = __uint_as_float(tau | 0x1FFu) * (1.0f + p.band) + kDenormSlack;
  __shared__ int band_i[kDenseBand];
  __shared__ float band_v[kDenseBand];
  __shared__ int n_band, n_above, short_ok;
  __shared__ uint32_t short_tau;
  __shared__ int short_quota;
  const int n_words = (qr.head + E + 31) >> 5;
  const bool use_bitmap = n_words * 4 <= p.bitmap_bytes;
  if (tid == 0) n_band = n_above = short_ok = 0;
  if (use_bitmap)
    for (int w = tid; w < n_words; w += kTopkThreads) bitmap[w] = 0u;
  __syncthreads();
  {
    auto member = [&](int i) {
      const int t = atomicAdd(&n_band, 1);
      if (t < kDenseBand) band_i[t] = i;
    };
    float ev = -1.f;
    if (edge_i >= 0) ev = cand[edge_i];
    int above = 0;  // wave-uniform: counted through ballots
    for (int q0 = qr.q_lo + (tid & ~63); q0 < qr.q_hi; q0 += kQuadUnroll * kTopkThreads) {  // wave-uniform trip count
      u32x4 v[kQuadUnroll];
#pragma unroll
      for (int u = 0; u < kQuadUnroll; ++u) {
        const int q = q0 + (tid & 63) + u * kTopkThreads;
        v[u] = qr.quads[q < qr.q_hi ? q : qr.q_hi - 1];
      }
#pragma unroll
      for (int u = 0; u < kQuadUnroll; ++u) {
        const int q = q0 + (tid & 63) + u * kTopkThreads;
        const bool valid = q < qr.q_hi;
        const float x[4] = {__uint_as_float(v[u].x), __uint_as_float(v[u].y), __uint_as_float(v[u].z),
                            __uint_as_float(v[u].w)};
        uint32_t nib = 0u;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const bool gt = valid && x[e] > hi;
          above += __popcll(__ballot(gt));
          nib |= gt ? 1u << e : 0u;
          if (valid && !gt && x[e] >= lo) member(4 * q - qr.head + e);
        }
        if (use_bitmap && nib) atomicOr(&bitmap[q >> 3], nib << (4 * (q & 7)));
      }
    }
    if ((tid & 63) == 0 && above) atomicAdd(&n_above, above);
    if (edge_i >= 0) {
      if (ev > hi) {
        atomicAdd(&n_above, 1);
        if (use_bitmap) atomicOr(&bitmap[(edge_i + qr.head) >> 5], 1u << ((edge_i + qr.head) & 31));
      } else if (ev >= lo) {
        member(edge_i);
      }
    }
  }
  __syncthreads();
  const int nb = n_band, r = k - n_above;
  bool general = nb > kDenseBand || r < 1 || r > nb;
  if (!general) {
    if (nb <= 4 * kTopkWaves) {  // the usual handful: one wave per member
      for (int t = tid >> 6; t < nb; t += kTopkWaves) {
        const int i = band_i[t];
        const float v = refined_score_wave<DT>(p.geo, p.q_last, p.K, p.pm, p.ks_problem, p.ks_head, p.ks_token, row_stats,
                                               prob, c, S + i, g_lo, g_hi);
        if ((tid & 63) == 0) {
          band_v[t] = v;
          cand[i] = v;
        }
      }
    } else {
      for (int t = tid; t < nb; t += kTopkThreads) {
        const int i = band_i[t];
        const float v = refined_score<DT>(p.geo, p.q_last, p.K, p.pm, p.ks_problem, p.ks_head, p.ks_token, row_stats, prob, c,
                                          S + i, g_lo, g_hi);
        band_v[t] = v;
        cand[i] = v;
      }
    }
    __syncthreads();
    for (int t = tid; t < nb; t += kTopkThreads) {
      const float v = band_v[t];
      const int i = band_i[t];
      int rank = 0, greater = 0;
      for (int u = 0; u < nb; ++u) {
        greater += band_v[u] > v;
        rank += band_v[u] > v || (band_v[u] == v && band_i[u] < i);
      }
      if (rank == r - 1 && v > lo && v < hi) {  // the threshold element, strictly inside the band
        short_tau = __float_as_uint(v);
        short_quota = r - greater;
        short_ok = 1;
      }
      if (use_bitmap && rank < r) atomicOr(&bitmap[(i + qr.head) >> 5], 1u << ((i + qr.head) & 31));
    }
    __syncthreads();
    general = !short_ok;
    if (!general) {
      if (use_bitmap) {  // 4., usual route
        bitmap_compact(bitmap, n_words, S - qr.head, kept + S, k, sh.wave_tot);
        return;
      }
      tau = short_tau;
      quota = short_quota;
    }
  } else {
    for (int i0 = tid; i0 < E; i0 += 4 * kTopkThreads) {
      float v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + u * kTopkThreads;
        v[u] = i < E ? cand[i] : -1.f;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + u * kTopkThreads;
        if (v[u] >= lo && v[u] <= hi)
          cand[i] = refined_score<DT>(p.geo, p.q_last, p.K, p.pm, p.ks_problem, p.ks_head, p.ks_token, row_stats, prob, c,
                                          S + i, g_lo, g_hi);
      }
    }
  }
  __syncthreads();

  // 3. general route: exact threshold by a radix select over the patched scores
  if (general) radix_select(sh, cand, E, k, false, &tau, &quota);

  // 4., general route or a row too long for the bitmap.  Every wave owns a contiguous sixteenth of the row's quads (wave 0 also
  //    the first edge, the last wave the last edge): it first counts its keys above and equal to
  //    the threshold, the sixteen counts give every wave its first output slot, then it reads its
  //    part again (cache-hot) and writes the selected positions in order; ties go to the lowest
  //    indices.  No workgroup barrier inside either loop.  Keys are compared as signed integers
  //    (scores are non-negative floats), so -1 stands for "no element".
  __shared__ int wave_gt[kTopkWaves], wave_eq[kTopkWaves];
  const int lane = tid & 63, wave = tid >> 6;
  const int itau = (int)tau;
  const int seg = ((qr.q_hi - qr.q_lo + kTopkWaves - 1) / kTopkWaves + 63) / 64 * 64;  // quads per wave
  const int seg_lo = qr.q_lo + wave * seg;
  const int seg_hi = seg_lo + seg < qr.q_hi ? seg_lo + seg : qr.q_hi;
  // edge elements as one more round of the first / the last wave: lanes 0..3 hold one element each
  int edge_key = -1, edge_at = 0;
  if (wave == 0 || wave == kTopkWaves - 1) {
    const int ei = lane < 4 ? edge_index(qr, (wave == 0 ? 0 : 4) + lane) : -1;
    if (ei >= 0) {
      edge_key = (int)__float_as_uint(cand[ei]);
      edge_at = ei;
    }
  }
  {
    int n_gt = 0, n_eq = 0;  // wave-uniform
    for (int q0 = seg_lo; q0 < seg_hi; q0 += kQuadUnroll * 64) {
      u32x4 v[kQuadUnroll];
#pragma unroll
      for (int u = 0; u < kQuadUnroll; ++u) {
        const int q = q0 + lane + u * 64;
        v[u] = qr.quads[q < seg_hi ? q : seg_hi - 1];
      }
#pragma unroll
      for (int u = 0; u < kQuadUnroll; ++u) {
        const bool valid = q0 + lane + u * 64 < seg_hi;
        const int key[4] = {(int)v[u].x, (int)v[u].y, (int)v[u].z, (int)v[u].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          n_gt += __popcll(__ballot(valid && key[e] > itau));
          n_eq += __popcll(__ballot(valid && key[e] == itau));
        }
      }
    }
    n_gt += __popcll(__ballot(edge_key > itau));
    n_eq += __popcll(__ballot(edge_key == itau));
    if (lane == 0) {
      wave_gt[wave] = n_gt;
      wave_eq[wave] = n_eq;
    }
  }
  __syncthreads();
  int run_sel = 0, run_eq = 0;  // selected / equal keys before this wave's part (wave-uniform)
  for (int w = 0; w < wave; ++w) {
    run_sel += wave_gt[w];
    run_eq += wave_eq[w];
  }
  run_sel += run_eq < quota ? run_eq : quota;
  // one round: every lane holds four keys (key[e] = -1: none) of row elements at0 .. at0+3
  auto round = [&](const int (&key)[4], int at0) {
    bool sel[4];
    unsigned long long any_eq = 0ull;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      sel[e] = key[e] > itau;
      any_eq |= __ballot(key[e] == itau);
    }
    if (any_eq) {  // rare: equal keys are selected while the quota lasts, lowest indices first
      int mine = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) mine += key[e] == itau;
      int incl = mine;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int y = __shfl_up(incl, o);
        if (lane >= o) incl += y;
      }
      int before = run_eq + incl - mine;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (key[e] == itau) {
          sel[e] = before < quota;
          ++before;
        }
      run_eq += __shfl(incl, 63);
    }
    int pos = run_sel, total = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const unsigned long long b = __ballot(sel[e]);
      pos += lanes_below(b);
      total += __popcll(b);
    }
    if (sel[0] | sel[1] | sel[2] | sel[3]) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (sel[e]) {
          if (pos < k) kept[S + pos] = (int32_t)(S + at0 + e);
          ++pos;
        }
    }
    run_sel += total;
  };
  if (wave == 0) {
    const int key[4] = {edge_key, -1, -1, -1};
    round(key, edge_at);
  }
  for (int q0 = seg_lo; q0 < seg_hi; q0 += kQuadUnroll * 64) {
    u32x4 v[kQuadUnroll];
#pragma unroll
    for (int u = 0; u < kQuadUnroll; ++u) {
      const int q = q0 + lane + u * 64;
      v[u] = qr.quads[q < seg_hi ? q : seg_hi - 1];
    }
#pragma unroll
    for (int u = 0; u < kQuadUnroll; ++u) {
      const int q = q0 + lane + u * 64;
      const bool valid = q < seg_hi;
      const int key[4] = {valid ? (int)v[u].x : -1, valid ? (int)v[u].y : -1, valid ? (int)v[u].z : -1,
                          valid ? (int)v[u].w : -1};
      round(key, 4 * q - qr.head);
    }
  }
  if (wave == kTopkWaves - 1) {
    const int key[4] = {edge_key, -1, -1, -1};
    round(key, edge_at);
  }
}

// ---- gather -----------------------------------------------------------------------------------
constexpr int kGatherThreads = 256;
constexpr int kGatherTokens = 64;  // reduced-cache rows one workgroup copies

template <int LPT>
__global__ __launch_bounds__(kGatherThreads) void gather_kernel(GatherParams p, int eb) {
  const int row = blockIdx.y;
  const int prob = row / p.geo.Hkv, c = row % p.geo.Hkv;
  const int sub = threadIdx.x / LPT, cl = threadIdx.x % LPT;
  constexpr int TPI = kGatherThreads / LPT;  // tokens per iteration
  const int64_t row_bytes = (int64_t)p.geo.D * eb;
  const CacheRow Kc = cache_row(p.Kc, p.cpm, false, prob, c, row, p.cap, (int)row_bytes, eb);
  const CacheRow Vc = cache_row(p.Vc, p.cpm, true, prob, c, row, p.cap, (int)row_bytes, eb);
  const int32_t* kept = p.kept_idx + (int64_t)row * p.n_kept;
  const int t0 = blockIdx.x * kGatherTokens;
  constexpr int NIT = kGatherTokens / TPI;
  // all of a thread's loads are issued before its first store: positions first, then the rows
  // (streaming loads: the full cache is not read again)
  int64_t src[NIT];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int t = t0 + it * TPI + sub;
    src[it] = kept[t < p.n_kept ? t : p.n_kept - 1];
  }
  uint4 a[NIT], b[NIT];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int64_t i = src[it] < 0 ? 0 : (src[it] >= p.geo.L ? p.geo.L - 1 : src[it]);  // never read outside the row
    const int64_t ko = kv_offset(p.pm, p.pm.ks_page, p.ks_problem, p.ks_head, p.ks_token, prob, c, i);
    const int64_t vo = kv_offset(p.pm, p.pm.vs_page, p.vs_problem, p.vs_head, p.vs_token, prob, c, i);
    a[it] = ld16_stream((const char*)p.K + ko * eb + cl * 16);
    b[it] = ld16_stream((const char*)p.V + vo * eb + cl * 16);
  }
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int t = t0 + it * TPI + sub;
    if (t < p.n_kept) {
      st16(Kc.at(t) + cl * 16, a[it]);
      st16(Vc.at(t) + cl * 16, b[it]);
    }
  }
}

}  // namespace

hipError_t launch_topk(const TopkParams& p0, hipStream_t s) {
  constexpr int kMaxBitmap = 64 * 1024;
  static uint64_t done_bf16 = 0, done_f32 = 0;
  hipError_t e = p0.geo.dtype == DT_BF16 ? allow_dynamic_lds((const void*)topk_kernel<DT_BF16>, kMaxBitmap, &done_bf16)
                                         : allow_dynamic_lds((const void*)topk_kernel<DT_F32>, kMaxBitmap, &done_f32);
  if (e != hipSuccess) return e;
  TopkParams p = p0;
  const int64_t E = p.geo.L - p.S - p.W;
  const int64_t need = ((E + 3 + 31) / 32 + 3) / 4 * 16;  // one bit per candidate, whatever the row's alignment
  p.bitmap_bytes = need <= kMaxBitmap ? (int)need : 0;
  const int lists = p.geo.n_problems * p.geo.Hkv * p.n_lists;
  if (p.geo.dtype == DT_BF16)
    hipLaunchKernelGGL(topk_kernel<DT_BF16>, dim3((unsigned)lists), dim3(kTopkThreads), p.bitmap_bytes, s, p);
  else
    hipLaunchKernelGGL(topk_kernel<DT_F32>, dim3((unsigned)lists), dim3(kTopkThreads), p.bitmap_bytes, s, p);
  return hipGetLastError();
}

hipError_t launch_gather(const GatherParams& p, hipStream_t s) {
  const int rows = p.geo.n_problems * p.geo.Hkv;
  const int eb = p.geo.dtype == DT_BF16 ? 2 : 4;
  const int lpt = p.geo.D * eb / 16;
  dim3 grid((unsigned)((p.n_kept + kGatherTokens - 1) / kGatherTokens), (unsigned)rows);
  switch (lpt) {
    case 8: hipLaunchKernelGGL(gather_kernel<8>, grid, dim3(kGatherThreads), 0, s, p, eb); break;
    case 16: hipLaunchKernelGGL(gather_kernel<16>, grid, dim3(kGatherThreads), 0, s, p, eb); break;
    case 32: hipLaunchKernelGGL(gather_kernel<32>, grid, dim3(kGatherThreads), 0, s, p, eb); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace sagekv
