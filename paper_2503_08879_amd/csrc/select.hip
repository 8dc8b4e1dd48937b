// Eviction pass, selection stage (paper Sec. 2 Step 2 "top-k", Step 3 "Concat"):
// per row, the k candidates with the largest score, ties to the lower index, written in
// ascending position between the sink and the recent window; then the gather of K and V.
//
// topk_kernel: one 1024-thread workgroup per row.
//   1. coarse threshold: 3-digit radix select (11/11/9 bits) on the fp32 bit patterns of the
//      scores (all positive, so the unsigned order is the float order).  The first digit's
//      histogram was built by many workgroups in the combine stage; the other two are LDS
//      histograms over the row.
//   2. one scan counts the scores above a relative band around the coarse k-th score and lists the
//      band's members; those are re-evaluated in fp64 (dot products, exp, fp64-combined
//      normalisers), patched into the score row and ranked exactly among themselves (score
//      descending, index ascending), so the decision near the threshold does not depend on fp32
//      summation order.  The exact threshold is the (k - #above)-th of them.
//   3. only if the band holds more than kDenseBand members (a row of near-ties) or the refined
//      threshold sits on the band's edge: patch the band, exact radix select of the whole row.
//   4. ordered compaction: block scans keep the output ascending and give ties to the lowest
//      indices.
#include "device_utils.h"
#include "kernels.h"
#include "radix_select.h"

namespace sagekv {

namespace {

constexpr int kDenseBand = 1024;  // band members whose exact ranking is done among themselves

template <int DT>
__global__ __launch_bounds__(kTopkThreads) void topk_kernel(TopkParams p) {
  __shared__ TopkShared sh;
  const int tid = threadIdx.x;
  int list = blockIdx.x;  // selection list: one per row (group-sum) or one per (row, query head)
  if (p.gate.row_map) {
    if ((int)blockIdx.x / p.n_lists >= *p.gate.n_active) return;
    list = p.gate.row_map[blockIdx.x / p.n_lists] * p.n_lists + blockIdx.x % p.n_lists;
  }
  const int row = list / p.n_lists, gl = list % p.n_lists;
  const int g_lo = p.n_lists > 1 ? gl : 0, g_hi = p.n_lists > 1 ? gl + 1 : p.geo.G;
  const int prob = row / p.geo.Hkv, c = row % p.geo.Hkv;
  const int S = p.S, W = p.W, k = p.k;
  const int64_t L = p.geo.L, E = L - S - W;
  const int n_kept = S + p.n_lists * k + W;
  int32_t* kept_row = p.kept_idx + (int64_t)row * n_kept;
  int32_t* kept = kept_row + gl * k;  // this list's k slots start at kept[S]
  float* cand = p.scores + (int64_t)list * p.pitch + S;

  if (gl == 0) {
    for (int t = tid; t < S; t += kTopkThreads) kept_row[t] = t;
    for (int t = tid; t < W; t += kTopkThreads) kept_row[S + p.n_lists * k + t] = (int32_t)(L - W + t);
  }
  if (k == 0) return;

  // 1. coarse threshold from the fp32 scores
  for (int b = tid; b < kHistBins; b += kTopkThreads) sh.hist[b] = p.ghist[(int64_t)list * kHistBins + b];
  __syncthreads();
  uint32_t tau;
  int quota;
  radix_select(sh, cand, E, k, true, &tau, &quota);

  // 2. the band around it.  Scores above the band are selected whatever their exact value; the
  //    members of the band are re-evaluated in fp64 (and patched into the score row).  With a band
  //    of at most kDenseBand members the exact threshold is found among them alone: it is the
  //    (k - #above)-th largest refined value, provided it still lies strictly inside the band
  //    (then no score outside the band can compare differently).  Anything else (a huge band of
  //    near-ties, a refined value on the band's edge) takes the general route: patch, then a full
  //    radix select of the patched row.
  const float tf = __uint_as_float(tau);
  const float lo = tf * (1.0f - p.band), hi = tf * (1.0f + p.band);
  __shared__ int band_i[kDenseBand];
  __shared__ float band_v[kDenseBand];
  __shared__ int n_band, n_above, short_ok;
  __shared__ uint32_t short_tau;
  __shared__ int short_quota;
  if (tid == 0) n_band = n_above = short_ok = 0;
  __syncthreads();
  for (int64_t i0 = tid; i0 < E; i0 += 4 * kTopkThreads) {  // four independent loads in flight
    float v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t i = i0 + (int64_t)u * kTopkThreads;
      v[u] = i < E ? cand[i] : -1.f;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t i = i0 + (int64_t)u * kTopkThreads;
      const bool above = v[u] > hi;
      const unsigned long long bal = __ballot(above);
      if ((tid & 63) == 0 && bal) atomicAdd(&n_above, __popcll(bal));
      if (v[u] >= lo && v[u] <= hi) {
        const int t = atomicAdd(&n_band, 1);
        if (t < kDenseBand) band_i[t] = (int)i;
      }
    }
  }
  __syncthreads();
  const int nb = n_band, r = k - n_above;
  bool general = nb > kDenseBand || r < 1 || r > nb;
  if (!general) {
    for (int t = tid; t < nb; t += kTopkThreads) {
      const int i = band_i[t];
      const float v = refined_score<DT>(p.geo, p.q_last, p.K, p.pm, p.ks_problem, p.ks_head, p.ks_token, p.stats, prob, c, row,
                                        S + i, g_lo, g_hi);
      band_v[t] = v;
      cand[i] = v;
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
    }
    __syncthreads();
    general = !short_ok;
    if (!general) {
      tau = short_tau;
      quota = short_quota;
    }
  } else {
    for (int64_t i0 = tid; i0 < E; i0 += 4 * kTopkThreads) {
      float v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int64_t i = i0 + (int64_t)u * kTopkThreads;
        v[u] = i < E ? cand[i] : -1.f;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int64_t i = i0 + (int64_t)u * kTopkThreads;
        if (v[u] >= lo && v[u] <= hi)
          cand[i] = refined_score<DT>(p.geo, p.q_last, p.K, p.pm, p.ks_problem, p.ks_head, p.ks_token, p.stats, prob, c, row,
                                      S + i, g_lo, g_hi);
      }
    }
  }
  __syncthreads();

  // 3. general route: exact threshold by a radix select over the patched scores
  if (general) radix_select(sh, cand, E, k, false, &tau, &quota);

  // 4. ordered compaction
  int run_gt = 0, run_eq = 0;
  for (int64_t base = 0; base < E; base += kTopkThreads * 4) {
    const int64_t i0 = base + (int64_t)tid * 4;
    uint32_t key[4];
    int n_gt = 0, n_eq = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      key[j] = (i0 + j < E) ? __float_as_uint(cand[i0 + j]) : 0u;
      n_gt += (i0 + j < E) && key[j] > tau;
      n_eq += (i0 + j < E) && key[j] == tau;
    }
    int tot;
    const int packed = n_gt | (n_eq << 16);
    const int incl = block_scan_incl<kTopkThreads>(packed, sh.wave_tot, &tot);
    int gt_before = run_gt + ((incl - packed) & 0xFFFF);
    int eq_before = run_eq + ((incl - packed) >> 16);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (i0 + j < E) {
        const bool gt = key[j] > tau, eq = key[j] == tau;
        if (gt || (eq && eq_before < quota)) {
          const int pos = gt_before + (eq_before < quota ? eq_before : quota);
          if (pos < k) kept[S + pos] = (int32_t)(S + i0 + j);
        }
        gt_before += gt;
        eq_before += eq;
      }
    }
    run_gt += tot & 0xFFFF;
    run_eq += tot >> 16;
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
  char* Kc = (char*)p.Kc + (int64_t)row * p.cap * row_bytes;
  char* Vc = (char*)p.Vc + (int64_t)row * p.cap * row_bytes;
  const int32_t* kept = p.kept_idx + (int64_t)row * p.n_kept;
  const int t0 = blockIdx.x * kGatherTokens;
#pragma unroll
  for (int it = 0; it < kGatherTokens / TPI; ++it) {
    const int t = t0 + it * TPI + sub;
    if (t < p.n_kept) {
      int64_t src = kept[t];
      src = src < 0 ? 0 : (src >= p.geo.L ? p.geo.L - 1 : src);  // never read outside the row
      const int64_t ko = kv_offset(p.pm, p.pm.ks_page, p.ks_problem, p.ks_head, p.ks_token, prob, c, src);
      const int64_t vo = kv_offset(p.pm, p.pm.vs_page, p.vs_problem, p.vs_head, p.vs_token, prob, c, src);
      const uint4 a = ld16((const char*)p.K + ko * eb + cl * 16);
      const uint4 b = ld16((const char*)p.V + vo * eb + cl * 16);
      st16(Kc + t * row_bytes + cl * 16, a);
      st16(Vc + t * row_bytes + cl * 16, b);
    }
  }
}

}  // namespace

hipError_t launch_topk(const TopkParams& p, hipStream_t s) {
  const int lists = p.geo.n_problems * p.geo.Hkv * p.n_lists;
  if (p.geo.dtype == DT_BF16)
    hipLaunchKernelGGL(topk_kernel<DT_BF16>, dim3((unsigned)lists), dim3(kTopkThreads), 0, s, p);
  else
    hipLaunchKernelGGL(topk_kernel<DT_F32>, dim3((unsigned)lists), dim3(kTopkThreads), 0, s, p);
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
