// Eviction pass, selection stage (paper Sec. 2 Step 2 "top-k", Step 3 "Concat"):
// per row, the k candidates with the largest score, ties to the lower index, written in
// ascending position between the sink and the recent window; then the gather of K and V.
//
// topk_kernel: one 1024-thread workgroup per row.
//   1. coarse threshold: 3-digit radix select (11/11/9 bits) on the fp32 bit patterns of the
//      scores (all positive, so the unsigned order is the float order).  The first digit's
//      histogram was built by many workgroups in the combine stage; the other two are LDS
//      histograms over the row.
//   2. every candidate whose fp32 score lies within a relative band of the coarse k-th score is
//      re-evaluated in fp64 (dot products, exp, fp64-combined normalisers) and its score is
//      overwritten with the rounded result, so the decision near the threshold does not depend
//      on fp32 summation order.
//   3. exact radix select again on the patched scores -> (threshold, number of ties to take).
//   4. ordered compaction: block scans keep the output ascending and give ties to the lowest
//      indices.
#include "device_utils.h"
#include "kernels.h"

namespace sagekv {

namespace {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / kWave;

struct TopkShared {
  int hist[kHistBins];
  int wave_tot[kTopkWaves];
  int pick_bin;
  int pick_rem;
};

// Largest digit b such that count(digits >= b) >= k_rem; returns b and the rank left inside it.
__device__ void pick_digit(TopkShared& sh, int nb, int k_rem, int* bin, int* rem) {
  const int t = threadIdx.x;
  if (t == 0) {
    sh.pick_bin = 0;
    sh.pick_rem = 1;
  }
  const int i0 = nb - 1 - 2 * t, i1 = nb - 2 - 2 * t;  // descending digits
  const int c0 = i0 >= 0 ? sh.hist[i0] : 0;
  const int c1 = i1 >= 0 ? sh.hist[i1] : 0;
  int tot;
  const int incl = block_scan_incl<kTopkThreads>(c0 + c1, sh.wave_tot, &tot);
  const int before = incl - c0 - c1;
  if (before < k_rem && k_rem <= before + c0) {
    sh.pick_bin = i0;
    sh.pick_rem = k_rem - before;
  } else if (before + c0 < k_rem && k_rem <= incl) {
    sh.pick_bin = i1;
    sh.pick_rem = k_rem - before - c0;
  }
  __syncthreads();
  *bin = sh.pick_bin;
  *rem = sh.pick_rem;
  __syncthreads();
}

__device__ void hist_pass(TopkShared& sh, const float* cand, int64_t E, uint32_t prefix, uint32_t mask, int shift,
                          int nbits) {
  for (int b = threadIdx.x; b < kHistBins; b += kTopkThreads) sh.hist[b] = 0;
  __syncthreads();
  const uint32_t dm = (1u << nbits) - 1u;
  for (int64_t i = threadIdx.x; i < E; i += kTopkThreads) {
    const uint32_t key = __float_as_uint(cand[i]);
    if ((key & mask) == prefix) atomicAdd(&sh.hist[(key >> shift) & dm], 1);
  }
  __syncthreads();
}

// k-th largest key among cand[0..E) and how many elements equal to it belong to the top k.
// first_hist_ready: sh.hist already holds the histogram of the first digit.
__device__ void radix_select(TopkShared& sh, const float* cand, int64_t E, int k, bool first_hist_ready,
                             uint32_t* tau, int* quota) {
  int bin, rem = k;
  if (!first_hist_ready) hist_pass(sh, cand, E, 0u, 0u, 20, 11);
  pick_digit(sh, 1 << 11, rem, &bin, &rem);
  uint32_t prefix = (uint32_t)bin << 20;
  hist_pass(sh, cand, E, prefix, 0xFFF00000u, 9, 11);
  pick_digit(sh, 1 << 11, rem, &bin, &rem);
  prefix |= (uint32_t)bin << 9;
  hist_pass(sh, cand, E, prefix, 0xFFFFFE00u, 0, 9);
  pick_digit(sh, 1 << 9, rem, &bin, &rem);
  *tau = prefix | (uint32_t)bin;
  *quota = rem;
}

template <int DT>
__device__ double elem_f64(const void* base, int64_t i);
template <>
__device__ double elem_f64<DT_BF16>(const void* base, int64_t i) {
  return (double)__uint_as_float((uint32_t)((const uint16_t*)base)[i] << 16);
}
template <>
__device__ double elem_f64<DT_F32>(const void* base, int64_t i) {
  return (double)((const float*)base)[i];
}

// Score of token `tok` of the row in fp64, rounded once to fp32.
template <int DT>
__device__ float refined_score(const TopkParams& p, int prob, int c, int row, int64_t tok) {
  const int D = p.geo.D, G = p.geo.G;
  const int64_t k_off = (int64_t)prob * p.ks_problem + (int64_t)c * p.ks_head + tok * p.ks_token;
  const double inv = 1.0 / sqrt((double)D);
  double tot = 0.0;
  for (int g = 0; g < G; ++g) {
    const int64_t q_off = ((int64_t)prob * p.geo.Hq + c * G + g) * D;
    double acc = 0.0;
    for (int j = 0; j < D; ++j) acc += elem_f64<DT>(p.q_last, q_off + j) * elem_f64<DT>(p.K, k_off + j);
    const RowStat st = p.stats[(int64_t)row * G + g];
    tot += exp(acc * inv - (double)st.M) / st.Z;
  }
  return (float)tot;
}

template <int DT>
__global__ __launch_bounds__(kTopkThreads) void topk_kernel(TopkParams p) {
  __shared__ TopkShared sh;
  const int row = blockIdx.x, tid = threadIdx.x;
  const int prob = row / p.geo.Hkv, c = row % p.geo.Hkv;
  const int S = p.S, W = p.W, k = p.k;
  const int64_t L = p.geo.L, E = L - S - W;
  const int n_kept = S + k + W;
  int32_t* kept = p.kept_idx + (int64_t)row * n_kept;
  float* cand = p.scores + (int64_t)row * p.pitch + S;

  for (int t = tid; t < S; t += kTopkThreads) kept[t] = t;
  for (int t = tid; t < W; t += kTopkThreads) kept[S + k + t] = (int32_t)(L - W + t);
  if (k == 0) return;

  // 1. coarse threshold from the fp32 scores
  for (int b = tid; b < kHistBins; b += kTopkThreads) sh.hist[b] = p.ghist[(int64_t)row * kHistBins + b];
  __syncthreads();
  uint32_t tau;
  int quota;
  radix_select(sh, cand, E, k, true, &tau, &quota);

  // 2. fp64 re-evaluation of the band around it
  const float tf = __uint_as_float(tau);
  const float lo = tf * (1.0f - p.band), hi = tf * (1.0f + p.band);
  for (int64_t i = tid; i < E; i += kTopkThreads) {
    const float v = cand[i];
    if (v >= lo && v <= hi) cand[i] = refined_score<DT>(p, prob, c, row, S + i);
  }
  __syncthreads();

  // 3. exact threshold on the patched scores
  radix_select(sh, cand, E, k, false, &tau, &quota);

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
  const char* Kr = (const char*)p.K + ((int64_t)prob * p.ks_problem + (int64_t)c * p.ks_head) * eb;
  const char* Vr = (const char*)p.V + ((int64_t)prob * p.vs_problem + (int64_t)c * p.vs_head) * eb;
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
      const uint4 a = ld16(Kr + src * p.ks_token * eb + cl * 16);
      const uint4 b = ld16(Vr + src * p.vs_token * eb + cl * 16);
      st16(Kc + t * row_bytes + cl * 16, a);
      st16(Vc + t * row_bytes + cl * 16, b);
    }
  }
}

}  // namespace

hipError_t launch_topk(const TopkParams& p, hipStream_t s) {
  const int rows = p.geo.n_problems * p.geo.Hkv;
  if (p.geo.dtype == DT_BF16)
    hipLaunchKernelGGL(topk_kernel<DT_BF16>, dim3((unsigned)rows), dim3(kTopkThreads), 0, s, p);
  else
    hipLaunchKernelGGL(topk_kernel<DT_F32>, dim3((unsigned)rows), dim3(kTopkThreads), 0, s, p);
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
