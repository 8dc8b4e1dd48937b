// Block-wide radix select on fp32 bit patterns (positive floats: unsigned order = float order)
// and the fp64 re-evaluation of a token's score.  Shared by the dense and the candidate-list
// selection kernels; all functions are called by every thread of a 1024-thread workgroup.
#pragma once
#include "device_utils.h"
#include "kernels.h"

namespace sagekv {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / kWave;

struct TopkShared {
  int hist[kHistBins];
  int wave_tot[kTopkWaves];
  int pick_bin;
  int pick_rem;
};

// Exact softmax statistics of one head of a row from its per-chunk partials (max, sum exp(x - max)):
// M = overall maximum of the fp32 logits, Z = sum_i exp(l_i - M) combined in fp64.  Called by all 64
// lanes of a wave; every lane gets the result.
__device__ inline RowStat merge_partials_wave(const float2* pr, int n_chunks) {
  const int lane = threadIdx.x & 63;
  float M = -INFINITY;
  for (int i = lane; i < n_chunks; i += 64) M = fmaxf(M, pr[i].x);
  M = wave_max(M);
  double z = 0.0;
  for (int i = lane; i < n_chunks; i += 64) {
    const float2 v = pr[i];
    z += (double)v.y * exp((double)v.x - (double)M);
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) z += __shfl_xor(z, o);
  RowStat st;
  st.M = M;
  st.Z = z;
  st.invZ = (float)(1.0 / z);
  return st;
}

// Largest digit b such that count(digits >= b) >= k_rem; returns b and the rank left inside it.
__device__ inline void pick_digit(TopkShared& sh, int nb, int k_rem, int* bin, int* rem) {
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

__device__ inline void hist_pass(TopkShared& sh, const float* cand, int64_t E, uint32_t prefix, uint32_t mask, int shift,
                          int nbits) {
  for (int b = threadIdx.x; b < kHistBins; b += kTopkThreads) sh.hist[b] = 0;
  __syncthreads();
  const uint32_t dm = (1u << nbits) - 1u;
  for (int64_t i0 = threadIdx.x; i0 < E; i0 += 4 * kTopkThreads) {  // four independent loads in flight
    uint32_t key[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t i = i0 + (int64_t)u * kTopkThreads;
      key[u] = i < E ? __float_as_uint(cand[i]) : ~prefix;  // a key that never matches the prefix
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t i = i0 + (int64_t)u * kTopkThreads;
      if (i < E && (key[u] & mask) == prefix) atomicAdd(&sh.hist[(key[u] >> shift) & dm], 1);
    }
  }
  __syncthreads();
}

// k-th largest key among cand[0..E) and how many elements equal to it belong to the top k.
// first_hist_ready: sh.hist already holds the histogram of the first digit.
__device__ inline void radix_select(TopkShared& sh, const float* cand, int64_t E, int k, bool first_hist_ready,
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

// Ordered output of a selection kept as a bitmap in LDS (16-byte aligned): writes first + (index of
// the j-th set bit) to out[j] for j < k.  Every thread takes four consecutive words per round.
__device__ inline void bitmap_compact(const uint32_t* bitmap, int n_words, int first, int32_t* out, int k,
                                      int* wave_tot) {
  int run = 0;
  for (int w0 = 0; w0 < n_words; w0 += 4 * kTopkThreads) {
    const int w = w0 + 4 * (int)threadIdx.x;
    uint32_t word[4] = {0u, 0u, 0u, 0u};
    if (w + 3 < n_words) {
      const uint4 v = *reinterpret_cast<const uint4*>(bitmap + w);
      word[0] = v.x, word[1] = v.y, word[2] = v.z, word[3] = v.w;
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (w + j < n_words) word[j] = bitmap[w + j];
    }
    const int cnt = __popc(word[0]) + __popc(word[1]) + __popc(word[2]) + __popc(word[3]);
    int tot;
    const int incl = block_scan_incl<kTopkThreads>(cnt, wave_tot, &tot);
    int pos = run + incl - cnt;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint32_t x = word[j];
      while (x) {
        const int b = __ffs(x) - 1;
        x &= x - 1;
        if (pos < k) out[pos] = (int32_t)(first + (w + j) * 32 + b);
        ++pos;
      }
    }
    run += tot;
  }
}

template <int DT>
__device__ inline double elem_f64(const void* base, int64_t i);
template <>
__device__ inline double elem_f64<DT_BF16>(const void* base, int64_t i) {
  return (double)__uint_as_float((uint32_t)((const uint16_t*)base)[i] << 16);
}
template <>
__device__ inline double elem_f64<DT_F32>(const void* base, int64_t i) {
  return (double)((const float*)base)[i];
}

// Score of token `tok` of the row in fp64 (heads g_lo .. g_hi-1 of the group), rounded once to fp32.
// row_stats: the exact (M, Z) of the row's G heads (global or LDS).
template <int DT>
__device__ inline float refined_score(const RowGeom& geo, const void* q_last, const void* K, const PageMap& pm,
                                   int64_t ks_problem, int64_t ks_head, int64_t ks_token, const RowStat* row_stats,
                                   int prob, int c, int64_t tok, int g_lo, int g_hi) {
  const int D = geo.D, G = geo.G;
  const int64_t k_off = kv_offset(pm, pm.ks_page, ks_problem, ks_head, ks_token, prob, c, tok);
  const double inv = 1.0 / sqrt((double)D);
  double tot = 0.0;
  for (int g = g_lo; g < g_hi; ++g) {
    const int64_t q_off = ((int64_t)prob * geo.Hq + c * G + g) * D;
    double acc = 0.0;
    for (int j = 0; j < D; ++j) acc += elem_f64<DT>(q_last, q_off + j) * elem_f64<DT>(K, k_off + j);
    const RowStat st = row_stats[g];
    tot += exp(acc * inv - (double)st.M) / st.Z;
  }
  return (float)tot;
}

// The same value computed by one whole wave: lanes split head_dim, fp64 tree reduction (the fp64
// sum order differs from the sequential one by ~1e-16 relative, far below fp32 rounding).
template <int DT>
__device__ inline float refined_score_wave(const RowGeom& geo, const void* q_last, const void* K, const PageMap& pm,
                                        int64_t ks_problem, int64_t ks_head, int64_t ks_token, const RowStat* row_stats,
                                        int prob, int c, int64_t tok, int g_lo, int g_hi) {
  const int D = geo.D, G = geo.G, lane = threadIdx.x & 63;
  const int64_t k_off = kv_offset(pm, pm.ks_page, ks_problem, ks_head, ks_token, prob, c, tok);
  const double inv = 1.0 / sqrt((double)D);
  double tot = 0.0;
  for (int g = g_lo; g < g_hi; ++g) {
    const int64_t q_off = ((int64_t)prob * geo.Hq + c * G + g) * D;
    double acc = 0.0;
    for (int j = lane; j < D; j += 64) acc += elem_f64<DT>(q_last, q_off + j) * elem_f64<DT>(K, k_off + j);
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o);
    const RowStat st = row_stats[g];
    tot += exp(acc * inv - (double)st.M) / st.Z;
  }
  return (float)tot;
}

}  // namespace sagekv
