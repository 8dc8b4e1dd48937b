// Fast eviction path (paper Sec. 2 Step 2, same result as the dense path): instead of writing
// every token's logits during the K stream and reading them back, keep only the few tokens that
// can reach the top-k.
//
//   sample_kernel     a strided sample of each row -> approximate softmax statistics (M^, Z^) per
//                     head and a conservative threshold tau^ on the approximate score: the sample
//                     quantile of rank ~1.5 k/E, so about 1.5 k tokens of the row pass it.
//   (score pass)      score_mfma_kernel<FILTER>: exact logits, exact softmax partials; tokens
//                     whose approximate score reaches tau^ are kept, with their exact fp32 logits,
//                     in the slots of their score chunk (no global atomics).
//   (stats)           exact (M, Z) per head and the bound rho * tau^ on the exact score of every
//                     token that was dropped.
//   topk_cand_kernel  exact scores of the candidates, radix select, fp64 re-evaluation near the
//                     k-th score, exact select, then an LDS bitmap turns the unordered list into
//                     ascending positions.  The row is only accepted if its k-th score clears the
//                     bound, i.e. if no dropped token could have been selected; otherwise the row
//                     is flagged and the dense path redoes it.
#include "device_utils.h"
#include "kernels.h"
#include "radix_select.h"

namespace sagekv {

namespace {

constexpr int kMaxTies = 1024;
constexpr int kFastMaxG = 16;

__device__ inline float block_max(float v, float* red) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int i = 1; i < kTopkWaves; ++i) r = fmaxf(r, red[i]);
  return r;
}

__device__ inline float block_sum(float v, float* red) {
  v = group_sum<64>(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = 0.f;
#pragma unroll
  for (int i = 0; i < kTopkWaves; ++i) r += red[i];
  return r;
}

template <int D>
__global__ __launch_bounds__(kTopkThreads) void sample_kernel(SampleParams p) {
  constexpr int CH = D / 8, TPL = 64 / CH, U = 8;
  __shared__ TopkShared sh;
  __shared__ float red[kTopkWaves];
  __shared__ float sM[kFastMaxG], sInv[kFastMaxG];

  const int row = blockIdx.x, tid = threadIdx.x;
  const int prob = row / p.geo.Hkv, c = row % p.geo.Hkv;
  const int lane = tid & 63, wave = tid >> 6;
  const int tq = lane / CH, cl = lane % CH;
  const int G = p.geo.G;
  const int64_t L = p.geo.L, S = p.S, W = p.W, E = L - S - W;
  const int nA = p.n_sink_s, nB = p.n_cand_s, nC = p.n_recent_s, ns = nA + nB + nC;

  if (tid == 0) p.row_fail[row] = 0;

  auto sample_token = [&](int j) -> int64_t {
    if (j < nA) return (int64_t)j * S / nA;
    j -= nA;
    if (j < nB) return S + (int64_t)j * E / nB;
    j -= nB;
    return L - W + (int64_t)j * W / nC;
  };
  auto sample_weight = [&](int j) -> float {
    if (j < nA) return (float)S / (float)nA;
    if (j < nA + nB) return (float)E / (float)nB;
    return (float)W / (float)nC;
  };

  // 1. logits of the sampled tokens
  const char* Krow = (const char*)p.K + ((int64_t)prob * p.ks_problem + (int64_t)c * p.ks_head) * 2;
  const char* qrow = (const char*)p.q_last + ((int64_t)prob * p.geo.Hq + (int64_t)c * G) * D * 2;
  float* slog = p.samp_logit + (int64_t)row * ns * G;
  for (int j0 = wave * TPL * U; j0 < ns; j0 += kTopkWaves * TPL * U) {
    uint4 kv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int j = j0 + u * TPL + tq;
      j = j < ns ? j : ns - 1;
      kv[u] = ld16(Krow + sample_token(j) * p.ks_token * 2 + cl * 16);
    }
    for (int g = 0; g < G; ++g) {
      const uint4 qv = ld16(qrow + ((int64_t)g * D + cl * 8) * 2);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float v = group_sum<CH>(dot16<DT_BF16>(kv[u], qv, 0.f)) * p.scale;
        const int j = j0 + u * TPL + tq;
        if (j < ns && cl == 0) slog[(int64_t)j * G + g] = v;
      }
    }
  }
  __syncthreads();

  // 2. approximate softmax statistics per head: M^ = max, Z^ = sum of weight * exp(l - M^)
  for (int g = 0; g < G; ++g) {
    float mx = -INFINITY;
    for (int j = tid; j < ns; j += kTopkThreads) mx = fmaxf(mx, slog[(int64_t)j * G + g]);
    mx = block_max(mx, red);
    float z = 0.f;
    for (int j = tid; j < ns; j += kTopkThreads) z += sample_weight(j) * exp_fast(slog[(int64_t)j * G + g] - mx);
    z = block_sum(z, red);
    if (tid == 0) {
      sM[g] = mx;
      sInv[g] = 1.0f / z;
      p.samp_stats[(int64_t)row * G + g] = make_float2(mx, 1.0f / z);
    }
  }
  __syncthreads();

  // 3. approximate scores of the sampled candidates, 4. their rank-th largest value
  float* ss = p.samp_score + (int64_t)row * nB;
  for (int j = tid; j < nB; j += kTopkThreads) {
    float a = 0.f;
    for (int g = 0; g < G; ++g) a += exp_fast(slog[(int64_t)(nA + j) * G + g] - sM[g]) * sInv[g];
    ss[j] = a;
  }
  __syncthreads();
  float tau_f = 0.f;  // rank beyond the sample: everything passes (the row then overflows and is redone)
  if (p.rank >= 1 && p.rank <= nB) {
    uint32_t tau;
    int quota;
    radix_select(sh, ss, nB, p.rank, false, &tau, &quota);
    tau_f = __uint_as_float(tau);
  }
  if (tid == 0) p.samp_tau[row] = tau_f;
}

template <int DT>
__global__ __launch_bounds__(kTopkThreads) void topk_cand_kernel(TopkCandParams p) {
  __shared__ TopkShared sh;
  __shared__ float sM[kFastMaxG], sInv[kFastMaxG];
  __shared__ int tie_idx[kMaxTies];
  __shared__ int n_tie;
  extern __shared__ uint32_t bitmap[];  // one bit per eviction candidate of the row

  const int row = blockIdx.x, tid = threadIdx.x;
  const int prob = row / p.geo.Hkv, c = row % p.geo.Hkv;
  const int S = p.S, W = p.W, k = p.k, G = p.geo.G;
  const int64_t L = p.geo.L, E = L - S - W;
  const int n_kept = S + k + W;
  int32_t* kept = p.kept_idx + (int64_t)row * n_kept;

  for (int t = tid; t < S; t += kTopkThreads) kept[t] = t;
  for (int t = tid; t < W; t += kTopkThreads) kept[S + k + t] = (int32_t)(L - W + t);
  if (k == 0) return;

  // candidates per score chunk -> offsets of a dense list
  __shared__ int chunk_off[1025];
  const int* cnt = p.cand_count + (int64_t)row * p.n_chunks;
  {
    const int v = tid < p.n_chunks ? cnt[tid] : 0;
    int tot;
    const int incl = block_scan_incl<kTopkThreads>(v, sh.wave_tot, &tot);
    if (tid < p.n_chunks) chunk_off[tid] = incl - v;
    if (tid == 0) chunk_off[p.n_chunks] = tot;
  }
  if (tid < G) {
    const RowStat st = p.stats[(int64_t)row * G + tid];
    sM[tid] = st.M;
    sInv[tid] = st.invZ;
  }
  if (tid == 0) n_tie = 0;
  __syncthreads();
  const int n_c = chunk_off[p.n_chunks];
  if (n_c > p.cap || n_c < k) {  // far more candidates than planned, or the threshold was too high
    if (tid == 0) p.row_fail[row] = 1;
    return;
  }

  // exact fp32 scores of the candidates (same arithmetic and order as the dense combine stage);
  // one wave per chunk
  float* cs = p.cand_score + (int64_t)row * p.cap;
  int32_t* ci = p.cand_pos + (int64_t)row * p.cap;
  for (int ch = tid >> 6; ch < p.n_chunks; ch += kTopkWaves) {
    const int n = chunk_off[ch + 1] - chunk_off[ch];
    const int64_t slot = ((int64_t)row * p.n_chunks + ch) * kScoreChunk;
    for (int j = tid & 63; j < n; j += 64) {
      const float* lg = p.cand_logit + (slot + j) * p.Gs;
      float a = 0.f;
      for (int g = 0; g < G; ++g) a += exp_accurate(lg[g] - sM[g]) * sInv[g];
      cs[chunk_off[ch] + j] = a;
      ci[chunk_off[ch] + j] = p.cand_idx[slot + j];
    }
  }
  __syncthreads();

  uint32_t tau;
  int quota;
  radix_select(sh, cs, n_c, k, false, &tau, &quota);
  const float tf = __uint_as_float(tau);
  const float lo = tf * (1.0f - p.band), hi = tf * (1.0f + p.band);
  for (int j = tid; j < n_c; j += kTopkThreads) {
    const float v = cs[j];
    if (v >= lo && v <= hi)
      cs[j] = refined_score<DT>(p.geo, p.q_last, p.K, p.ks_problem, p.ks_head, p.ks_token, p.stats, prob, c, row, ci[j]);
  }
  __syncthreads();
  radix_select(sh, cs, n_c, k, false, &tau, &quota);

  // every token outside the list scores below bound[row]: accept only if neither the k-th score
  // nor anything in its re-evaluation band could be such a token
  if (!(__uint_as_float(tau) * (1.0f - 2.0f * p.band) > p.bound[row])) {
    if (tid == 0) p.row_fail[row] = 1;
    return;
  }

  const int n_words = (int)((E + 31) / 32);
  for (int w = tid; w < n_words; w += kTopkThreads) bitmap[w] = 0u;
  __syncthreads();
  for (int j = tid; j < n_c; j += kTopkThreads) {
    const uint32_t key = __float_as_uint(cs[j]);
    const int pos = ci[j] - S;
    if (key > tau) {
      atomicOr(&bitmap[pos >> 5], 1u << (pos & 31));
    } else if (key == tau) {
      const int t = atomicAdd(&n_tie, 1);
      if (t < kMaxTies) tie_idx[t] = pos;
    }
  }
  __syncthreads();
  const int nt = n_tie;
  if (nt > kMaxTies) {  // a degenerate row of equal scores: leave it to the dense path
    if (tid == 0) p.row_fail[row] = 1;
    return;
  }
  for (int t = tid; t < nt; t += kTopkThreads) {  // ties go to the lowest indices
    const int me = tie_idx[t];
    int rank = 0;
    for (int u = 0; u < nt; ++u) rank += tie_idx[u] < me;
    if (rank < quota) atomicOr(&bitmap[me >> 5], 1u << (me & 31));
  }
  __syncthreads();

  int run = 0;
  for (int w0 = 0; w0 < n_words; w0 += kTopkThreads) {
    const int w = w0 + tid;
    uint32_t word = w < n_words ? bitmap[w] : 0u;
    const int cnt = __popc(word);
    int tot;
    const int incl = block_scan_incl<kTopkThreads>(cnt, sh.wave_tot, &tot);
    int pos = run + incl - cnt;
    while (word) {
      const int b = __ffs(word) - 1;
      word &= word - 1;
      if (pos < k) kept[S + pos] = (int32_t)(S + w * 32 + b);
      ++pos;
    }
    run += tot;
  }
}

__global__ __launch_bounds__(kTopkThreads) void collect_failed_kernel(const int* row_fail, int rows, int* fail_list,
                                                                      int* n_fail) {
  __shared__ int wave_tot[kTopkWaves];
  int run = 0;
  for (int r0 = 0; r0 < rows; r0 += kTopkThreads) {
    const int r = r0 + threadIdx.x;
    const int f = r < rows ? (row_fail[r] != 0) : 0;
    int tot;
    const int incl = block_scan_incl<kTopkThreads>(f, wave_tot, &tot);
    if (f) fail_list[run + incl - 1] = r;
    run += tot;
  }
  if (threadIdx.x == 0) *n_fail = run;
}

}  // namespace

hipError_t launch_sample(const SampleParams& p, hipStream_t s) {
  const int rows = p.geo.n_problems * p.geo.Hkv;
  if (p.geo.dtype != DT_BF16 || p.geo.G > kFastMaxG) return hipErrorInvalidValue;
  if (p.geo.D == 128)
    hipLaunchKernelGGL(sample_kernel<128>, dim3((unsigned)rows), dim3(kTopkThreads), 0, s, p);
  else
    hipLaunchKernelGGL(sample_kernel<64>, dim3((unsigned)rows), dim3(kTopkThreads), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_topk_cand(const TopkCandParams& p, hipStream_t s) {
  const int rows = p.geo.n_problems * p.geo.Hkv;
  const int64_t E = p.geo.L - p.S - p.W;
  const size_t lds = (size_t)((E + 31) / 32) * 4;
  if (lds > 64 * 1024 || p.geo.G > kFastMaxG) return hipErrorInvalidValue;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)topk_cand_kernel<DT_BF16>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(topk_cand_kernel<DT_BF16>, dim3((unsigned)rows), dim3(kTopkThreads), lds, s, p);
  return hipGetLastError();
}

hipError_t launch_collect_failed(const int* row_fail, int rows, int* fail_list, int* n_fail, hipStream_t s) {
  hipLaunchKernelGGL(collect_failed_kernel, dim3(1), dim3(kTopkThreads), 0, s, row_fail, rows, fail_list, n_fail);
  return hipGetLastError();
}

}  // namespace sagekv
