// Fast eviction path (paper Sec. 2 Step 2, same result as the dense path): instead of writing
// every token's logits during the K stream and reading them back, keep only the few tokens that
// can reach the top-k.
//
//   sample_*_kernel   a strided sample of each row -> approximate softmax statistics (M^, Z^) per
//                     head and a conservative threshold tau^ on the approximate score: a sample
//                     quantile chosen so that, four sigma low, 1.15 k tokens of the row still pass.
//   (score pass)      score_mfma_kernel in SCORE_FILTER mode: exact logits, exact softmax partials;
//                     tokens whose approximate score reaches tau^ are kept, with their exact fp32 logits,
//                     in the slots of their score chunk (no global atomics) or, once a chunk has used
//                     its slots up, in the row's overflow pool.
//   topk_cand_kernel  exact (M, Z) per head from the partials and the bound rho * tau^ on the exact
//                     score of every token that was dropped; exact scores of the candidates, radix select
//                     of the k-th score, fp64 re-evaluation and exact ranking of the few candidates around
//                     it, then an LDS bitmap turns the unordered selection into ascending positions.  The
//                     row is only accepted if its k-th score clears the bound, i.e. if no dropped token
//                     could have been selected; otherwise it is flagged and the dense stages redo it.
#include "device_utils.h"
#include "kernels.h"
#include "radix_select.h"

namespace sagekv {

namespace {

constexpr int kMaxBand = 1024;  // candidates re-scored in fp64 per row on the fast path
constexpr int kFastMaxG = 16;
constexpr float kHeavyShare = 0.01f;  // see sample_stats_kernel (0.3 % and 0.1 % measured worse)

// Per row: approximate softmax statistics of every head from the sampled logits; per selection list
// (one per row, or one per query head): approximate scores of the sampled candidates and their
// rank-th largest value = the list's filter threshold.  A row with several lists is shared by
// gridDim.y workgroups, each repeating the (cheap) statistics and taking its part of the lists.
__global__ __launch_bounds__(kTopkThreads) void sample_stats_kernel(SampleParams p) {
  __shared__ TopkShared sh;
  __shared__ float2 red[kTopkWaves][kFastMaxG];
  __shared__ float sM[kFastMaxG], sInv[kFastMaxG], sHeavy[kFastMaxG];
  __shared__ float ss[8192];  // approximate scores of the sampled candidates

  const int row = blockIdx.x, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int G = p.geo.G, Gs = p.Gs;
  const bool per_head = p.n_lists > 1;
  const int lists_per_wg = (p.n_lists + (int)gridDim.y - 1) / (int)gridDim.y;
  const int list_lo = (int)blockIdx.y * lists_per_wg;
  const int list_hi = list_lo + lists_per_wg < p.n_lists ? list_lo + lists_per_wg : p.n_lists;
  const int n_slots = 64 * (p.nA + p.nB + p.nC), nB = 64 * p.nB;
  const float* slog = p.samp_logit + (int64_t)row * n_slots * Gs;
  if (tid == 0 && blockIdx.y == 0) {
    p.row_fail[row] = 0;
    p.ovf_count[row] = 0;
    if (row == 0) *p.n_fail = 0;
  }

  // weight of sample slot s (0 = the slot is outside the part its block samples)
  auto weight = [&](int s) -> float {
    const int b = s >> 6, t = s & 63;
    if (b < p.nA) return t < p.validA ? p.wA : 0.f;
    if (b < p.nA + p.nB) return p.wB;
    return 64 * (p.nA + p.nB + p.nC) - s <= p.validC ? p.wC : 0.f;
  };
  // logits of heads g4 .. g4 + 3 of sample slot s (rows of samp_logit are padded to a multiple of 4
  // heads: 16-byte loads)
  auto load4 = [&](int s, int g4, float (&xs)[4]) {
    const float4 v = *reinterpret_cast<const float4*>(slog + (int64_t)s * Gs + g4);
    xs[0] = v.x, xs[1] = v.y, xs[2] = v.z, xs[3] = v.w;
  };

  // approximate softmax statistics per head, one pass: M^ = max, Z^ = sum of weight * exp(l - M^)
  {
    float m[kFastMaxG], z[kFastMaxG];
#pragma unroll
    for (int g = 0; g < kFastMaxG; ++g) {
      m[g] = -INFINITY;
      z[g] = 0.f;
    }
    for (int s = tid; s < n_slots; s += kTopkThreads) {
      const float w = weight(s);
      if (w > 0.f) {
#pragma unroll
        for (int g4 = 0; g4 < kFastMaxG; g4 += 4)
          if (g4 < G) {
            float xs[4];
            load4(s, g4, xs);
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (g4 + e < G) {
                const int g = g4 + e;
                const float mn = fmaxf(m[g], xs[e]);
                z[g] = z[g] * exp_fast(m[g] - mn) + w * exp_fast(xs[e] - mn);
                m[g] = mn;
              }
          }
      }
    }
#pragma unroll
    for (int g = 0; g < kFastMaxG; ++g)
      if (g < G) {
        const float M = wave_max(m[g]);
        float zz = (m[g] == -INFINITY) ? 0.f : z[g] * exp_fast(m[g] - M);
        zz = group_sum<64>(zz);
        if (lane == 0) red[wave][g] = make_float2(M, zz);
      }
    __syncthreads();
    if (tid < G) {
      float M = red[0][tid].x;
      for (int w = 1; w < kTopkWaves; ++w) M = fmaxf(M, red[w][tid].x);
      float zz = 0.f;
      for (int w = 0; w < kTopkWaves; ++w)
        zz += (red[w][tid].x == -INFINITY) ? 0.f : red[w][tid].y * exp_fast(red[w][tid].x - M);
      sM[tid] = M;
      sInv[tid] = zz;  // first estimate of Z^, refined below
    }
    __syncthreads();
    // Second pass: a sampled token that would alone stand for more than 1 % of the head's mass is a
    // heavy token, and heavy tokens are rare: it is counted once, not once per token it was meant
    // to represent.  (Attention mass sits on few tokens; scaling such a token up by the sampling
    // rate would put the head's normaliser off by a large factor and the row could not be
    // certified.  Under-counting only lets a few more candidates through.)
    float zh[kFastMaxG];  // what the heavy tokens had added to the first estimate
#pragma unroll
    for (int g = 0; g < kFastMaxG; ++g) z[g] = zh[g] = 0.f;
    for (int s = tid; s < n_slots; s += kTopkThreads) {
      const float w = weight(s);
      if (w > 0.f) {
#pragma unroll
        for (int g4 = 0; g4 < kFastMaxG; g4 += 4)
          if (g4 < G) {
            float xs[4];
            load4(s, g4, xs);
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (g4 + i < G) {
                const int g = g4 + i;
                const float e = exp_fast(xs[i] - sM[g]);
                const bool heavy = w * e > kHeavyShare * sInv[g];
                z[g] += (heavy ? 1.f : w) * e;
                zh[g] += heavy ? w * e : 0.f;
              }
          }
      }
    }
    __syncthreads();  // every thread has read the first estimates
#pragma unroll
    for (int g = 0; g < kFastMaxG; ++g)
      if (g < G) {
        const float zz = group_sum<64>(z[g]);
        const float hh = group_sum<64>(zh[g]);
        if (lane == 0) red[wave][g] = make_float2(hh, zz);
      }
    __syncthreads();
    if (tid < G) {
      float zz = 0.f, hh = 0.f;
      for (int w = 0; w < kTopkWaves; ++w) {
        hh += red[w][tid].x;
        zz += red[w][tid].y;
      }
      sHeavy[tid] = hh / sInv[tid];  // share of the first estimate that came from heavy tokens
      sInv[tid] = 1.0f / zz;
      if (blockIdx.y == 0) p.samp_stats[(int64_t)row * G + tid] = make_float2(sM[tid], 1.0f / zz);
    }
  }
  __syncthreads();
  // A heavy-tailed row (the sample met heavy tokens) has heads whose normalisers are known with
  // very different accuracy, whatever the sampler does about the heavy tokens it saw: some head
  // has others it did not see.  The summed score then needs a threshold further down: the rank
  // grows with the largest heavy share, up to twice the planned one (the candidate capacity is
  // planned for that).  Per-query lists do not need it: a head's own scale cancels.
  int rank = p.rank;
  if (!per_head) {
    float h = 0.f;
    for (int g = 0; g < G; ++g) h = fmaxf(h, sHeavy[g]);
    const float grow = fminf(1.f, 4.f * fmaxf(0.f, h - 0.04f));
    rank = (int)((float)p.rank * (1.f + grow));
    if (rank > nB) rank = nB;
  }

  // group-sum: the threshold is on the summed approximate score; per-query: on the head's own
  for (int li = list_lo; li < list_hi; ++li) {
    __syncthreads();  // the previous list's select has read ss
    for (int s = tid; s < nB; s += kTopkThreads) {
      const float* lg = slog + (int64_t)(64 * p.nA + s) * Gs;
      float a = 0.f;
      if (per_head) {
        a = exp_fast(lg[li] - sM[li]) * sInv[li];
      } else {
#pragma unroll
        for (int g4 = 0; g4 < kFastMaxG; g4 += 4)
          if (g4 < G) {
            float xs[4];
            load4(64 * p.nA + s, g4, xs);
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (g4 + i < G) a += exp_fast(xs[i] - sM[g4 + i]) * sInv[g4 + i];
          }
      }
      ss[s] = a;
    }
    __syncthreads();
    float tau_f = 0.f;  // rank beyond the sample: everything passes (the row is then redone densely)
    if (rank >= 1 && p.rank <= nB) {
      uint32_t tau;
      int quota;
      radix_select(sh, ss, nB, rank, false, &tau, &quota);
      tau_f = __uint_as_float(tau);
    }
    if (tid == 0) p.samp_tau[(int64_t)row * p.n_lists + li] = tau_f;
  }
}

// The row cannot be certified (reason: 1 too many / too few candidates, 2 too few reach the bound,
// 3 the k-th score does not clear the bound, 4 a band of near-ties): the dense stages redo it.  Several
// lists of a row may flag it; the count of flagged rows goes up once.
__device__ __forceinline__ void flag_row(const TopkCandParams& p, int row, int reason) {
  if (atomicExch(&p.row_fail[row], reason) == 0) atomicAdd(p.n_fail, 1);
}

// PQ: per-query lists (n_lists = G > 1), each list keeps its own compacted candidates.
template <int DT, bool PQ>
__device__ __forceinline__ void topk_cand_body(const TopkCandParams& p) {
  __shared__ TopkShared sh;
  __shared__ float sM[kFastMaxG], sInv[kFastMaxG];
  __shared__ RowStat s_stat[kFastMaxG];  // exact statistics of this list's heads (group-sum: all G)
  __shared__ double s_rho[kFastMaxG], s_flushed[kFastMaxG];
  __shared__ int band_j[kMaxBand], band_tok[kMaxBand];
  __shared__ float band_v[kMaxBand];
  __shared__ int n_band, n_above, n_list;
  extern __shared__ __align__(16) uint32_t bitmap[];  // one bit per eviction candidate of the row

  const int list = blockIdx.x, tid = threadIdx.x;  // one list per row, or one per (row, query head)
  const int row = list / p.n_lists, gl = list % p.n_lists;
  const int prob = row / p.geo.Hkv, c = row % p.geo.Hkv;
  const int S = p.S, W = p.W, k = p.k, G = p.geo.G;
  const int g_lo = p.n_lists > 1 ? gl : 0, g_hi = p.n_lists > 1 ? gl + 1 : G;
  const int64_t L = p.geo.L, E = L - S - W;
  const int n_kept = S + p.n_lists * k + W;
  int32_t* kept_row = p.kept_idx + (int64_t)row * n_kept;
  int32_t* kept = kept_row + gl * k;  // this list's k slots start at kept[S]

  if (gl == 0) {
    for (int t = tid; t < S; t += kTopkThreads) kept_row[t] = t;
    for (int t = tid; t < W; t += kTopkThreads) kept_row[S + p.n_lists * k + t] = (int32_t)(L - W + t);
  }
  // the dense stages that redo a flagged row add to this list's first-digit histogram
  for (int b = tid; b < kHistBins; b += kTopkThreads) p.ghist[(int64_t)list * kHistBins + b] = 0;

  // Exact softmax statistics of this list's heads, one wave per head, from the partials of the
  // filtering pass; and how far the sampled statistics were off: rho = (exact weight) / (sampled weight).
  {
    const int wave = tid >> 6, g = g_lo + wave;
    if (g < g_hi) {
      const RowStat st = merge_partials_wave(p.partials + ((int64_t)row * G + g) * p.n_chunks, p.n_chunks);
      if ((tid & 63) == 0) {
        s_stat[g] = st;
        sM[g] = st.M;
        sInv[g] = st.invZ;
        p.stats[(int64_t)row * G + g] = st;
        const float2 ss = p.samp_stats[(int64_t)row * G + g];
        s_rho[g] = exp((double)ss.x - (double)st.M) / (st.Z * (double)ss.y);
        s_flushed[g] = 0x1p-126 * (double)ss.y;  // the filter's exponentials come out as 0 below 2^-126
      }
    }
  }
  if (k == 0) return;

  // candidates per score chunk -> offsets of a dense list: the chunks' own slots first, the row's
  // overflow pool behind them
  __shared__ int chunk_off[1025];
  __shared__ int s_raw_total;
  const int* cnt = p.cand_count + (int64_t)row * p.n_chunks;
  {
    const int raw = tid < p.n_chunks ? cnt[tid] : 0;
    const int v = raw < p.cap_c ? raw : p.cap_c;
    int tot, raw_tot;
    const int incl = block_scan_incl<kTopkThreads>(v, sh.wave_tot, &tot);
    if (tid < p.n_chunks) chunk_off[tid] = incl - v;
    if (tid == 0) chunk_off[p.n_chunks] = tot;
    block_scan_incl<kTopkThreads>(raw, sh.wave_tot, &raw_tot);
    if (tid == 0) s_raw_total = raw_tot;
  }
  if (tid == 0) n_band = n_above = n_list = 0;
  __syncthreads();
  // A token the filter dropped had approximate score < tau^, so its exact score is below rho * tau^
  // (plus what exponentials flushed to zero could hide, plus fp32 slack), rho the worst head's.
  float bound;
  {
    double rho = 0.0, fl = 0.0;
    for (int g = g_lo; g < g_hi; ++g) {
      const double r = s_rho[g];
      rho = r > rho || !(r == r) ? r : rho;
      fl += s_flushed[g];
    }
    bound = (float)(rho * ((double)p.samp_tau[list] + fl) * 1.001);
  }
  const int n_primary = chunk_off[p.n_chunks];
  const int n_ovf = s_raw_total - n_primary;  // = the row's overflow counter
  const int n_all = s_raw_total;
  if (n_all > p.cap || n_all < k || n_ovf > p.cap_o) {  // far more candidates than planned, or the threshold was too high
    if (tid == 0) flag_row(p, row, 1);
    return;
  }

  // Exact fp32 scores of the candidates (same arithmetic and order as the dense combine stage).
  // The list keeps those that reach the bound: a candidate below it is in the same position as a
  // token the filter dropped (the row is only accepted if the k-th score's band lies above the
  // bound), and with per-query lists most of the row's shared candidates came in through other heads.
  constexpr bool compact = PQ;
  float* cs = p.cand_score + (int64_t)list * p.cs_pitch;
  int32_t* ci = p.cand_pos + (int64_t)list * p.cs_pitch;
  const int64_t row_slots = (int64_t)row * p.slots_per_row;
  const int64_t ovf_base = row_slots + (int64_t)p.n_chunks * p.cap_c;
  for (int d0 = 0; d0 < n_all; d0 += 4 * kTopkThreads) {
    int64_t slot[4];  // the candidate's record, -1: past the end
#pragma unroll
    for (int u = 0; u < 4; ++u) {  // independent lookups: their loads overlap
      const int dj = d0 + u * kTopkThreads + tid;
      int lo_c = 0, hi_c = p.n_chunks;  // chunk with chunk_off[ch] <= dj < chunk_off[ch + 1]
      while (hi_c - lo_c > 1) {
        const int mid = (lo_c + hi_c) >> 1;
        if (chunk_off[mid] <= dj) lo_c = mid; else hi_c = mid;
      }
      slot[u] = dj >= n_all ? -1
                : dj < n_primary ? row_slots + (int64_t)lo_c * p.cap_c + (dj - chunk_off[lo_c])
                                 : ovf_base + (dj - n_primary);
    }
    if constexpr (compact) {  // per-query lists: only this list's head is read
      float x[4];
      int32_t ti[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int64_t sl = slot[u] < 0 ? row_slots : slot[u];
        ti[u] = p.cand_idx[sl];
        x[u] = p.cand_logit[sl * p.Gs + gl];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        float a = 0.f;
        a += exp_times(x[u] - sM[gl], sInv[gl]);
        const bool keep = slot[u] >= 0 && a >= bound;
        const unsigned long long bal = __ballot(keep);
        if (bal) {  // wave-uniform
          int base = 0;
          if ((tid & 63) == 0) base = atomicAdd(&n_list, __popcll(bal));
          base = __shfl(base, 0);
          if (keep) {
            const int pos = base + __popcll(bal & ((1ull << (tid & 63)) - 1ull));
            cs[pos] = a;
            ci[pos] = ti[u];
          }
        }
      }
    } else {
    // one list per row: nearly every candidate reaches the bound, they stay in place
    float4 lg[4][kFastMaxG / 4];
    int32_t ti[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t sl = slot[u] < 0 ? row_slots : slot[u];
      ti[u] = p.cand_idx[sl];
#pragma unroll
      for (int g4 = 0; g4 < kFastMaxG / 4; ++g4)
        if (g4 * 4 < G) lg[u][g4] = *reinterpret_cast<const float4*>(p.cand_logit + sl * p.Gs + g4 * 4);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int dj = d0 + u * kTopkThreads + tid;
      if (dj < n_all) {
        float a = 0.f;
#pragma unroll
        for (int g4 = 0; g4 < kFastMaxG / 4; ++g4)
          if (g4 * 4 < G) {
            const float x[4] = {lg[u][g4].x, lg[u][g4].y, lg[u][g4].z, lg[u][g4].w};
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (g4 * 4 + e < G) a += exp_times(x[e] - sM[g4 * 4 + e], sInv[g4 * 4 + e]);
          }
        cs[dj] = a;
        ci[dj] = ti[u];
      }
    }
    }
  }
  __syncthreads();
  const int n_c = compact ? n_list : n_all;
  if (n_c < k) {
    if (tid == 0) flag_row(p, row, 2);
    return;
  }

  // coarse k-th score, then the candidates within the band around it are re-scored in fp64 and
  // ranked exactly (score descending, index ascending); everything above the band is selected
  uint32_t tau;
  int quota;
  radix_select(sh, cs, n_c, k, false, &tau, &quota);
  const float tf = __uint_as_float(tau);
  const float lo = tf * (1.0f - p.band) - kDenormSlack, hi = tf * (1.0f + p.band) + kDenormSlack;
  // every token outside the list scores below bound[row]: the row is certified only if no such
  // token can reach the band
  if (!(lo * (1.0f - p.band) > bound)) {
    if (tid == 0) flag_row(p, row, 3);
    return;
  }
  const int n_words = (int)((E + 31) / 32);
  for (int w = tid; w < n_words; w += kTopkThreads) bitmap[w] = 0u;
  __syncthreads();
  for (int j0 = 0; j0 < n_c; j0 += kTopkThreads) {
    const int j = j0 + tid;
    const float v = j < n_c ? cs[j] : 0.f;
    const bool above = j < n_c && v > hi;
    if (above) {
      const int pos = ci[j] - S;
      atomicOr(&bitmap[pos >> 5], 1u << (pos & 31));
    } else if (j < n_c && v >= lo) {
      const int t = atomicAdd(&n_band, 1);
      if (t < kMaxBand) band_j[t] = j;
    }
    const unsigned long long bal = __ballot(above);
    if ((tid & 63) == 0 && bal) atomicAdd(&n_above, __popcll(bal));
  }
  __syncthreads();
  const int nb = n_band, r = k - n_above;
  if (nb > kMaxBand || r < 1 || r > nb) {  // a degenerate row of (nearly) equal scores: dense path
    if (tid == 0) flag_row(p, row, 4);
    return;
  }
  for (int t = tid >> 6; t < nb; t += kTopkWaves) {
    const int tok = ci[band_j[t]];
    const float v = refined_score_wave<DT>(p.geo, p.q_last, p.K, p.pm, p.ks_problem, p.ks_head, p.ks_token, s_stat, prob, c,
                                           tok, g_lo, g_hi);
    if ((tid & 63) == 0) {
      band_v[t] = v;
      band_tok[t] = tok;
    }
  }
  __syncthreads();
  for (int t = tid; t < nb; t += kTopkThreads) {
    const float v = band_v[t];
    const int tok = band_tok[t];
    int rank = 0;
    for (int u = 0; u < nb; ++u) rank += band_v[u] > v || (band_v[u] == v && band_tok[u] < tok);
    if (rank < r) atomicOr(&bitmap[(tok - S) >> 5], 1u << ((tok - S) & 31));
  }
  __syncthreads();

  bitmap_compact(bitmap, n_words, S, kept + S, k, sh.wave_tot);
}

template <int DT>
__global__ __launch_bounds__(kTopkThreads) void topk_cand_kernel(TopkCandParams p) {
  topk_cand_body<DT, false>(p);
}

// Per-query lists: G workgroups per row.  Registers are capped so that two workgroups share a CU
// (8 waves per SIMD): the kernel is a chain of dependent memory round trips, a second resident
// workgroup fills the waits.
template <int DT>
__global__ __launch_bounds__(kTopkThreads, 8) void topk_cand_pq_kernel(TopkCandParams p) {
  topk_cand_body<DT, true>(p);
}

}  // namespace

hipError_t launch_sample(const SampleParams& p, hipStream_t s) {
  const int rows = p.geo.n_problems * p.geo.Hkv;
  if (p.geo.dtype != DT_BF16 || p.geo.G > kFastMaxG || p.nB * 64 > 8192) return hipErrorInvalidValue;
  hipError_t e = launch_sample_logits(p, s);
  if (e != hipSuccess) return e;
  // one workgroup per row, also with several lists per row: at 7 lists x 448 rows, two workgroups per row
  // took 139 us, one per (row, list) 147 us, one per row 108 us (the statistics dominate, not the selects)
  hipLaunchKernelGGL(sample_stats_kernel, dim3((unsigned)rows, 1u), dim3(kTopkThreads), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_topk_cand(const TopkCandParams& p, hipStream_t s) {
  const int rows = p.geo.n_problems * p.geo.Hkv;
  const int64_t E = p.geo.L - p.S - p.W;
  const size_t lds = (size_t)((E + 31) / 32) * 4;
  if (lds > 64 * 1024 || p.geo.G > kFastMaxG) return hipErrorInvalidValue;
  static uint64_t done_one = 0, done_pq = 0;
  const hipError_t e = p.n_lists > 1
                           ? allow_dynamic_lds((const void*)topk_cand_pq_kernel<DT_BF16>, 64 * 1024, &done_pq)
                           : allow_dynamic_lds((const void*)topk_cand_kernel<DT_BF16>, 64 * 1024, &done_one);
  if (e != hipSuccess) return e;
  const dim3 grid((unsigned)(rows * p.n_lists));
  if (p.n_lists > 1)
    hipLaunchKernelGGL(topk_cand_pq_kernel<DT_BF16>, grid, dim3(kTopkThreads), lds, s, p);
  else
    hipLaunchKernelGGL(topk_cand_kernel<DT_BF16>, grid, dim3(kTopkThreads), lds, s, p);
  return hipGetLastError();
}

}  // namespace sagekv
