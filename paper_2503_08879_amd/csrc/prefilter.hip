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
//   cand_split_pq_kernel + topk_cand_pq_kernel
//                     the same for one list per query head: a workgroup per row splits the row's candidates
//                     into the heads' lists, then a workgroup per (row, head) selects its list.
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
      if (blockIdx.y == 0) {
        p.samp_stats[(int64_t)row * G + tid] = make_float2(sM[tid], 1.0f / zz);
        p.heavy_thr[(int64_t)row * G + tid] = heavy_logit_threshold(sM[tid], zz);
      }
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

// Shared state of the candidate selection kernels.
struct CandShared {
  TopkShared sh;
  float sM[kFastMaxG], sInv[kFastMaxG];
  RowStat stat[kFastMaxG];  // exact statistics of the row's heads
  double rho[kFastMaxG], flushed[kFastMaxG];
  float bound[kFastMaxG];   // per-query lists: the bound of each head's list,
  float thr[kFastMaxG];     // and the same bound as a logit of that head
  int n_list[kFastMaxG];    // per-query lists: candidates each list has kept
  int band_j[kMaxBand], band_tok[kMaxBand];
  float band_v[kMaxBand];
  int n_band, n_above;
  int chunk_off[1025];
  int raw_total;
};

// First half, one workgroup per row: sink and recent indices, the exact softmax statistics of the row's
// heads, and the candidates' scratch lists.  One list per row (PQ false): cand_score / cand_pos get the
// exact fp32 score and the token of every candidate; *bound = the bound on a dropped token's score,
// *n_c = the number of candidates.  Per-query lists (PQ): the row's shared candidate records are read
// once and list g gets the LOGIT of head g and the token of every candidate that can reach the list's
// bound (s.bound[g], counts in s.n_list[g]).  False: nothing to select (k = 0) or the row was flagged.
template <int DT, bool PQ>
__device__ __forceinline__ bool cand_lists(const TopkCandParams& p, CandShared& s, int row, float* bound, int* n_c) {
  const int tid = threadIdx.x;
  const int S = p.S, W = p.W, k = p.k, G = p.geo.G;
  const int64_t L = p.geo.L;
  const int n_kept = S + p.n_lists * k + W;
  int32_t* kept_row = p.kept_idx + (int64_t)row * n_kept;

  for (int t = tid; t < S; t += kTopkThreads) kept_row[t] = t;
  for (int t = tid; t < W; t += kTopkThreads) kept_row[S + p.n_lists * k + t] = (int32_t)(L - W + t);
  // the dense stages that redo a flagged row add to its lists' first-digit histograms
  for (int b = tid; b < kHistBins * p.n_lists; b += kTopkThreads) p.ghist[(int64_t)row * p.n_lists * kHistBins + b] = 0;

  // Exact softmax statistics of the row's heads, one wave per head, from the partials of the
  // filtering pass; and how far the sampled statistics were off: rho = (exact weight) / (sampled weight).
  {
    const int g = tid >> 6;
    if (g < G) {
      const RowStat st = merge_partials_wave(p.partials + ((int64_t)row * G + g) * p.n_chunks, p.n_chunks);
      if ((tid & 63) == 0) {
        s.stat[g] = st;
        s.sM[g] = st.M;
        s.sInv[g] = st.invZ;
        p.stats[(int64_t)row * G + g] = st;
        const float2 ss = p.samp_stats[(int64_t)row * G + g];
        s.rho[g] = exp((double)ss.x - (double)st.M) / (st.Z * (double)ss.y);
        s.flushed[g] = 0x1p-126 * (double)ss.y;  // the filter's exponentials come out as 0 below 2^-126
      }
    }
  }
  if (k == 0) return false;

  // candidates per score chunk -> offsets of a dense list: the chunks' own slots first, the row's
  // overflow pool behind them
  const int* cnt = p.cand_count + (int64_t)row * p.n_chunks;
  {
    const int raw = tid < p.n_chunks ? cnt[tid] : 0;
    const int v = raw < p.cap_c ? raw : p.cap_c;
    int tot, raw_tot;
    const int incl = block_scan_incl<kTopkThreads>(v, s.sh.wave_tot, &tot);
    if (tid < p.n_chunks) s.chunk_off[tid] = incl - v;
    if (tid == 0) s.chunk_off[p.n_chunks] = tot;
    block_scan_incl<kTopkThreads>(raw, s.sh.wave_tot, &raw_tot);
    if (tid == 0) s.raw_total = raw_tot;
  }
  if (tid == 0) s.n_band = s.n_above = 0;
  if (tid < kFastMaxG) s.n_list[tid] = 0;
  __syncthreads();
  // A token the filter dropped had approximate score < tau^, so its exact score is below rho * tau^
  // (plus what exponentials flushed to zero could hide, plus fp32 slack), rho the worst head's; a
  // per-query list has its own head's.
  if (PQ) {
    if (tid < G) {
      const double bd = s.rho[tid] * ((double)p.samp_tau[(int64_t)row * G + tid] + s.flushed[tid]) * 1.001;
      s.bound[tid] = (float)bd;
      // exp(x - M) / Z >= bd  <=>  x >= M + log(bd Z); lowered by more than fp32 rounding can move either side
      s.thr[tid] = (float)((double)s.stat[tid].M + log(bd * s.stat[tid].Z) - 1e-4);
    }
  } else {
    double rho = 0.0, fl = 0.0;
    for (int g = 0; g < G; ++g) {
      const double r = s.rho[g];
      rho = r > rho || !(r == r) ? r : rho;
      fl += s.flushed[g];
    }
    *bound = (float)(rho * ((double)p.samp_tau[row] + fl) * 1.001);
  }
  const int n_primary = s.chunk_off[p.n_chunks];
  const int n_ovf = s.raw_total - n_primary;  // = the row's overflow counter
  const int n_all = s.raw_total;
  *n_c = n_all;
  if (n_all > p.cap || n_all < k || n_ovf > p.cap_o) {  // far more candidates than planned, or the threshold was too high
    if (tid == 0) flag_row(p, row, 1);
    return false;
  }
  __syncthreads();  // s.thr

  float* cs0 = p.cand_score + (int64_t)row * p.n_lists * p.cs_pitch;
  int32_t* ci0 = p.cand_pos + (int64_t)row * p.n_lists * p.cs_pitch;
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
        if (s.chunk_off[mid] <= dj) lo_c = mid; else hi_c = mid;
      }
      slot[u] = dj >= n_all ? -1
                : dj < n_primary ? row_slots + (int64_t)lo_c * p.cap_c + (dj - s.chunk_off[lo_c])
                                 : ovf_base + (dj - n_primary);
    }
    int32_t ti[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) ti[u] = p.cand_idx[slot[u] < 0 ? row_slots : slot[u]];
    if constexpr (PQ) {
      // four heads at a time: their logits are one 16-byte load per candidate
      for (int g4 = 0; g4 < G; g4 += 4) {
        float4 lg[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
          lg[u] = *reinterpret_cast<const float4*>(p.cand_logit + (slot[u] < 0 ? row_slots : slot[u]) * p.Gs + g4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int g = g4 + e;
          if (g >= G) break;  // workgroup-uniform
          float* cs = cs0 + (int64_t)g * p.cs_pitch;
          int32_t* ci = ci0 + (int64_t)g * p.cs_pitch;
          const float thr = s.thr[g];
          float x[4];
          unsigned long long bal[4];
          int n_wave = 0;
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            x[u] = e == 0 ? lg[u].x : e == 1 ? lg[u].y : e == 2 ? lg[u].z : lg[u].w;
            bal[u] = __ballot(slot[u] >= 0 && x[u] >= thr);
            n_wave += __popcll(bal[u]);
          }
          if (n_wave) {  // wave-uniform
            int base = 0;
            if ((tid & 63) == 0) base = atomicAdd(&s.n_list[g], n_wave);
            base = __shfl(base, 0);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              if ((bal[u] >> (tid & 63)) & 1ull) {
                const int pos = base + __popcll(bal[u] & ((1ull << (tid & 63)) - 1ull));
                cs[pos] = x[u];
                ci[pos] = ti[u];
              }
              base += __popcll(bal[u]);
            }
          }
        }
      }
    } else {
      // exact fp32 scores, same arithmetic and order as the dense combine stage; nearly every candidate
      // reaches the bound, they stay in place
      float4 lg[4][kFastMaxG / 4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int64_t sl = slot[u] < 0 ? row_slots : slot[u];
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
                if (g4 * 4 + e < G) a += exp_times(x[e] - s.sM[g4 * 4 + e], s.sInv[g4 * 4 + e]);
            }
          cs0[dj] = a;
          ci0[dj] = ti[u];
        }
      }
    }
  }
  __syncthreads();
  return true;
}

// Second half, one workgroup per list: the k best of the list's n_c candidates (cs: scores, or with
// `logits` the logits of head g_lo, turned into scores here; ci: tokens), certified against `bound`:
// every token outside the list scores below it.  s.stat[g_lo .. g_hi), s.sM, s.sInv hold the heads'
// statistics, s.n_band = s.n_above = 0; `kept` = the list's k output slots.
template <int DT>
__device__ __forceinline__ void select_list(const TopkCandParams& p, CandShared& s, uint32_t* bitmap, int row, int g_lo,
                                            int g_hi, float* cs, const int32_t* ci, int n_c, float bound, bool logits,
                                            int32_t* kept) {
  const int tid = threadIdx.x;
  const int prob = row / p.geo.Hkv, c = row % p.geo.Hkv;
  const int S = p.S, k = p.k;
  const int64_t E = p.geo.L - S - p.W;
  if (n_c < k) {
    if (tid == 0) flag_row(p, row, 2);
    return;
  }
  if (logits) {  // exact fp32 scores, same arithmetic as the dense stages
    const float M = s.sM[g_lo], inv = s.sInv[g_lo];
    for (int j = tid; j < n_c; j += kTopkThreads) cs[j] = exp_times(cs[j] - M, inv);
    __syncthreads();
  }
  // coarse k-th score, then the candidates within the band around it are re-scored in fp64 and
  // ranked exactly (score descending, index ascending); everything above the band is selected
  uint32_t tau;
  int quota;
  radix_select(s.sh, cs, n_c, k, false, &tau, &quota);
  const float tf = __uint_as_float(tau);
  const float lo = tf * (1.0f - p.band) - kDenormSlack, hi = tf * (1.0f + p.band) + kDenormSlack;
  // the row is certified only if no token outside the list can reach the band
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
      const int t = atomicAdd(&s.n_band, 1);
      if (t < kMaxBand) s.band_j[t] = j;
    }
    const unsigned long long bal = __ballot(above);
    if ((tid & 63) == 0 && bal) atomicAdd(&s.n_above, __popcll(bal));
  }
  __syncthreads();
  const int nb = s.n_band, r = k - s.n_above;
  if (nb > kMaxBand || r < 1 || r > nb) {  // a degenerate row of (nearly) equal scores: dense path
    if (tid == 0) flag_row(p, row, 4);
    return;
  }
  for (int t = tid >> 6; t < nb; t += kTopkWaves) {
    const int tok = ci[s.band_j[t]];
    const float v = refined_score_wave<DT>(p.geo, p.q_last, p.K, p.pm, p.ks_problem, p.ks_head, p.ks_token, s.stat, prob, c,
                                           tok, g_lo, g_hi);
    if ((tid & 63) == 0) {
      s.band_v[t] = v;
      s.band_tok[t] = tok;
    }
  }
  __syncthreads();
  for (int t = tid; t < nb; t += kTopkThreads) {
    const float v = s.band_v[t];
    const int tok = s.band_tok[t];
    int rank = 0;
    for (int u = 0; u < nb; ++u) rank += s.band_v[u] > v || (s.band_v[u] == v && s.band_tok[u] < tok);
    if (rank < r) atomicOr(&bitmap[(tok - S) >> 5], 1u << ((tok - S) & 31));
  }
  __syncthreads();
  bitmap_compact(bitmap, n_words, S, kept + S, k, s.sh.wave_tot);
}

// One list per row: both halves in one workgroup.
template <int DT>
__global__ __launch_bounds__(kTopkThreads) void topk_cand_kernel(TopkCandParams p) {
  __shared__ CandShared s;
  extern __shared__ __align__(16) uint32_t bitmap[];  // one bit per eviction candidate of the row
  const int row = blockIdx.x;
  float bound = 0.f;
  int n_c = 0;
  if (!cand_lists<DT, false>(p, s, row, &bound, &n_c)) return;
  select_list<DT>(p, s, bitmap, row, 0, p.geo.G, p.cand_score + (int64_t)row * p.cs_pitch,
                  p.cand_pos + (int64_t)row * p.cs_pitch, n_c, bound, false,
                  p.kept_idx + (int64_t)row * (p.S + p.k + p.W));
}

// Per-query lists, first launch: one workgroup per row splits the row's candidates into the lists
// (a list re-reading all of the row's records costs more than everything else it does) and leaves
// each list's count and bound in list_info; count -1: nothing to select for this row.
// Registers are capped in both launches so that two workgroups share a CU (8 waves per SIMD): the
// kernels are chains of dependent memory round trips, a second resident workgroup fills the waits.
template <int DT>
__global__ __launch_bounds__(kTopkThreads, 8) void cand_split_pq_kernel(TopkCandParams p) {
  __shared__ CandShared s;
  const int row = blockIdx.x, G = p.geo.G;
  float bound = 0.f;
  int n_c = 0;
  const bool ok = cand_lists<DT, true>(p, s, row, &bound, &n_c);  // its exits are workgroup-uniform
  if ((int)threadIdx.x < G)
    p.list_info[(int64_t)row * G + threadIdx.x] = make_float2(__int_as_float(ok ? s.n_list[threadIdx.x] : -1),
                                                               s.bound[threadIdx.x]);
}

// Per-query lists, second launch: one workgroup per (row, head).
template <int DT>
__global__ __launch_bounds__(kTopkThreads, 8) void topk_cand_pq_kernel(TopkCandParams p) {
  __shared__ CandShared s;
  extern __shared__ __align__(16) uint32_t bitmap[];
  const int list = blockIdx.x, G = p.geo.G;
  const int row = list / G, g = list % G;
  const float2 info = p.list_info[list];
  const int n_c = __float_as_int(info.x);
  if (n_c < 0) return;
  if (threadIdx.x == 0) {
    const RowStat st = p.stats[(int64_t)row * G + g];
    s.stat[g] = st;
    s.sM[g] = st.M;
    s.sInv[g] = st.invZ;
    s.n_band = s.n_above = 0;
  }
  __syncthreads();
  select_list<DT>(p, s, bitmap, row, g, g + 1, p.cand_score + (int64_t)list * p.cs_pitch,
                  p.cand_pos + (int64_t)list * p.cs_pitch, n_c, info.y, true,
                  p.kept_idx + (int64_t)row * (p.S + G * p.k + p.W) + g * p.k);
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
  // the bitmap (one bit per candidate, up to 128 KiB) sits next to about 25 KiB of static LDS; a CU has 160 KiB
  const size_t lds = (size_t)((E + 31) / 32) * 4;
  if (lds > 128 * 1024 || p.geo.G > kFastMaxG) return hipErrorInvalidValue;
  static uint64_t done_one = 0, done_pq = 0;
  const hipError_t e = p.n_lists > 1
                           ? allow_dynamic_lds((const void*)topk_cand_pq_kernel<DT_BF16>, 128 * 1024, &done_pq)
                           : allow_dynamic_lds((const void*)topk_cand_kernel<DT_BF16>, 128 * 1024, &done_one);
  if (e != hipSuccess) return e;
  if (p.n_lists > 1) {
    hipLaunchKernelGGL(cand_split_pq_kernel<DT_BF16>, dim3((unsigned)rows), dim3(kTopkThreads), 0, s, p);
    hipLaunchKernelGGL(topk_cand_pq_kernel<DT_BF16>, dim3((unsigned)(rows * p.n_lists)), dim3(kTopkThreads), lds, s, p);
  } else {
    hipLaunchKernelGGL(topk_cand_kernel<DT_BF16>, dim3((unsigned)rows), dim3(kTopkThreads), lds, s, p);
  }
  return hipGetLastError();
}

}  // namespace sagekv
