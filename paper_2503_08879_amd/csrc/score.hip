// Eviction pass, scoring stage (paper Sec. 2 Step 2: attention scores of the last token's
// query against the cached keys).
//
//   score_kernel (fp32), score_mfma_kernel (bf16)
//                   stream K once: logit[g][i] = q[g].K[i]/sqrt(d) for the G heads of a row.  What a
//                   pass leaves behind depends on its mode (ScoreMode): fp32 logits + per-chunk softmax
//                   partials (max, sum exp) for the one-sweep dense path; partials + the records of
//                   the tokens that pass the sample threshold (pre-filtered path); partials only, or
//                   every token's score from known (M, Z) (two-sweep dense path: rows the pre-filter
//                   could not certify, without a logit scratch).
//   sample_logits_kernel  logits of the sampled blocks of the pre-filtered path.
//   stats_kernel    merges the partials of a row into (M, Z) per head, in fp64.
//   combine_kernel  score[i] = sum_g exp(logit[g][i] - M_g) / Z_g  (fp32) and the first radix
//                   histogram of the candidates' scores, merged across workgroups with atomics.
#include "device_utils.h"
#include "kernels.h"
#include "radix_select.h"

namespace sagekv {

namespace {

constexpr int kScoreThreads = 256;
constexpr int kScoreWaves = kScoreThreads / kWave;
constexpr int kGatedRowBlocks = 16;  // y-blocks of a gated score / combine launch
constexpr int kBlocksPerWave = kScoreChunk / (kScoreWaves * 64);  // 64-token blocks per wave

// Logit scratch layout: [row][chunk][head][kScoreChunk], so a score workgroup writes one
// contiguous block and the combine stage still reads 16 bytes per head per thread.
__device__ __forceinline__ int64_t logit_index(const RowGeom& geo, int n_chunks, int row, int g, int64_t tok) {
  const int64_t chunk = tok / kScoreChunk;
  return (((int64_t)row * n_chunks + chunk) * geo.G + g) * kScoreChunk + (tok - chunk * kScoreChunk);
}

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
        const int64_t off = kv_offset(p.pm, p.pm.ks_page, p.ks_problem, p.ks_head, p.ks_token, prob, c, tok);
        kv[i] = ld16((const char*)p.K + off * EB + cl * 16);
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
        p.logits[logit_index(p.geo, p.n_chunks, row, p.g0 + g, tok)] = x;
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

// exp(l - m) for a term the softmax sum takes with an fp64 exponent (ScoreParams::heavy_thr): the logit of
// the head whose query row is qrow (bf16, D elements) and of token t of the wave's staged block
// (16-byte chunks, XOR-swizzled as the staging loop wrote them) is recomputed in fp64.  Called by all 64
// lanes of the wave with the same arguments (two elements per lane); every lane gets the result.
// Rare: out of line.
template <int D>
__device__ __noinline__ float heavy_term(const uint4* buf, int t, const uint32_t* qrow, float m) {
  constexpr int CH = D / 8;
  const int lane = threadIdx.x & 63;
  double acc = 0.0;
  if (lane < D / 2) {
    const int kk = lane >> 2;  // 16-byte chunk of elements 2 * lane, 2 * lane + 1
    const uint32_t kw = reinterpret_cast<const uint32_t*>(&buf[t * CH + (kk ^ (t & (CH - 1)))])[lane & 3];
    const uint32_t qw = qrow[lane];
    acc = (double)__uint_as_float(kw << 16) * (double)__uint_as_float(qw << 16) +
          (double)__uint_as_float(kw & 0xFFFF0000u) * (double)__uint_as_float(qw & 0xFFFF0000u);
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o);
  return (float)exp(acc / sqrt((double)D) - (double)m);
}


// bf16 scoring on the matrix cores.  The dot products of a 16-token tile against the group's
// query heads are one 16x16x(head_dim) product: A = queries (heads in rows, zero padded),
// B = keys (tokens in columns), fp32 accumulate.  MFMA operands want a lane to hold 8
// consecutive elements of ONE token per column lane, while coalesced loads give adjacent lanes
// adjacent 16-byte chunks of the SAME token, so each wave stages its 64-token block through a
// private, XOR-swizzled LDS buffer (conflict free both ways).  GPAD = heads padded to 4, 8 or
// 16: 16/GPAD tiles share an accumulator (the queries of tile t sit in rows t*GPAD..), so after
// a block every lane owns 4 logits and all stores are coalesced.
//
// MODE (ScoreMode) says what the pass leaves behind:
//   SCORE_LOGITS    every logit, to the scratch of the one-sweep dense path, and the softmax partials;
//   SCORE_FILTER    the pre-filtered path: nothing is written per token.  A lane keeps its logits only for
//                   tokens whose approximate score (sample statistics) reaches the row's conservative
//                   threshold, and appends (index, logits) to the chunk's candidate slots, or, once those
//                   are used up, to the row's overflow pool;
//   SCORE_PARTIALS  the softmax partials only;
//   SCORE_SCORES    with (M, Z) of every head known: every token's score (summed over the group, or one
//                   row per head), and the first radix histogram of the candidates' scores.
//
// PAGED: the chunk's pages (at most 64: pages hold 16 tokens or more) are looked up once, one per
// lane, and every load takes its page from the lane that holds it.
// One score chunk (kScoreChunk tokens of row `row`) by one workgroup of kScoreThreads threads.
template <int D, int GPAD, int MODE, bool PAGED>
__device__ __forceinline__ void score_mfma_chunk(const ScoreParams& p, int gb, int row, int chunk) {
  constexpr int CH = D / 8;         // 16-byte chunks per token
  constexpr int TPL = 64 / CH;      // tokens per coalesced wave load
  constexpr int NLOAD = 64 / TPL;   // loads per 64-token block
  constexpr int KSTEPS = D / 32;    // MFMA k-steps per tile
  constexpr int TILES = 16 / GPAD;  // 16-token tiles per accumulator
  constexpr int NACC = 4 / TILES;   // accumulators per block
  constexpr bool FILTER = MODE == SCORE_FILTER;
  constexpr bool KEEP = MODE == SCORE_LOGITS || MODE == SCORE_SCORES;  // per-token values held to the end
  constexpr bool PARTIALS = MODE != SCORE_SCORES;

  __shared__ uint4 lds[kScoreWaves][64 * CH];
  __shared__ float2 part[kScoreWaves][4][4];
  __shared__ int n_kept_wg;  // FILTER: candidates this workgroup has kept so far

  const int prob = row / p.geo.Hkv, c = row % p.geo.Hkv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int tq = lane / CH, cl = lane % CH;  // load role: token sub-index, chunk
  const int n = lane & 15, j = lane >> 4;    // MFMA role: column (token), k-group / row block
  const int64_t L = p.geo.L;
  uint4* buf = lds[wave];

  const char* Krow = (const char*)p.K + ((int64_t)prob * p.ks_problem + (int64_t)c * p.ks_head) * 2;
  const int64_t tok_bytes = p.ks_token * 2;
  int my_page = 0, first_page = 0;
  if (PAGED) {
    Krow = (const char*)p.K + (int64_t)c * p.ks_head * 2;
    first_page = (int)(((int64_t)chunk * kScoreChunk) >> p.pm.shift);
    const int last_page = (int)((L - 1) >> p.pm.shift);
    const int pg = first_page + lane < last_page ? first_page + lane : last_page;
    my_page = page_of(p.pm, prob, (int64_t)pg << p.pm.shift);
  }
  // address of this lane's 16 bytes of token tok (every lane of the wave calls it together)
  auto k_addr = [&](int64_t tok) -> const char* {
    if (PAGED) {
      const int pid = __shfl(my_page, (int)(tok >> p.pm.shift) - first_page);
      return Krow + ((int64_t)pid * p.pm.ks_page * 2 + (tok & ((1 << p.pm.shift) - 1)) * tok_bytes) + cl * 16;
    }
    return Krow + tok * tok_bytes + cl * 16;
  };

  // The waves of a workgroup take the chunk's 64-token blocks round robin, so the workgroup reads
  // one contiguous 64 KiB run at a time; the first block's loads go out before anything else.
  const int64_t wave_base = (int64_t)chunk * kScoreChunk + (int64_t)wave * 64;
  constexpr int64_t kBlockStride = 64 * kScoreWaves;
  uint4 kv[NLOAD];
  if (wave_base < L) {
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
      int64_t tok = wave_base + i * TPL + tq;
      tok = tok < L ? tok : L - 1;  // tail: re-read the last token, masked below
      kv[i] = ld16_stream(k_addr(tok));
    }
  }
  // A operand: lane (row m = n, k-group j) holds q[head m % GPAD][8*(4*kc + j) ..+8]
  const int my_head = n % GPAD, my_slot = n / GPAD;
  uint4 qa[KSTEPS];
#pragma unroll
  for (int kc = 0; kc < KSTEPS; ++kc) {
    qa[kc] = make_uint4(0u, 0u, 0u, 0u);
    if (my_head < gb) {
      const int h = c * p.geo.G + p.g0 + my_head;
      qa[kc] = ld16((const char*)p.q_last + (((int64_t)prob * p.geo.Hq + h) * D + (4 * kc + j) * 8) * 2);
    }
  }

  // each lane ends up with the logits of heads hbase .. hbase+3
  const int hbase = (4 * j) % GPAD;
  float m[4], sum[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    m[r] = -INFINITY;
    sum[r] = 0.f;
  }

  // softmax weights of this lane's 4 heads: the sample's (M^, 1/Z^) for the filter, the exact (M, 1/Z)
  // for the scores; the row's filter threshold(s)
  float fM[4] = {0.f, 0.f, 0.f, 0.f}, fInv[4] = {0.f, 0.f, 0.f, 0.f}, ftau = 0.f;
  // terms with an fp64 exponent (ScoreParams::heavy_thr): the passes that follow a sample stage; the
  // one-sweep dense pass (SCORE_LOGITS) leaves them to stats_exact_kernel
  constexpr bool HEAVY = MODE == SCORE_FILTER || MODE == SCORE_PARTIALS;
  float hthr[4] = {INFINITY, INFINITY, INFINITY, INFINITY};
  if (HEAVY && p.heavy_thr) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (hbase + r < gb) hthr[r] = p.heavy_thr[(int64_t)row * p.geo.G + p.g0 + hbase + r];
  }
  const uint32_t* q_group = reinterpret_cast<const uint32_t*>(
      (const char*)p.q_last + (((int64_t)prob * p.geo.Hq + c * p.geo.G + p.g0) * D) * 2);  // query rows of this launch's heads
  float ftau_h[4] = {INFINITY, INFINITY, INFINITY, INFINITY};  // per-query lists: a threshold per head
  const bool per_head = FILTER && p.filt.n_lists > 1;
  if (FILTER) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (hbase + r < gb) {
        const float2 st = p.filt.samp_stats[(int64_t)row * p.geo.G + hbase + r];
        fM[r] = st.x;
        fInv[r] = st.y;
        if (per_head) ftau_h[r] = p.filt.samp_tau[(int64_t)row * p.geo.G + hbase + r];
      }
    if (!per_head) ftau = p.filt.samp_tau[row];
    if (threadIdx.x == 0) n_kept_wg = 0;
    __syncthreads();
  }
  if (MODE == SCORE_SCORES) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (hbase + r < gb) {
        const RowStat st = p.stats[(int64_t)row * p.geo.G + p.g0 + hbase + r];
        fM[r] = st.M;
        fInv[r] = st.invZ;
      }
  }
  // FILTER: this chunk's own candidate slots, and the row's overflow pool behind all chunks' slots
  const int64_t row_slots = (int64_t)row * p.filt.slots_per_row;
  const int64_t slot_base = row_slots + (int64_t)chunk * p.filt.cap_c;
  const int64_t ovf_base = row_slots + (int64_t)p.n_chunks * p.filt.cap_c;

  // Software pipeline: the loads of block b+1 are issued right after block b went to LDS, so
  // their latency overlaps block b's MFMA phase.  Per-token results stay in registers until the wave
  // has loaded its last block: loads and stores share one in-order completion counter, so a
  // store inside the loop would put its write-ack latency on the critical path of every block.
  float xs[KEEP ? kBlocksPerWave : 1][NACC][4];
#pragma unroll
  for (int blk = 0; blk < kBlocksPerWave; ++blk) {
    const int64_t tok_base = wave_base + (int64_t)blk * kBlockStride;
    if (tok_base < L) {  // wave-uniform
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");  // previous block's LDS reads are done
#pragma unroll
      for (int i = 0; i < NLOAD; ++i) {
        const int t = i * TPL + tq;
        buf[t * CH + (cl ^ (t & (CH - 1)))] = kv[i];
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      if (blk + 1 < kBlocksPerWave && tok_base + kBlockStride < L) {
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) {
          int64_t tok = tok_base + kBlockStride + i * TPL + tq;
          tok = tok < L ? tok : L - 1;
          kv[i] = ld16_stream(k_addr(tok));
        }
      }
      f32x4_t acc[NACC];
#pragma unroll
      for (int a = 0; a < NACC; ++a) {
        acc[a] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ts = 0; ts < TILES; ++ts) {
          const int t = (a * TILES + ts) * 16 + n;
#pragma unroll
          for (int kc = 0; kc < KSTEPS; ++kc) {
            const uint4 b = buf[t * CH + ((4 * kc + j) ^ (n & (CH - 1)))];
            const uint4 qv = (my_slot == ts) ? qa[kc] : make_uint4(0u, 0u, 0u, 0u);
            acc[a] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, qv),
                                                             __builtin_bit_cast(bf16x8_t, b), acc[a], 0, 0, 0);
          }
        }
      }
      // lane (j, n), accumulator a, register r: row 4j + r = (tile slot, head), column n = token
      bool any_heavy = false;
#pragma unroll
      for (int a = 0; a < NACC; ++a) {
        const int64_t tok = tok_base + (a * TILES + (4 * j) / GPAD) * 16 + n;
        float approx = 0.f;
        int any_head = 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float x = acc[a][r] * p.scale;
          xs[KEEP ? blk : 0][a][r] = x;
          if (tok < L && hbase + r < gb) {
            if (PARTIALS) {
              const float mn = fmaxf(m[r], x);
              const bool hv = HEAVY && x >= hthr[r];  // rare: its term is added below, with an fp64 exponent
              any_heavy |= hv;
              sum[r] = sum[r] * exp_fast(m[r] - mn) + (hv ? 0.f : exp_fast(x - mn));
              m[r] = mn;
            }
            if (FILTER) {
              const float pr = exp_fast(x - fM[r]) * fInv[r];
              approx += pr;
              any_head |= !(pr < ftau_h[r]);
            }
            if (MODE == SCORE_SCORES) xs[KEEP ? blk : 0][a][r] = exp_times(x - fM[r], fInv[r]);
          } else if (MODE == SCORE_SCORES) {
            xs[KEEP ? blk : 0][a][r] = 0.f;
          }
        }
        if (FILTER) {
          // the heads of a token sit in GPAD/4 lanes (same n, adjacent j): combine their parts
          if (GPAD >= 8) {
            approx += __shfl_xor(approx, 16);
            any_head |= __shfl_xor(any_head, 16);
          }
          if (GPAD >= 16) {
            approx += __shfl_xor(approx, 32);
            any_head |= __shfl_xor(any_head, 32);
          }
          const bool reach = per_head ? any_head != 0 : !(approx < ftau);
          const bool pass = tok >= p.filt.S && tok < L - p.filt.W && reach;
          const bool rep = (4 * j) % GPAD == 0;  // one lane per token counts it
          const unsigned long long bal = __ballot(pass && rep);
          if (bal) {  // wave-uniform
            int base = 0;
            if (lane == 0) base = atomicAdd(&n_kept_wg, __popcll(bal));  // LDS counter
            base = __shfl(base, 0);
            int pos = base + __popcll(bal & ((1ull << lane) - 1ull));
            const int src = ((j - j % (GPAD / 4)) << 4) | n;  // the token's counting lane
            pos = __shfl(pos, src);                           // every lane of the token
            int64_t slot = slot_base + pos;
            if (base + __popcll(bal) > p.filt.cap_c) {  // wave-uniform, rare: the chunk's own slots are used up
              int o = 0;
              if (pass && rep && pos >= p.filt.cap_c) o = atomicAdd(&p.filt.ovf_count[row], 1);
              o = __shfl(o, src);
              if (pos >= p.filt.cap_c) slot = o < p.filt.cap_o ? ovf_base + o : -1;  // pool full: dropped, the row is redone
            }
            if (pass && hbase < gb && slot >= 0) {
              if (rep) p.filt.cand_idx[slot] = (int32_t)tok;
              float* rec = p.filt.cand_logit + slot * p.filt.Gs + hbase;
              *reinterpret_cast<float4*>(rec) = make_float4(xs[0][a][0], xs[0][a][1], xs[0][a][2], xs[0][a][3]);
            }
          }
        }
      }
      if (HEAVY && __any(any_heavy)) {  // wave-uniform, rare: the wave takes its heavy terms one at a time
#pragma unroll
        for (int a = 0; a < NACC; ++a) {
          const int t_local = (a * TILES + (4 * j) / GPAD) * 16 + n;
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            unsigned long long todo = __ballot(tok_base + t_local < L && hbase + r < gb && xs[0][a][r] >= hthr[r]);
            while (todo) {
              const int src = __ffsll((long long)todo) - 1;  // the lane that holds this (token, head)
              todo &= todo - 1;
              const int js = src >> 4, ns = src & 15;
              const int t_src = (a * TILES + (4 * js) / GPAD) * 16 + ns;
              const int h_src = (4 * js) % GPAD + r;
              const float term = heavy_term<D>(buf, t_src, q_group + (int64_t)h_src * (D / 2), __shfl(m[r], src));
              if (lane == src) sum[r] += term;
            }
          }
        }
      }
    }
  }
  if (MODE == SCORE_LOGITS) {
#pragma unroll
    for (int blk = 0; blk < kBlocksPerWave; ++blk) {
#pragma unroll
      for (int a = 0; a < NACC; ++a) {
        const int64_t tok = wave_base + (int64_t)blk * kBlockStride + (a * TILES + (4 * j) / GPAD) * 16 + n;
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (tok < L && hbase + r < gb)
            p.logits[logit_index(p.geo, p.n_chunks, row, p.g0 + hbase + r, tok)] = xs[KEEP ? blk : 0][a][r];
      }
    }
  }
  if (MODE == SCORE_SCORES) {
    // xs holds exp(l - M) / Z of this lane's heads.  One list per row: the group's sum (the lanes that
    // share a token add up, ascending heads within a lane); one list per head: each value is a score.
    __shared__ int hist[kHistBins];
    const bool per_q = p.n_lists > 1;
    const bool rep = (4 * j) % GPAD == 0;
    const int64_t cand_lo = p.S, cand_hi = L - p.W;
    if (!per_q) {
#pragma unroll
      for (int blk = 0; blk < kBlocksPerWave; ++blk)
#pragma unroll
        for (int a = 0; a < NACC; ++a) {
          float v = (xs[KEEP ? blk : 0][a][0] + xs[KEEP ? blk : 0][a][1]) + (xs[KEEP ? blk : 0][a][2] + xs[KEEP ? blk : 0][a][3]);
          if (GPAD >= 8) v += __shfl_xor(v, 16);
          if (GPAD >= 16) v += __shfl_xor(v, 32);
          xs[KEEP ? blk : 0][a][0] = v;
        }
    }
    const int n_pass = per_q ? gb : 1;  // histogram passes: one list at a time through the LDS histogram
    for (int li = 0; li < n_pass; ++li) {
      for (int b = threadIdx.x; b < kHistBins; b += kScoreThreads) hist[b] = 0;
      __syncthreads();
      const int64_t list = (int64_t)row * p.n_lists + (per_q ? p.g0 + li : 0);
      float* out = p.scores + list * p.pitch;
      // the lane that holds this list's value of a token: the counting lane (sum), or head li's lane and register
      const bool mine = per_q ? (hbase <= li && li < hbase + 4) : rep;
      const int r_sel = per_q ? (li - hbase) & 3 : 0;
#pragma unroll
      for (int blk = 0; blk < kBlocksPerWave; ++blk)
#pragma unroll
        for (int a = 0; a < NACC; ++a) {
          const int64_t tok = wave_base + (int64_t)blk * kBlockStride + (a * TILES + (4 * j) / GPAD) * 16 + n;
          float v = xs[KEEP ? blk : 0][a][0];
          if (per_q) {
            v = r_sel == 1 ? xs[KEEP ? blk : 0][a][1] : v;
            v = r_sel == 2 ? xs[KEEP ? blk : 0][a][2] : v;
            v = r_sel == 3 ? xs[KEEP ? blk : 0][a][3] : v;
          }
          if (mine && tok < L) {
            out[tok] = v;
            if (tok >= cand_lo && tok < cand_hi) atomicAdd(&hist[(__float_as_uint(v) >> 20) & (kHistBins - 1)], 1);
          }
        }
      __syncthreads();
      int* gh = p.ghist + list * kHistBins;
      for (int b = threadIdx.x; b < kHistBins; b += kScoreThreads) {
        const int v = hist[b];
        if (v) atomicAdd(&gh[b], v);
      }
      __syncthreads();
    }
    return;
  }

  // (max, sum) of the chunk: the 16 lanes of a row block share their heads
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    float M = m[r];
#pragma unroll
    for (int o = 8; o >= 1; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));
    float sm = (m[r] == -INFINITY) ? 0.f : sum[r] * exp_fast(m[r] - M);
    sm = group_sum<16>(sm);
    if (n == 0) part[wave][j][r] = make_float2(M, sm);
  }
  __syncthreads();
  if (FILTER && threadIdx.x == 0) p.filt.cand_count[(int64_t)row * p.n_chunks + chunk] = n_kept_wg;
  if ((int)threadIdx.x < gb) {
    const int g = threadIdx.x;
    float M = -INFINITY;
    for (int w = 0; w < kScoreWaves; ++w)
      for (int jj = 0; jj < 4; ++jj)
        if ((4 * jj) % GPAD == (g / 4) * 4) M = fmaxf(M, part[w][jj][g % 4].x);
    float sm = 0.f;
    for (int w = 0; w < kScoreWaves; ++w)
      for (int jj = 0; jj < 4; ++jj)
        if ((4 * jj) % GPAD == (g / 4) * 4) {
          const float2 pw = part[w][jj][g % 4];
          sm += (pw.x == -INFINITY) ? 0.f : pw.y * exp_fast(pw.x - M);
        }
    p.partials[((int64_t)row * p.geo.G + p.g0 + g) * p.n_chunks + chunk] = make_float2(M, sm);
  }
}

// grid (chunks, rows).  A gated launch (rows the pre-filter could not certify, usually none) has a
// few y-blocks only, each walking over all rows and working on the flagged ones: an empty launch
// then costs a handful of workgroups instead of one per (chunk, row).
template <int D, int GPAD, int MODE, bool PAGED>
__global__ __launch_bounds__(kScoreThreads) void score_mfma_kernel(ScoreParams p, int gb) {
  if (MODE != SCORE_FILTER && p.gate.row_flag) {
    if (*p.gate.n_flagged == 0) return;  // the usual case: nothing to redo
    const int rows = p.geo.n_problems * p.geo.Hkv;
    for (int row = blockIdx.y; row < rows; row += gridDim.y) {
      if (p.gate.row_flag[row] == 0) continue;  // workgroup-uniform
      score_mfma_chunk<D, GPAD, MODE, PAGED>(p, gb, row, (int)blockIdx.x);
      __syncthreads();  // the chunk's last LDS reads, before the next row's writes
    }
    return;
  }
  score_mfma_chunk<D, GPAD, MODE, PAGED>(p, gb, (int)blockIdx.y, (int)blockIdx.x);
}

// Logits of the sampled blocks (fast path), same MFMA scheme as score_mfma_kernel: one wave per
// 64-token block, logits to samp_logit[row][slot][Gs] (16 bytes per lane).
template <int D, int GPAD>
__global__ __launch_bounds__(kScoreThreads) void sample_logits_kernel(SampleParams p) {
  constexpr int CH = D / 8, TPL = 64 / CH, NLOAD = 64 / TPL, KSTEPS = D / 32;
  constexpr int TILES = 16 / GPAD, NACC = 4 / TILES;
  __shared__ uint4 lds[kScoreWaves][64 * CH];

  const int row = blockIdx.y;
  const int prob = row / p.geo.Hkv, c = row % p.geo.Hkv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int tq = lane / CH, cl = lane % CH;
  const int n = lane & 15, j = lane >> 4;
  const int64_t L = p.geo.L;
  const int G = p.geo.G;
  const int blk = blockIdx.x * kScoreWaves + wave;
  if (blk >= p.nA + p.nB + p.nC) return;  // wave-uniform; no workgroup barrier below
  uint4* buf = lds[wave];
  uint4 kv[NLOAD];
#pragma unroll
  for (int i = 0; i < NLOAD; ++i) {
    int64_t tok = sample_token(p, blk, i * TPL + tq);
    tok = tok < 0 ? 0 : (tok < L ? tok : L - 1);
    const int64_t off = kv_offset(p.pm, p.pm.ks_page, p.ks_problem, p.ks_head, p.ks_token, prob, c, tok);
    kv[i] = ld16((const char*)p.K + off * 2 + cl * 16);
  }
  const int my_head = n % GPAD, my_slot = n / GPAD;
  uint4 qa[KSTEPS];
#pragma unroll
  for (int kc = 0; kc < KSTEPS; ++kc) {
    qa[kc] = make_uint4(0u, 0u, 0u, 0u);
    if (my_head < G) {
      const int h = c * G + my_head;
      qa[kc] = ld16((const char*)p.q_last + (((int64_t)prob * p.geo.Hq + h) * D + (4 * kc + j) * 8) * 2);
    }
  }
#pragma unroll
  for (int i = 0; i < NLOAD; ++i) {
    const int t = i * TPL + tq;
    buf[t * CH + (cl ^ (t & (CH - 1)))] = kv[i];
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  const int hbase = (4 * j) % GPAD;
  float* out = p.samp_logit + ((int64_t)row * (p.nA + p.nB + p.nC) + blk) * 64 * p.Gs;
#pragma unroll
  for (int a = 0; a < NACC; ++a) {
    f32x4_t acc = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ts = 0; ts < TILES; ++ts) {
      const int t = (a * TILES + ts) * 16 + n;
#pragma unroll
      for (int kc = 0; kc < KSTEPS; ++kc) {
        const uint4 b = buf[t * CH + ((4 * kc + j) ^ (n & (CH - 1)))];
        const uint4 qv = (my_slot == ts) ? qa[kc] : make_uint4(0u, 0u, 0u, 0u);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, qv), __builtin_bit_cast(bf16x8_t, b),
                                                      acc, 0, 0, 0);
      }
    }
    const int t_local = (a * TILES + (4 * j) / GPAD) * 16 + n;
    if (hbase < p.Gs)
      *reinterpret_cast<float4*>(out + (int64_t)t_local * p.Gs + hbase) =
          make_float4(acc[0] * p.scale, acc[1] * p.scale, acc[2] * p.scale, acc[3] * p.scale);
  }
}

__global__ __launch_bounds__(64) void stats_kernel(StatsParams p) {
  const int lane = threadIdx.x, row = blockIdx.x;
  if (p.ghist)
    for (int b = lane; b < kHistBins * p.n_lists; b += 64) p.ghist[(int64_t)row * p.n_lists * kHistBins + b] = 0;
  for (int g = 0; g < p.G; ++g) {
    const RowStat st = merge_partials_wave(p.partials + ((int64_t)row * p.G + g) * p.n_chunks, p.n_chunks);
    if (lane == 0) p.stats[(int64_t)row * p.G + g] = st;
  }
}

// One-sweep dense path: every token's fp32 logit is in scratch, so a head's normaliser is summed from
// there once its maximum is known: Z = sum_i exp(l_i - M) in fp64, the terms heavy enough for their
// logit's fp32 error to show in Z (heavy_logit_threshold) with the logit recomputed in fp64 from K.
// (The pre-filtered and two-sweep paths do the same inside the score kernel, with a threshold from
// the sample; here nothing is known about the row before the sweep.)  One workgroup per row.
constexpr int kMaxHeavy = 4096;  // heavy terms per (row, head) taken exactly; beyond: as fp32 terms

template <int DT>
__global__ __launch_bounds__(kTopkThreads) void stats_exact_kernel(ExactStatsParams p) {
  __shared__ double red_d[kTopkWaves];
  __shared__ RowStat s_stat[64];  // up to 64 heads per KV head
  __shared__ float s_thr[64];
  __shared__ int heavy_tok[kMaxHeavy];
  __shared__ int n_heavy;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, row = blockIdx.x;
  const int G = p.geo.G, D = p.geo.D;
  const int prob = row / p.geo.Hkv, c = row % p.geo.Hkv;
  const int64_t L = p.geo.L;
  for (int b = tid; b < kHistBins * p.n_lists; b += kTopkThreads) p.ghist[(int64_t)row * p.n_lists * kHistBins + b] = 0;
  // the chunks' maxima and fp32 sums, one wave per head: M, and a Z that stands unless the head has heavy terms
  for (int g = wave; g < G; g += kTopkWaves) {
    const RowStat st = merge_partials_wave(p.partials + ((int64_t)row * G + g) * p.n_chunks, p.n_chunks);
    if (lane == 0) {
      s_stat[g] = st;
      s_thr[g] = heavy_logit_threshold(st.M, (float)st.Z);
    }
  }
  __syncthreads();
  auto block_sum = [&](double v) -> double {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
    __syncthreads();  // red_d free
    if (lane == 0) red_d[wave] = v;
    __syncthreads();
    double t = 0.0;
    for (int w = 0; w < kTopkWaves; ++w) t += red_d[w];
    return t;
  };
  for (int g = 0; g < G; ++g) {
    const float M = s_stat[g].M, thr = s_thr[g];
    if (!(thr <= M)) continue;  // no term of this head is heavy enough (workgroup-uniform)
    __syncthreads();            // the previous head's list has been read
    if (tid == 0) n_heavy = 0;
    __syncthreads();
    // the row's logits of this head, four at a time (a chunk's kScoreChunk logits of a head are contiguous)
    double z = 0.0;
    for (int64_t t4 = (int64_t)tid * 4; t4 < L; t4 += 4 * kTopkThreads) {
      const float4 v = *reinterpret_cast<const float4*>(p.logits + logit_index(p.geo, p.n_chunks, row, g, t4));
      const float x[4] = {v.x, v.y, v.z, v.w};
      float part = 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (t4 + e >= L) break;
        bool exact = x[e] >= thr;
        if (exact) {
          const int i = atomicAdd(&n_heavy, 1);
          if (i < kMaxHeavy) heavy_tok[i] = (int)(t4 + e); else exact = false;
        }
        if (!exact) part += exp_fast(x[e] - M);
      }
      z += (double)part;
    }
    z = block_sum(z);  // (its barriers also publish heavy_tok)
    const int nh = n_heavy < kMaxHeavy ? n_heavy : kMaxHeavy;
    const double inv = 1.0 / sqrt((double)D);
    const int64_t q_off = ((int64_t)prob * p.geo.Hq + c * G + g) * D;
    double zh = 0.0;
    for (int i = wave; i < nh; i += kTopkWaves) {
      const int64_t k_off = kv_offset(p.pm, p.pm.ks_page, p.ks_problem, p.ks_head, p.ks_token, prob, c, heavy_tok[i]);
      double acc = 0.0;
      for (int jj = lane; jj < D; jj += 64) acc += elem_f64<DT>(p.q_last, q_off + jj) * elem_f64<DT>(p.K, k_off + jj);
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o);
      if (lane == 0) zh += exp(acc * inv - (double)M);
    }
    z += block_sum(zh);
    if (tid == 0) {
      s_stat[g].Z = z;
      s_stat[g].invZ = (float)(1.0 / z);
    }
  }
  __syncthreads();
  if (tid < G) p.stats[(int64_t)row * G + tid] = s_stat[tid];
}

constexpr int kCombineThreads = 256;
constexpr int kMaxG = 64;

__global__ __launch_bounds__(kCombineThreads) void combine_kernel(CombineParams p) {
  __shared__ int hist[kHistBins];
  __shared__ float sM[kMaxG], sInv[kMaxG];
  const int tid = threadIdx.x;
  const int row = blockIdx.y;
  const int G = p.geo.G;
  const int64_t L = p.geo.L;
  for (int b = tid; b < kHistBins; b += kCombineThreads) hist[b] = 0;
  if (tid < G) {
    RowStat st = p.stats[(int64_t)row * G + tid];
    sM[tid] = st.M;
    sInv[tid] = st.invZ;
  }
  __syncthreads();
  // group-sum: one score row per KV head; per-query: blockIdx.z picks the head, one row each
  const int g_lo = p.n_lists > 1 ? blockIdx.z : 0, g_hi = p.n_lists > 1 ? g_lo + 1 : G;
  const int64_t list = (int64_t)row * p.n_lists + (p.n_lists > 1 ? g_lo : 0);
  float* out = p.scores + list * p.pitch;
  const int64_t cand_lo = p.S, cand_hi = L - p.W;
  const bool vec_out = (p.pitch & 3) == 0;
  const int64_t base = (int64_t)blockIdx.x * kCombineChunk;
#pragma unroll
  for (int it = 0; it < kCombineChunk / (kCombineThreads * 4); ++it) {
    const int64_t tok = base + (int64_t)it * kCombineThreads * 4 + tid * 4;
    if (tok >= L) break;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int g = g_lo; g < g_hi; ++g) {
      const float4 x = *reinterpret_cast<const float4*>(p.logits + logit_index(p.geo, p.n_chunks, row, g, tok));
      const float M = sM[g], inv = sInv[g];
      acc[0] += exp_times(x.x - M, inv);
      acc[1] += exp_times(x.y - M, inv);
      acc[2] += exp_times(x.z - M, inv);
      acc[3] += exp_times(x.w - M, inv);
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
  int* gh = p.ghist + list * kHistBins;
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

template <int D, int MODE, bool PAGED>
hipError_t launch_score_mfma_p(const ScoreParams& p, int gb, dim3 grid, hipStream_t s) {
  if (gb <= 4)
    hipLaunchKernelGGL((score_mfma_kernel<D, 4, MODE, PAGED>), grid, dim3(kScoreThreads), 0, s, p, gb);
  else if (gb <= 8)
    hipLaunchKernelGGL((score_mfma_kernel<D, 8, MODE, PAGED>), grid, dim3(kScoreThreads), 0, s, p, gb);
  else
    hipLaunchKernelGGL((score_mfma_kernel<D, 16, MODE, PAGED>), grid, dim3(kScoreThreads), 0, s, p, gb);
  return hipGetLastError();
}

template <int D, int MODE>
hipError_t launch_score_mfma(const ScoreParams& p, int gb, dim3 grid, hipStream_t s) {
  return p.pm.table ? launch_score_mfma_p<D, MODE, true>(p, gb, grid, s)
                    : launch_score_mfma_p<D, MODE, false>(p, gb, grid, s);
}

template <int MODE>
hipError_t launch_score_mfma_d(const ScoreParams& p, int gb, dim3 grid, hipStream_t s) {
  return p.geo.D == 128 ? launch_score_mfma<128, MODE>(p, gb, grid, s) : launch_score_mfma<64, MODE>(p, gb, grid, s);
}

}  // namespace

// Fast path: bf16, G <= 16 (one launch covers the group).
hipError_t launch_score_filter(const ScoreParams& p0, hipStream_t s) {
  const int rows = p0.geo.n_problems * p0.geo.Hkv;
  dim3 grid((unsigned)p0.n_chunks, (unsigned)rows);
  ScoreParams p = p0;
  p.g0 = 0;
  p.gate.row_flag = nullptr;
  if (p.geo.dtype != DT_BF16 || p.geo.G > 16) return hipErrorInvalidValue;
  return launch_score_mfma_d<SCORE_FILTER>(p, p.geo.G, grid, s);
}

hipError_t launch_sample_logits(const SampleParams& p, hipStream_t s) {
  const int rows = p.geo.n_problems * p.geo.Hkv;
  const int nb = p.nA + p.nB + p.nC;
  if (p.geo.dtype != DT_BF16 || p.geo.G > 16) return hipErrorInvalidValue;
  dim3 grid((unsigned)((nb + kScoreWaves - 1) / kScoreWaves), (unsigned)rows);
#define SAGEKV_LAUNCH(DD, GP) hipLaunchKernelGGL((sample_logits_kernel<DD, GP>), grid, dim3(kScoreThreads), 0, s, p)
  if (p.geo.D == 128) {
    if (p.geo.G <= 4) SAGEKV_LAUNCH(128, 4); else if (p.geo.G <= 8) SAGEKV_LAUNCH(128, 8); else SAGEKV_LAUNCH(128, 16);
  } else {
    if (p.geo.G <= 4) SAGEKV_LAUNCH(64, 4); else if (p.geo.G <= 8) SAGEKV_LAUNCH(64, 8); else SAGEKV_LAUNCH(64, 16);
  }
#undef SAGEKV_LAUNCH
  return hipGetLastError();
}

int max_group_per_launch() { return 8; }

// Dense passes.  bf16: any mode, gated or not; fp32 caches: SCORE_LOGITS over every row only.
hipError_t launch_score(const ScoreParams& p0, ScoreMode mode, hipStream_t s) {
  const int rows = p0.geo.n_problems * p0.geo.Hkv;
  const bool bf16 = p0.geo.dtype == DT_BF16;
  if (mode == SCORE_FILTER || (!bf16 && (mode != SCORE_LOGITS || p0.gate.row_flag))) return hipErrorInvalidValue;
  dim3 grid((unsigned)p0.n_chunks, (unsigned)(p0.gate.row_flag && rows > kGatedRowBlocks ? kGatedRowBlocks : rows));
  const int per_launch = bf16 ? 16 : max_group_per_launch();
  for (int g0 = 0; g0 < p0.geo.G; g0 += per_launch) {
    ScoreParams p = p0;
    p.g0 = g0;
    const int gb = p0.geo.G - g0 < per_launch ? p0.geo.G - g0 : per_launch;
    hipError_t e;
    if (!bf16)
      e = p.geo.D == 128 ? launch_score_g<DT_F32, 128>(p, gb, grid, s) : launch_score_g<DT_F32, 64>(p, gb, grid, s);
    else if (mode == SCORE_LOGITS)
      e = launch_score_mfma_d<SCORE_LOGITS>(p, gb, grid, s);
    else if (mode == SCORE_PARTIALS)
      e = launch_score_mfma_d<SCORE_PARTIALS>(p, gb, grid, s);
    else
      e = launch_score_mfma_d<SCORE_SCORES>(p, gb, grid, s);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_stats(const StatsParams& p, int rows, hipStream_t s) {
  hipLaunchKernelGGL(stats_kernel, dim3((unsigned)rows), dim3(64), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_stats_exact(const ExactStatsParams& p, hipStream_t s) {
  const int rows = p.geo.n_problems * p.geo.Hkv;
  if (p.geo.dtype == DT_BF16)
    hipLaunchKernelGGL(stats_exact_kernel<DT_BF16>, dim3((unsigned)rows), dim3(kTopkThreads), 0, s, p);
  else
    hipLaunchKernelGGL(stats_exact_kernel<DT_F32>, dim3((unsigned)rows), dim3(kTopkThreads), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_combine(const CombineParams& p, hipStream_t s) {
  const int rows = p.geo.n_problems * p.geo.Hkv;
  const unsigned nx = (unsigned)((p.geo.L + kCombineChunk - 1) / kCombineChunk);
  hipLaunchKernelGGL(combine_kernel, dim3(nx, (unsigned)rows, (unsigned)p.n_lists), dim3(kCombineThreads), 0, s, p);
  return hipGetLastError();
}

}  // namespace sagekv
