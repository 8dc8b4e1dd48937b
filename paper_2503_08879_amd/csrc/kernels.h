// Internal launch interface between the C ABI (api.hip) and the kernels.
// Host-side argument checks live in api.hip; launchers assume valid shapes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sagekv {

// Softmax statistics of one (row, query head of the group): row maximum of the fp32 logits and
// Z = sum_i exp(logit_i - M), combined in fp64 from per-chunk fp32 partial sums.
struct RowStat {
  float M;
  float invZ;
  double Z;
};

constexpr int kHistBins = 2048;      // first radix digit: key bits 30..20
constexpr int kScoreChunk = 1024;    // tokens one score workgroup covers
constexpr int kCombineChunk = 4096;  // tokens one combine workgroup covers

struct RowGeom {
  int n_problems, Hq, Hkv, G, D, dtype;
  int64_t L;
  int64_t Lp;  // pitch (floats) of the logit rows, multiple of 4
};

// Paged caches.  table = nullptr: the cache is one strided array and token t of (problem, head)
// sits at problem * s_problem + head * s_head + t * s_token (elements).  Otherwise a row's tokens
// are cut into pages of 2^shift tokens and page j of a problem is physical page
// table[problem * pitch + j] of a pool: page * s_page + head * s_head + (t mod 2^shift) * s_token.
// Table entries are clamped to [0, n_pages) before use.
struct PageMap {
  const int32_t* table;
  int64_t pitch;
  int64_t ks_page, vs_page;  // elements between pages of the K pool, of the V pool
  int shift;
  int n_pages;
};

__device__ __forceinline__ int page_of(const PageMap& pm, int prob, int64_t tok) {
  const int pid = pm.table[(int64_t)prob * pm.pitch + (tok >> pm.shift)];
  return pid < 0 ? 0 : (pid >= pm.n_pages ? pm.n_pages - 1 : pid);
}

// Element offset of token tok of (prob, head c) in K (or, with the V strides, in V).
__device__ __forceinline__ int64_t kv_offset(const PageMap& pm, int64_t s_page, int64_t s_problem, int64_t s_head,
                                             int64_t s_token, int prob, int c, int64_t tok) {
  if (!pm.table) return (int64_t)prob * s_problem + (int64_t)c * s_head + tok * s_token;
  return (int64_t)page_of(pm, prob, tok) * s_page + (int64_t)c * s_head + (tok & ((1 << pm.shift) - 1)) * s_token;
}

// One row of the reduced cache, K or V: dense [cap][D] elements, or spread over pages of a pool (a
// page holds [Hkv][2^shift][D] elements).  at(t) = address of logical token t of the row.
struct CacheRow {
  char* base;          // dense: the row's first token; paged: the pool, advanced to the row's KV head
  const int32_t* tab;  // paged: the problem's row of the block table, else null
  int64_t page_bytes;
  int shift, n_pages, rowb;
  __device__ __forceinline__ char* at(int tok) const {
    if (!tab) return base + (int64_t)tok * rowb;
    int pid = tab[tok >> shift];
    pid = pid < 0 ? 0 : (pid >= n_pages ? n_pages - 1 : pid);
    return base + (int64_t)pid * page_bytes + (int64_t)(tok & ((1 << shift) - 1)) * rowb;
  }
};
// The same with the layout fixed at compile time (the bf16 decode kernels: a run-time choice in
// their load addresses costs them 9 % at 256 rows x 4096 tokens).
template <bool PAGED, int ROWB>
struct CacheRowT {
  CacheRow r;
  __device__ __forceinline__ char* at(int tok) const {
    if (!PAGED) return r.base + (int64_t)tok * ROWB;
    int pid = r.tab[tok >> r.shift];
    pid = pid < 0 ? 0 : (pid >= r.n_pages ? r.n_pages - 1 : pid);
    return r.base + (int64_t)pid * r.page_bytes + (int64_t)(tok & ((1 << r.shift) - 1)) * ROWB;
  }
};
__device__ __forceinline__ CacheRow cache_row(void* cache, const PageMap& cpm, bool v, int prob, int c, int row, int cap,
                                              int rowb, int eb /* bytes per element */) {
  CacheRow r;
  r.rowb = rowb;
  if (!cpm.table) {
    r.base = (char*)cache + (int64_t)row * cap * rowb;
    r.tab = nullptr;
    r.page_bytes = 0;
    r.shift = r.n_pages = 0;
  } else {
    r.base = (char*)cache + ((int64_t)c << cpm.shift) * rowb;
    r.tab = cpm.table + (int64_t)prob * cpm.pitch;
    r.page_bytes = (v ? cpm.vs_page : cpm.ks_page) * (int64_t)eb;
    r.shift = cpm.shift;
    r.n_pages = cpm.n_pages;
  }
  return r;
}

// Raises a kernel's dynamic LDS limit once per device (the attribute belongs to the device's copy of
// the kernel).  `done`: one bit per device, file-scope state of the caller.  Two host threads racing
// here at worst set the attribute twice.
inline hipError_t allow_dynamic_lds(const void* kernel, int bytes, uint64_t* done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 64 && ((*done >> dev) & 1ull)) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess && dev < 64) *done |= 1ull << dev;
  return e;
}

// Rows a gated launch works on: those whose flag is nonzero (device memory, one int per row; set by
// the pre-filtered path for the rows it could not certify).  Null = every row.  A gated launch has a
// few row blocks that walk over all rows and skip the unflagged ones, so a launch with nothing to
// do costs a handful of workgroups.
struct RowGate {
  const int* row_flag;
  const int* n_flagged;  // how many flags are set (one int): a gated launch looks here first
};

// Candidate pre-filter of the fast eviction path.  A strided sample of the row gives approximate
// softmax statistics and a conservative score threshold; the streaming score pass then keeps
// only the tokens whose approximate score passes it (index + exact fp32 logits), instead of
// writing every token's logits.
struct FilterParams {
  const float2* samp_stats;  // [rows][G]  (M^, 1/Z^) from the sample
  const float* samp_tau;     // [rows * n_lists] threshold on the approximate score (per head if n_lists = G)
  int n_lists;               // 1: the group's summed score is compared; G: a token passes if ANY head's
                             //    own probability reaches that head's threshold
  // Candidate records (token index + exact fp32 logits of the Gs heads).  Each score workgroup owns
  // cap_c slots for its chunk (an LDS counter hands them out: no global atomics); a chunk that keeps
  // more spills into the row's overflow pool of cap_o slots through one global counter per row.
  // Row r: slots [r * slots_per_row, +n_chunks * cap_c) by chunk, then cap_o overflow slots.
  int* cand_count;           // [rows][n_chunks]  tokens each chunk kept (may exceed cap_c: the rest overflowed)
  int* ovf_count;            // [rows]            tokens sent to the overflow pool (may exceed cap_o: dropped,
                             //                   the row then has more candidates than planned and is redone)
  int32_t* cand_idx;         // [rows][slots_per_row]
  float* cand_logit;         // [rows][slots_per_row][Gs]
  int cap_c, cap_o;
  int64_t slots_per_row;
  int Gs;
  int S, W;
};

// What a pass over K leaves behind.
enum ScoreMode : int {
  SCORE_LOGITS = 0,    // every token's fp32 logits + softmax partials per chunk (one-sweep dense path)
  SCORE_FILTER = 1,    // softmax partials + candidate records of the tokens that pass the sample threshold
  SCORE_PARTIALS = 2,  // softmax partials only (first sweep of the two-sweep dense path)
  SCORE_SCORES = 3,    // every token's score from known (M, Z) + first radix histogram (second sweep)
};

struct ScoreParams {
  RowGeom geo;
  RowGate gate;
  FilterParams filt;  // SCORE_FILTER only
  const void* q_last;
  const void* K;
  int64_t ks_problem, ks_head, ks_token;  // elements
  PageMap pm;
  // [rows][G] or null.  A logit x >= heavy_thr enters its chunk's softmax sum as exp(l - m) with l
  // recomputed in fp64: an fp32 logit of magnitude |l| is off by about |l| * 2.5e-7, which is the relative
  // error of its exponential, and a head whose mass sits on a few such tokens would get a normaliser that
  // is off by as much; two heads' errors differ, and that can reorder group-sum scores a few 1e-6 apart.
  const float* heavy_thr;
  float* logits;                          // SCORE_LOGITS: [rows][n_chunks][G][kScoreChunk]
  float2* partials;                       // [rows][G][n_chunks]  (max, sum exp(x - max))
  int n_chunks;
  int g0;  // first head of the group handled by this launch
  float scale;
  // SCORE_SCORES: score[i] = sum_g exp(l[g][i] - M_g) / Z_g (or one row per head), histogram of the
  // candidates' first radix digit added to ghist (zeroed beforehand)
  const RowStat* stats;  // [rows][G]
  float* scores;         // [rows * n_lists][pitch]
  int64_t pitch;
  int* ghist;            // [rows * n_lists][kHistBins]
  int S, W, n_lists;
};

struct StatsParams {
  const float2* partials;
  RowStat* stats;  // [rows][G]
  int* ghist;      // [rows * n_lists][kHistBins], zeroed here (nullable)
  int G, n_chunks;
  int n_lists;     // selection lists per row: 1 (group-sum) or G (per-query)
};

// One-sweep dense path: exact statistics from the logit scratch (see stats_exact_kernel).
struct ExactStatsParams {
  RowGeom geo;
  const float2* partials;  // [rows][G][n_chunks]: the chunks' maxima are used
  const float* logits;     // the score pass's scratch
  int n_chunks;
  RowStat* stats;          // out [rows][G]
  int* ghist;              // [rows * n_lists][kHistBins], zeroed here
  int n_lists;
  const void* q_last;
  const void* K;
  int64_t ks_problem, ks_head, ks_token;
  PageMap pm;
};

struct CombineParams {
  RowGeom geo;
  RowGate gate;
  const float* logits;
  int n_chunks;  // score chunks per row (logit scratch layout)
  const RowStat* stats;
  float* scores;  // [rows * n_lists][pitch]
  int64_t pitch;
  int* ghist;
  int S, W;
  int n_lists;    // 1: score = sum over the group's heads; G: one score row per query head
};

struct TopkParams {
  RowGeom geo;
  RowGate gate;
  float* scores;
  int64_t pitch;
  const int* ghist;
  const RowStat* stats;
  const void* q_last;
  const void* K;
  int64_t ks_problem, ks_head, ks_token;
  PageMap pm;
  int32_t* kept_idx;  // [rows][S + n_lists * k + W]
  int S, W, k;
  int n_lists;        // 1 or G; list g of a row ranks head g's own probabilities
  float band;  // relative half-width of the fp64 re-evaluation band around the k-th score
  int bitmap_bytes;  // dynamic LDS of the launch (set by launch_topk): room for one bit per candidate, or 0
};

// The sample of the fast path, in blocks of 64 tokens (one wave-block of the MFMA kernels each):
// the first block of the row if there is a sink, nB blocks over the eviction candidates, each made
// of four runs of 16 consecutive tokens (4 * nB runs spread evenly), nC blocks at the end of the
// recent window.
struct SampleParams {
  RowGeom geo;
  const void* q_last;
  const void* K;
  int64_t ks_problem, ks_head, ks_token;
  PageMap pm;
  int S, W, k;
  int nA, nB, nC;       // blocks per part
  int64_t stepB;        // 48.16 fixed-point distance between the starts of the 16-token candidate runs
  int validA, validC;   // sink tokens in block A; recent tokens covered by the C blocks
  float wA, wB, wC;     // tokens of the row one sampled token stands for
  int rank;             // rank (1-based) of the threshold among the 64 * nB sampled candidates
  int n_lists;          // 1: one threshold on the summed score; G: one per query head
  int Gs;               // heads per token in samp_logit (G rounded up to a multiple of 4)
  float* samp_logit;    // [rows][64 * (nA + nB + nC)][Gs] scratch
  float2* samp_stats;   // out [rows][G]
  float* heavy_thr;     // out [rows][G]: logits at or above it take part in the softmax sum with an fp64 exponent
  float* samp_tau;      // out [rows * n_lists]
  int* row_fail;        // out [rows] = 0
  int* ovf_count;       // out [rows] = 0
  int* n_fail;          // out: 0 rows flagged so far (and: this call runs the pre-filtered path)
  float scale;
};

// Token sampled by slot t (0..63) of sample block b (may lie outside [0, L) for the C blocks of a
// short row: the caller clamps).
__host__ __device__ inline int64_t sample_token(const SampleParams& p, int b, int t) {
  if (b < p.nA) return t;
  b -= p.nA;
  if (b < p.nB) return p.S + (((int64_t)(4 * b + (t >> 4)) * p.stepB) >> 16) + (t & 15);
  b -= p.nB;
  return p.geo.L - 64 * (int64_t)(p.nC - b) + t;
}

// Final selection of the fast path, on the candidate list of each row.
struct TopkCandParams {
  RowGeom geo;
  const float2* partials;    // [rows][G][n_chunks] exact softmax partials of the filtering pass
  RowStat* stats;            // out [rows][G]: exact (M, Z), merged here in fp64
  const float2* samp_stats;  // sample statistics and thresholds, for the bound on a dropped token's score
  const float* samp_tau;
  int* ghist;                // [rows * n_lists][kHistBins]: zeroed here for the dense stages that may follow
  const int* cand_count;     // see FilterParams
  const int32_t* cand_idx;
  const float* cand_logit;
  int cap_c, cap_o;
  int64_t slots_per_row;
  int n_chunks;
  float* cand_score;         // [rows * n_lists][cs_pitch] scratch: exact scores of the candidates, dense
  int32_t* cand_pos;         // [rows * n_lists][cs_pitch] scratch: their token indices
  int64_t cs_pitch;          // floats between the lists' scratch rows (>= cap)
  int cap, Gs;               // cap: candidates a row may have; more = redo
  float2* list_info;         // per-query lists, [rows * n_lists]: (count as int bits, bound), between the two launches
  int n_lists;               // 1 or G: list g of a row ranks head g's own probability
  const void* q_last;
  const void* K;
  int64_t ks_problem, ks_head, ks_token;
  PageMap pm;
  int32_t* kept_idx;
  int* row_fail;  // nonzero (a reason code) when the row must be redone by the general path
  int* n_fail;    // number of flagged rows, incremented with the flag
  int S, W, k;
  float band;
};

struct GatherParams {
  RowGeom geo;
  const void* K;
  const void* V;
  int64_t ks_problem, ks_head, ks_token, vs_problem, vs_head, vs_token;
  PageMap pm;
  const int32_t* kept_idx;
  void* Kc;
  void* Vc;
  int n_kept, cap;
  PageMap cpm;  // reduced cache in pages (see DecodeParams), table = null: dense rows of `cap` tokens
};

struct DecodeParams {
  int n_problems, Hq, Hkv, G, D, dtype;
  const void* q;       // [P][Hq][D]
  const void* q_sink;  // nullable [P][Hq][D]: the query the sink tokens [0, qs_S) are scored with
  int qs_S;
  void* Kc;            // [rows][cap][D]
  void* Vc;
  const void* k_new;   // nullable: [rows][D]
  const void* v_new;
  int slot;            // row position the new token takes, -1 = no append
  int len, cap;
  int n_splits, tokens_per_split;
  // Device-side ring state (nullable).  ring[0] = tokens appended so far, ring[1] = arrival ticket of
  // the launch that advances it.  When set, slot / len / tokens_per_split above are ignored and
  // derived from ring[0] in the kernels (see ring_position); with ring_advance the workgroup that
  // completes the last row of the launch (whole rows) or the merge launch (sliced rows) stores ring[0] + 1.
  int* ring;
  int ring_base, ring_W, ring_grow, ring_advance;
  int stream_loads;    // reduced cache larger than the on-chip caches: read it with streaming loads
  // per-query head mode: rows are [sink | list of head 0 | ... | list of head G-1 | recent]; head g
  // attends the sink, its own list and the recent window.  pq_k = 0: every head attends everything.
  int pq_S, pq_k;
  // Reduced cache in pages (cpm.table != null): Kc / Vc are page pools, a page holds [Hkv][2^shift][D]
  // elements and logical token t of problem p sits in page cpm.table[p * cpm.pitch + (t >> shift)].
  PageMap cpm;
  float* part_acc;     // [rows][n_splits][G][D]
  float2* part_ml;     // [rows][n_splits][G]   (max, sum)
  float* out;          // [P][Hq][D]
  float scale;
};

hipError_t launch_sample(const SampleParams& p, hipStream_t s);         // logits + statistics
hipError_t launch_sample_logits(const SampleParams& p, hipStream_t s);
hipError_t launch_score_filter(const ScoreParams& p, hipStream_t s);
hipError_t launch_topk_cand(const TopkCandParams& p, hipStream_t s);
hipError_t launch_score(const ScoreParams& p, ScoreMode mode, hipStream_t s);  // any mode but SCORE_FILTER
hipError_t launch_stats(const StatsParams& p, int rows, hipStream_t s);
hipError_t launch_stats_exact(const ExactStatsParams& p, hipStream_t s);
hipError_t launch_combine(const CombineParams& p, hipStream_t s);
hipError_t launch_topk(const TopkParams& p, hipStream_t s);
hipError_t launch_gather(const GatherParams& p, hipStream_t s);
hipError_t launch_decode(const DecodeParams& p, hipStream_t s);
hipError_t launch_append(const DecodeParams& p, hipStream_t s);
hipError_t launch_fill_u32(void* ptr, size_t n_words, uint32_t value, hipStream_t s);

// Where the new token goes and how many tokens are attended, from the count n of tokens appended
// before this step (paper Sec. 2 Step 4: the recent window is a FIFO of W entries, kept as a ring at
// [base, base + W); grow mode keeps everything, rows [base + W, ...)).  A grown row that is full
// keeps its length: the token is then not stored (slot = -1) and not attended.
struct RingPos {
  int slot, len;
};
__host__ __device__ inline RingPos ring_position(int base, int W, int grow, int cap, int n) {
  RingPos r;
  if (!grow) {
    r.slot = base + n % W;
    r.len = base + W;
  } else if (base + W + n < cap) {
    r.slot = base + W + n;
    r.len = r.slot + 1;
  } else {
    r.slot = -1;
    r.len = cap;
  }
  return r;
}

// Tokens per split of a row of `len` tokens cut into n_splits slices of whole 64-token blocks.
__host__ __device__ inline int split_tokens(int len, int n_splits) {
  return ((len + n_splits - 1) / n_splits + 63) / 64 * 64;
}

// Does query head g (index inside its group of G) attend position tok of a reduced row?
__host__ __device__ inline bool head_attends(int pq_S, int pq_k, int G, int g, int tok) {
  if (pq_k <= 0 || tok < pq_S || tok >= pq_S + G * pq_k) return true;
  return (tok - pq_S) / pq_k == g;
}

int max_group_per_launch();  // heads of a group one score / decode launch can hold in registers

}  // namespace sagekv
