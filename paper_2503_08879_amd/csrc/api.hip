// C ABI of the library: argument checks, workspace layout, launch order.
#include "../../include/sagekv.h"
#include "../../include/sagekv_bench.h"

#include <math.h>
#include <stdint.h>

#include <mutex>
#include <vector>

#include "kernels.h"

using namespace sagekv;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Relative half-width of the band around the coarse k-th score whose members are re-scored in
// fp64.  fp32 scores carry a relative error of a few 1e-6 at most (dot products of <= 128
// exact products summed pairwise, one exp, one multiply per head), so 2^-12 leaves two orders
// of magnitude of margin while the band still holds only a handful of candidates per row.
constexpr float kBand = 1.0f / 4096.0f;

// Sizes of the fast (pre-filtered) eviction path for one descriptor; ok = the path applies.
struct FastPlan {
  bool ok;
  int nA, nB, nC, validA, validC, rank, cap, Gs;
  int cap_c;  // candidate slots each score chunk owns; what does not fit goes to the row's overflow pool (cap slots)
  int64_t stepB;
  float wA, wB, wC;
};

FastPlan fast_plan(const sagekv_select_desc* d) {
  FastPlan f = {};
  const int G = d->n_q_heads / d->n_kv_heads;
  const int64_t E = d->L - d->n_sink - d->n_recent;
  f.ok = d->dtype == SAGEKV_BF16 && G <= 16 && d->k > 0 && E <= 1048576 && d->L <= 1024 * (int64_t)kScoreChunk &&
         !(d->flags & SAGEKV_SELECT_DENSE);
  if (!f.ok) return f;
  const int lists = d->head_mode == SAGEKV_HEADS_PER_QUERY ? G : 1;
  // sample: runs of 16 consecutive tokens, about 1/64 of the candidates (64 to 512 runs); the
  // sample is read from HBM on top of the full pass over K, so its share is kept small
  int64_t nb = E / 4096;
  f.nB = (int)(nb < 16 ? 16 : (nb > 128 ? 128 : nb));
  f.stepB = ((E - 16) << 16) / (4 * f.nB - 1);  // between 16-token runs
  f.nA = d->n_sink > 0 ? 1 : 0;
  f.validA = d->n_sink < 64 ? d->n_sink : 64;
  // the recent window is where a trained model puts much of its attention: up to its last 512 tokens
  // are all sampled
  f.nC = d->n_recent >= 512 ? 8 : (d->n_recent + 63) / 64;
  f.validC = d->n_recent < 64 * f.nC ? d->n_recent : 64 * f.nC;
  f.wA = f.nA ? (float)d->n_sink / (float)f.validA : 0.f;
  f.wB = (float)E / (float)(64 * f.nB);
  f.wC = (float)d->n_recent / (float)f.validC;
  // Threshold = the rank-th largest approximate score among the n sampled candidates.  About
  // rank * E / n tokens of the row exceed it, with relative sigma 1/sqrt(rank); the rank is the
  // smallest whose 4-sigma low side still keeps (1 + margin) k tokens: rank - 4 sqrt(rank) >=
  // (1 + margin) k n / E.  The margin covers the error of the sampled softmax normalisers; the
  // bound on a dropped token's score takes the worst head's, so it grows with the group size
  // (15 % at G = 4, 20 % at G = 8, 46 % at G = 16: measured, a redone row costs far more than the
  // extra candidates).
  const double margin = 0.10 + 0.0125 * (double)G + (G > 8 ? 0.02 * (double)(G - 8) : 0.0);
  const double r0 = (1.0 + margin) * (double)d->k * (double)(64 * f.nB) / (double)E;
  const double x = 2.0 + sqrt(4.0 + r0);
  f.rank = (int)ceil(x * x);
  // Room for the candidates: about rank * wB tokens pass a list's threshold, 4 sigma high side
  // (rank + 4 sqrt(rank)) * wB; per-query lists share one candidate list per row (their union).
  // (a heavy-tailed row may raise its rank to twice the planned one, see sample_stats_kernel)
  const double high = (2.0 * (double)f.rank + 4.0 * sqrt(2.0 * (double)f.rank)) * (double)f.wB;
  const double planned = 2.5 * (double)d->k;
  int64_t cap = (int64_t)ceil(high > planned ? high : planned) * lists + 4096;
  f.cap = (int)(cap < E ? cap : E);
  // k is a large share of the row: the filter would be expected to keep half of it or more
  if (2.0 * lists * (double)f.rank * (double)f.wB > (double)E || 5 * (int64_t)d->k * lists > E) {
    f.ok = false;
    return f;
  }
  f.Gs = (G + 3) / 4 * 4;
  // A chunk's own slots: twice the candidates an average chunk is expected to keep (rank * wB tokens
  // per list over the row's chunks), so that only chunks where the candidates crowd (a needle
  // cluster, the tokens next to the recent window of a trained model) reach into the overflow pool.
  const int64_t n_chunks = (d->L + kScoreChunk - 1) / kScoreChunk;
  const double per_chunk = (double)f.rank * (double)f.wB * lists / (double)n_chunks;
  int cap_c = 32;
  while (cap_c < 2.0 * per_chunk + 16.0 && cap_c < kScoreChunk) cap_c *= 2;
  f.cap_c = cap_c;
  return f;
}

struct SelectLayout {
  // small: the pre-filtered path applies to the descriptor; rows it cannot certify (and calls that
  // ask for every score) take the two-sweep dense path, which needs no logit scratch.
  bool small;
  size_t logits, scores, partials, stats, ghist, total;
  // pre-filtered path
  size_t samp_logit, samp_stats, heavy_thr, samp_tau, list_info, cand_count, ovf_count, cand_idx, cand_logit, cand_score, cand_pos,
      row_fail, n_fail;
  int64_t slots_per_row, cs_pitch;
  FastPlan fast;
  int64_t Lp;
  int n_chunks, rows, G, n_lists;
};

bool check_select(const sagekv_select_desc* d, sagekv_status* st) {
  *st = SAGEKV_ERR_INVALID_ARG;
  if (!d) return false;
  if (d->n_problems < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->n_q_heads % d->n_kv_heads) return false;
  if (d->L < 1 || d->L > 0x7FFFFFF0ll) return false;
  if (d->n_sink < 0 || d->n_recent < 1 || d->k < 0) return false;
  if ((int64_t)d->n_sink + d->n_recent + d->k > d->L) return false;
  if (d->head_mode != SAGEKV_HEADS_GROUP_SUM && d->head_mode != SAGEKV_HEADS_PER_QUERY) return false;
  const int64_t lists = d->head_mode == SAGEKV_HEADS_PER_QUERY ? d->n_q_heads / d->n_kv_heads : 1;
  if ((int64_t)d->compact_capacity < (int64_t)d->n_sink + d->n_recent + lists * d->k) return false;
  if (d->flags & ~(uint32_t)SAGEKV_SELECT_DENSE) return false;
  *st = SAGEKV_ERR_UNSUPPORTED;
  if (d->dtype != SAGEKV_BF16 && d->dtype != SAGEKV_F32) return false;
  if (d->head_dim != 64 && d->head_dim != 128) return false;
  if (d->n_q_heads / d->n_kv_heads > 64) return false;
  // rows (and selection lists) index one grid dimension of the launches
  if ((int64_t)d->n_problems * d->n_kv_heads * lists > 65535) return false;
  const int epl = d->dtype == SAGEKV_BF16 ? 8 : 4;  // 16-byte alignment of every token row
  const int64_t strides[6] = {d->k_stride_problem, d->k_stride_head, d->k_stride_token,
                              d->v_stride_problem, d->v_stride_head, d->v_stride_token};
  for (int i = 0; i < 6; ++i)
    if (strides[i] < 0 || strides[i] % epl) return false;
  if (d->k_stride_token < d->head_dim || d->v_stride_token < d->head_dim) return false;
  *st = SAGEKV_OK;
  return true;
}

// Workspace layout.  Descriptors the pre-filtered path cannot serve get the one-sweep dense path's
// scratch (every token's fp32 logits: G * 4 bytes per token).  All others get: a score row per
// selection list (used by the rows that have to be redone, and by calls that ask for scores_out
// through the caller's array instead), the candidate records (a few slots per score chunk and an
// overflow pool per row) and small per-row arrays.  The dense candidate arrays of the final
// selection live in the list's score row while it is not in use.
SelectLayout select_layout(const sagekv_select_desc* d, bool own_scores) {
  SelectLayout l = {};
  l.rows = d->n_problems * d->n_kv_heads;
  l.G = d->n_q_heads / d->n_kv_heads;
  l.n_lists = d->head_mode == SAGEKV_HEADS_PER_QUERY ? l.G : 1;
  l.Lp = (d->L + 3) / 4 * 4;
  l.n_chunks = (int)((d->L + kScoreChunk - 1) / kScoreChunk);
  l.fast = fast_plan(d);
  l.small = l.fast.ok;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off = align_up(off + bytes);
    return at;
  };
  const size_t rows = (size_t)l.rows;
  l.logits = take(l.small ? 0 : rows * l.n_chunks * l.G * kScoreChunk * sizeof(float));
  l.partials = take(rows * l.G * l.n_chunks * sizeof(float2));
  l.stats = take(rows * l.G * sizeof(RowStat));
  l.ghist = take(rows * l.n_lists * kHistBins * sizeof(int));
  bool cs_in_scores = false;
  if (l.small) {
    const FastPlan& f = l.fast;
    const size_t ns = (size_t)64 * (f.nA + f.nB + f.nC);
    l.samp_logit = take(rows * ns * f.Gs * sizeof(float));
    l.samp_stats = take(rows * l.G * sizeof(float2));
    l.heavy_thr = take(rows * l.G * sizeof(float));
    l.samp_tau = take(rows * l.n_lists * sizeof(float));
    l.list_info = take(rows * l.n_lists * sizeof(float2));
    l.slots_per_row = (int64_t)l.n_chunks * f.cap_c + f.cap;
    l.cand_count = take(rows * l.n_chunks * sizeof(int));
    l.ovf_count = take(rows * sizeof(int));
    l.cand_idx = take(rows * l.slots_per_row * sizeof(int32_t));
    l.cand_logit = take(rows * l.slots_per_row * f.Gs * sizeof(float));
    l.row_fail = take(rows * sizeof(int));
    l.n_fail = take(sizeof(int));
    cs_in_scores = 2 * (int64_t)f.cap <= l.Lp;
    l.cs_pitch = cs_in_scores ? l.Lp : f.cap;
    if (!cs_in_scores) {
      l.cand_score = take(rows * l.n_lists * f.cap * sizeof(float));
      l.cand_pos = take(rows * l.n_lists * f.cap * sizeof(int32_t));
    }
  }
  // last, so that no other offset depends on whether the caller brought its own score rows
  l.scores = take(own_scores ? rows * l.n_lists * l.Lp * sizeof(float) : 0);
  if (cs_in_scores) {  // the first half of a list's score row: exact scores, the second: token indices
    l.cand_score = l.scores;
    l.cand_pos = l.scores + (size_t)l.fast.cap * sizeof(float);
  }
  l.total = off;
  return l;
}

int decode_lists(const sagekv_decode_desc* d) {
  return d->head_mode == SAGEKV_HEADS_PER_QUERY ? d->n_q_heads / d->n_kv_heads : 1;
}

bool check_decode(const sagekv_decode_desc* d, sagekv_status* st) {
  *st = SAGEKV_ERR_INVALID_ARG;
  if (!d) return false;
  if (d->n_problems < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->n_q_heads % d->n_kv_heads) return false;
  if (d->n_sink < 0 || d->n_recent < 1 || d->k < 0) return false;
  if (d->head_mode != SAGEKV_HEADS_GROUP_SUM && d->head_mode != SAGEKV_HEADS_PER_QUERY) return false;
  if ((int64_t)d->compact_capacity < (int64_t)d->n_sink + d->n_recent + (int64_t)decode_lists(d) * d->k) return false;
  *st = SAGEKV_ERR_UNSUPPORTED;
  if ((int64_t)d->n_problems * d->n_kv_heads > 65535) return false;  // rows index one grid dimension
  if (d->dtype != SAGEKV_BF16 && d->dtype != SAGEKV_F32) return false;
  if (d->head_dim != 64 && d->head_dim != 128) return false;
  *st = SAGEKV_OK;
  return true;
}

struct DecodeLayout {
  size_t part_ml, part_acc, total;
  int max_splits, rows, G;
};

// Splits per row.  With about one row per CU or more, a single 8-wave workgroup per row fills
// the chip and needs no merge launch; otherwise enough workgroups to fill 256 CUs several times
// over, at least 128 tokens each.
int splits_for(int rows, int len) {
  if (rows >= 192) return 1;
  int want = (2048 + rows - 1) / rows;
  int most = (len + 127) / 128;
  int n = want < most ? want : most;
  return n < 1 ? 1 : n;
}

DecodeLayout decode_layout(const sagekv_decode_desc* d) {
  DecodeLayout l;
  l.rows = d->n_problems * d->n_kv_heads;
  l.G = d->n_q_heads / d->n_kv_heads;
  l.max_splits = splits_for(l.rows, d->compact_capacity);
  size_t off = 0;
  l.part_ml = off;
  off = align_up(off + (size_t)l.rows * l.max_splits * l.G * sizeof(float2));
  l.part_acc = off;
  off = align_up(off + (size_t)l.rows * l.max_splits * l.G * d->head_dim * sizeof(float));
  l.total = l.max_splits > 1 ? off : 0;  // one split per row writes `out` directly
  return l;
}

// ---- stage timing -----------------------------------------------------------------------------
struct Timing {
  int n_calls = 0;
  int next_select = 0, next_decode = 0;
  std::vector<hipEvent_t> sel;  // [n_calls][SAGEKV_N_STAGES][2]
  std::vector<hipEvent_t> dec;  // [n_calls][2]
  std::vector<uint32_t> sel_mask;  // [n_calls] stages that recorded both events
  uint32_t stages = ~0u;           // select stages to bracket
  bool decode = true;              // bracket decode calls
} g_timing;

struct StageTimer {
  hipEvent_t* ev = nullptr;
  uint32_t* mask = nullptr;
  hipStream_t s;
  StageTimer(int which, hipStream_t stream) : s(stream) {
    if (g_timing.n_calls == 0) return;
    if (which == 0 && g_timing.next_select < g_timing.n_calls) {
      mask = &g_timing.sel_mask[g_timing.next_select];
      *mask = 0;
      ev = &g_timing.sel[(size_t)g_timing.next_select++ * SAGEKV_N_STAGES * 2];
    }
    if (which == 1 && g_timing.decode && g_timing.next_decode < g_timing.n_calls)
      ev = &g_timing.dec[(size_t)g_timing.next_decode++ * 2];
  }
  bool on(int stage) const { return ev && (!mask || ((g_timing.stages >> stage) & 1u)); }
  void begin(int stage) {
    if (on(stage)) (void)hipEventRecord(ev[stage * 2], s);
  }
  void end(int stage) {
    if (!on(stage)) return;
    (void)hipEventRecord(ev[stage * 2 + 1], s);
    if (mask) *mask |= 1u << stage;
  }
};

sagekv_status dev(hipError_t e) { return e == hipSuccess ? SAGEKV_OK : SAGEKV_ERR_DEVICE; }

// Checks the page description of a reduced cache of `capacity` tokens per row and turns it into the
// kernels' page map.
sagekv_status compact_page_map(const sagekv_paged_kv* pg, int dtype, int n_kv_heads, int head_dim, int64_t capacity,
                               PageMap* pm) {
  if (!pg || !pg->block_table || pg->n_pages < 1) return SAGEKV_ERR_INVALID_ARG;
  const int ps = pg->page_size;
  if (ps < 16 || (ps & (ps - 1))) return SAGEKV_ERR_INVALID_ARG;
  if (pg->table_pitch < (capacity + ps - 1) / ps) return SAGEKV_ERR_INVALID_ARG;
  const int64_t page_elems = (int64_t)n_kv_heads * ps * head_dim;
  if (pg->k_stride_page < page_elems || pg->v_stride_page < page_elems) return SAGEKV_ERR_INVALID_ARG;
  const int epl = dtype == SAGEKV_BF16 ? 8 : 4;
  if ((uintptr_t)pg->block_table & 3u || pg->k_stride_page % epl || pg->v_stride_page % epl) return SAGEKV_ERR_UNSUPPORTED;
  pm->table = pg->block_table;
  pm->pitch = pg->table_pitch;
  pm->ks_page = pg->k_stride_page;
  pm->vs_page = pg->v_stride_page;
  pm->shift = __builtin_ctz((unsigned)ps);
  pm->n_pages = pg->n_pages;
  return SAGEKV_OK;
}

// Scratch of sagekv_decode_step_static: the split partials of a decode step, for callers that cannot
// hand over device memory.  Every GPU the library runs on holds its own copy of this array at its
// own address; in host code the name is only a handle for hipGetSymbolAddress, never an address.
static __device__ __align__(256) unsigned char scratch[SAGEKV_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each GPU, once looked up

// Device address of the scratch array on the current GPU (looked up once per device, with that
// device current).
sagekv_status static_scratch(void** ptr) {
  int device = -1;
  if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return SAGEKV_ERR_DEVICE;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SAGEKV_ERR_DEVICE;
    g_scratch_ptr[device] = p;
  }
  *ptr = g_scratch_ptr[device];
  return SAGEKV_OK;
}

// Every cache and query row is read and written 16 bytes per lane.
inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// `ring` (nullable, device): the count of appended tokens lives on the device; slot and len are then
// derived in the kernels and the launch moves the count on.
sagekv_status run_decode(const sagekv_decode_desc* d, const void* q, const void* q_sink, const void* k_new,
                         const void* v_new,
                         void* Kc, void* Vc, int slot, int len, int32_t* ring, float* out, void* ws,
                         size_t ws_bytes, hipStream_t s, const PageMap* cpm = nullptr) {
  if (!aligned16(q) || !aligned16(q_sink) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(Kc) ||
      !aligned16(Vc) || ((uintptr_t)out & 3u) || !aligned16(ws) || ((uintptr_t)ring & 3u))
    return SAGEKV_ERR_UNSUPPORTED;
  const DecodeLayout l = decode_layout(d);
  if (l.total > 0 && (!ws || ws_bytes < l.total)) return SAGEKV_ERR_WORKSPACE;
  DecodeParams p = {};
  p.n_problems = d->n_problems;
  p.Hq = d->n_q_heads;
  p.Hkv = d->n_kv_heads;
  p.G = l.G;
  p.D = d->head_dim;
  p.dtype = d->dtype;
  p.q = q;
  p.q_sink = q_sink;
  p.qs_S = q_sink ? d->n_sink : 0;
  p.Kc = Kc;
  p.Vc = Vc;
  p.k_new = k_new;
  p.v_new = v_new;
  p.slot = slot;
  p.len = len;
  p.cap = d->compact_capacity;
  // with the count on the device the length of a growing row is not known here: as many slices as
  // the full capacity would take (a fixed-size window has its one length either way)
  p.n_splits = splits_for(l.rows, ring && d->grow_recent ? d->compact_capacity : len);
  if (p.n_splits > l.max_splits) p.n_splits = l.max_splits;
  p.tokens_per_split = split_tokens(len, p.n_splits);
  p.ring = ring;
  p.ring_base = d->n_sink + decode_lists(d) * d->k;
  p.ring_W = d->n_recent;
  p.ring_grow = d->grow_recent;
  p.ring_advance = ring != nullptr;
  if (cpm) p.cpm = *cpm;
  // a reduced cache that cannot stay in L2 / Infinity Cache between steps is streamed (measured: +8 %)
  p.pq_S = d->n_sink;
  p.pq_k = decode_lists(d) > 1 ? d->k : 0;
  p.stream_loads = 2.0 * l.rows * len * d->head_dim * (d->dtype == SAGEKV_BF16 ? 2 : 4) > 192.0 * 1024 * 1024;
  p.part_ml = (float2*)((char*)ws + l.part_ml);
  p.part_acc = (float*)((char*)ws + l.part_acc);
  p.out = out;
  p.scale = (float)(1.0 / sqrt((double)d->head_dim));
  StageTimer t(1, s);
  t.begin(0);
  hipError_t e = launch_decode(p, s);
  t.end(0);
  return dev(e);
}

}  // namespace

extern "C" {

sagekv_status sagekv_paper_budget(int32_t B, int32_t G, int32_t* n_sink, int32_t* k, int32_t* n_recent) {
  if (!n_sink || !k || !n_recent || G < 1 || B < 4 * (int64_t)G) return SAGEKV_ERR_INVALID_ARG;
  const int32_t share = B / (2 * G);  // >= 2
  int32_t pow2 = 1;
  while (pow2 <= share / 2) pow2 *= 2;
  *n_sink = B / 4;
  *k = pow2;
  *n_recent = B - B / 4 - G * pow2;
  return SAGEKV_OK;
}

const char* sagekv_status_string(sagekv_status s) {
  switch (s) {
    case SAGEKV_OK: return "ok";
    case SAGEKV_ERR_INVALID_ARG: return "invalid argument";
    case SAGEKV_ERR_UNSUPPORTED: return "unsupported configuration";
    case SAGEKV_ERR_WORKSPACE: return "workspace missing or too small";
    case SAGEKV_ERR_DEVICE: return "HIP launch failed";
    case SAGEKV_ERR_SCRATCH_LIMIT: return "problem exceeds the library's built-in scratch (SAGEKV_STATIC_SCRATCH_BYTES)";
  }
  return "unknown status";
}

size_t sagekv_select_workspace_bytes(const sagekv_select_desc* desc) {
  sagekv_status st;
  if (!check_select(desc, &st)) return 0;
  return select_layout(desc, true).total;
}

}  // extern "C"

namespace {

sagekv_status select_impl(const sagekv_select_desc* d, const PageMap& pm, const void* q_last, const void* K,
                          const void* V, void* Kc, void* Vc, int32_t* kept_idx, float* scores_out, void* workspace,
                          size_t workspace_bytes, void* hip_stream, const PageMap* out_pm = nullptr) {
  sagekv_status st;
  if (!check_select(d, &st)) return st;
  if (!q_last || !K || !V || !Kc || !Vc || !kept_idx) return SAGEKV_ERR_INVALID_ARG;
  if (!aligned16(q_last) || !aligned16(K) || !aligned16(V) || !aligned16(Kc) || !aligned16(Vc) ||
      ((uintptr_t)kept_idx & 3u) || ((uintptr_t)scores_out & 15u) || !aligned16(workspace))
    return SAGEKV_ERR_UNSUPPORTED;
  const SelectLayout l = select_layout(d, scores_out == nullptr);
  if (!workspace || workspace_bytes < l.total) return SAGEKV_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  // per-token scores are only produced by the dense stages
  const bool fast = l.small && scores_out == nullptr;

  RowGeom geo;
  geo.n_problems = d->n_problems;
  geo.Hq = d->n_q_heads;
  geo.Hkv = d->n_kv_heads;
  geo.G = l.G;
  geo.D = d->head_dim;
  geo.dtype = d->dtype;
  geo.L = d->L;
  geo.Lp = l.Lp;

  float* scores = scores_out ? scores_out : (float*)(ws + l.scores);
  const int64_t pitch = scores_out ? d->L : l.Lp;
  float2* partials = (float2*)(ws + l.partials);
  RowStat* stats = (RowStat*)(ws + l.stats);
  int* ghist = (int*)(ws + l.ghist);
  const float scale = (float)(1.0 / sqrt((double)d->head_dim));

  StageTimer t(0, s);
  hipError_t e;

  ScoreParams sp = {};
  sp.geo = geo;
  sp.q_last = q_last;
  sp.K = K;
  sp.ks_problem = d->k_stride_problem;
  sp.ks_head = d->k_stride_head;
  sp.ks_token = d->k_stride_token;
  sp.pm = pm;
  sp.logits = (float*)(ws + l.logits);
  sp.partials = partials;
  sp.n_chunks = l.n_chunks;
  sp.g0 = 0;
  sp.scale = scale;
  sp.stats = stats;
  sp.scores = scores;
  sp.pitch = pitch;
  sp.ghist = ghist;
  sp.S = d->n_sink;
  sp.W = d->n_recent;
  sp.n_lists = l.n_lists;

  StatsParams tp = {};
  tp.partials = partials;
  tp.stats = stats;
  tp.ghist = ghist;
  tp.G = l.G;
  tp.n_chunks = l.n_chunks;
  tp.n_lists = l.n_lists;

  TopkParams kp = {};
  kp.geo = geo;
  kp.scores = scores;
  kp.pitch = pitch;
  kp.ghist = ghist;
  kp.stats = stats;
  kp.q_last = q_last;
  kp.K = K;
  kp.ks_problem = d->k_stride_problem;
  kp.ks_head = d->k_stride_head;
  kp.ks_token = d->k_stride_token;
  kp.pm = pm;
  kp.kept_idx = kept_idx;
  kp.S = d->n_sink;
  kp.W = d->n_recent;
  kp.k = d->k;
  kp.n_lists = l.n_lists;
  kp.band = kBand;

  // The sample stage: approximate softmax statistics and filter thresholds for the pre-filtered path; both
  // that path and the two-sweep path take from it which terms of a softmax sum need an fp64 exponent.
  auto run_sample = [&]() -> hipError_t {
    const FastPlan& f = l.fast;
    SampleParams mp = {};
    mp.geo = geo;
    mp.q_last = q_last;
    mp.K = K;
    mp.ks_problem = d->k_stride_problem;
    mp.ks_head = d->k_stride_head;
    mp.ks_token = d->k_stride_token;
    mp.pm = pm;
    mp.S = d->n_sink;
    mp.W = d->n_recent;
    mp.k = d->k;
    mp.nA = f.nA;
    mp.nB = f.nB;
    mp.nC = f.nC;
    mp.stepB = f.stepB;
    mp.validA = f.validA;
    mp.validC = f.validC;
    mp.wA = f.wA;
    mp.wB = f.wB;
    mp.wC = f.wC;
    mp.rank = f.rank;
    mp.n_lists = l.n_lists;
    mp.Gs = f.Gs;
    mp.samp_logit = (float*)(ws + l.samp_logit);
    mp.samp_stats = (float2*)(ws + l.samp_stats);
    mp.heavy_thr = (float*)(ws + l.heavy_thr);
    mp.samp_tau = (float*)(ws + l.samp_tau);
    mp.row_fail = (int*)(ws + l.row_fail);
    mp.ovf_count = (int*)(ws + l.ovf_count);
    mp.n_fail = (int*)(ws + l.n_fail);
    mp.scale = scale;
    t.begin(SAGEKV_STAGE_SAMPLE);
    const hipError_t es = launch_sample(mp, s);
    t.end(SAGEKV_STAGE_SAMPLE);
    return es;
  };

  if (fast) {
    // ---- pre-filtered path: sample, one filtering pass over K, selection among the candidates
    const FastPlan& f = l.fast;
    float2* samp_stats = (float2*)(ws + l.samp_stats);
    float* samp_tau = (float*)(ws + l.samp_tau);
    int* row_fail = (int*)(ws + l.row_fail);
    e = run_sample();
    if (e != hipSuccess) return SAGEKV_ERR_DEVICE;
    sp.heavy_thr = (const float*)(ws + l.heavy_thr);

    ScoreParams fp = sp;
    fp.filt.samp_stats = samp_stats;
    fp.filt.samp_tau = samp_tau;
    fp.filt.cand_count = (int*)(ws + l.cand_count);
    fp.filt.ovf_count = (int*)(ws + l.ovf_count);
    fp.filt.cand_idx = (int32_t*)(ws + l.cand_idx);
    fp.filt.cand_logit = (float*)(ws + l.cand_logit);
    fp.filt.cap_c = f.cap_c;
    fp.filt.cap_o = f.cap;
    fp.filt.slots_per_row = l.slots_per_row;
    fp.filt.Gs = f.Gs;
    fp.filt.n_lists = l.n_lists;
    fp.filt.S = d->n_sink;
    fp.filt.W = d->n_recent;
    t.begin(SAGEKV_STAGE_SCORE);
    e = launch_score_filter(fp, s);
    t.end(SAGEKV_STAGE_SCORE);
    if (e != hipSuccess) return SAGEKV_ERR_DEVICE;

    TopkCandParams cp = {};
    cp.geo = geo;
    cp.partials = partials;
    cp.stats = stats;
    cp.samp_stats = samp_stats;
    cp.samp_tau = samp_tau;
    cp.ghist = ghist;
    cp.cand_count = fp.filt.cand_count;
    cp.cand_idx = fp.filt.cand_idx;
    cp.cand_logit = fp.filt.cand_logit;
    cp.cap_c = f.cap_c;
    cp.cap_o = f.cap;
    cp.slots_per_row = l.slots_per_row;
    cp.n_chunks = l.n_chunks;
    cp.cand_score = (float*)(ws + l.cand_score);
    cp.cand_pos = (int32_t*)(ws + l.cand_pos);
    cp.cs_pitch = l.cs_pitch;
    cp.list_info = (float2*)(ws + l.list_info);
    cp.cap = f.cap;
    cp.Gs = f.Gs;
    cp.n_lists = l.n_lists;
    cp.q_last = q_last;
    cp.K = K;
    cp.ks_problem = d->k_stride_problem;
    cp.ks_head = d->k_stride_head;
    cp.ks_token = d->k_stride_token;
    cp.pm = pm;
    cp.kept_idx = kept_idx;
    cp.row_fail = row_fail;
    cp.n_fail = (int*)(ws + l.n_fail);
    cp.S = d->n_sink;
    cp.W = d->n_recent;
    cp.k = d->k;
    cp.band = kBand;
    t.begin(SAGEKV_STAGE_TOPK);
    e = launch_topk_cand(cp, s);
    t.end(SAGEKV_STAGE_TOPK);
    if (e != hipSuccess) return SAGEKV_ERR_DEVICE;

    // Rows that could not be certified: a second pass over their K turns the now exact (M, Z) into
    // every token's score, then the dense selection.  Both launches are gated by the rows' flags:
    // with nothing flagged they are a handful of workgroups that look at the flags and leave.
    t.begin(SAGEKV_STAGE_REDO);
    sp.gate.row_flag = row_fail;
    sp.gate.n_flagged = (int*)(ws + l.n_fail);
    e = launch_score(sp, SCORE_SCORES, s);
    if (e != hipSuccess) return SAGEKV_ERR_DEVICE;
    kp.gate = sp.gate;
    e = launch_topk(kp, s);
    t.end(SAGEKV_STAGE_REDO);
    if (e != hipSuccess) return SAGEKV_ERR_DEVICE;
  } else if (l.small) {
    // ---- every score is asked for, no logit scratch: two sweeps over K (partials, then scores)
    e = run_sample();  // for heavy_thr (it also clears the flags; the marker below follows it)
    if (e != hipSuccess) return SAGEKV_ERR_DEVICE;
    sp.heavy_thr = (const float*)(ws + l.heavy_thr);
    if (launch_fill_u32(ws + l.n_fail, 1, 0xFFFFFFFFu, s) != hipSuccess) return SAGEKV_ERR_DEVICE;
    t.begin(SAGEKV_STAGE_SCORE);
    e = launch_score(sp, SCORE_PARTIALS, s);
    t.end(SAGEKV_STAGE_SCORE);
    if (e != hipSuccess) return SAGEKV_ERR_DEVICE;
    t.begin(SAGEKV_STAGE_STATS);
    e = launch_stats(tp, l.rows, s);
    t.end(SAGEKV_STAGE_STATS);
    if (e != hipSuccess) return SAGEKV_ERR_DEVICE;
    t.begin(SAGEKV_STAGE_COMBINE);
    e = launch_score(sp, SCORE_SCORES, s);
    t.end(SAGEKV_STAGE_COMBINE);
    if (e != hipSuccess) return SAGEKV_ERR_DEVICE;
    t.begin(SAGEKV_STAGE_TOPK);
    e = launch_topk(kp, s);
    t.end(SAGEKV_STAGE_TOPK);
    if (e != hipSuccess) return SAGEKV_ERR_DEVICE;
  } else {
    // ---- one-sweep dense path: logits to scratch, statistics, scores, selection
    t.begin(SAGEKV_STAGE_SCORE);
    e = launch_score(sp, SCORE_LOGITS, s);
    t.end(SAGEKV_STAGE_SCORE);
    if (e != hipSuccess) return SAGEKV_ERR_DEVICE;
    ExactStatsParams xp = {};
    xp.geo = geo;
    xp.partials = partials;
    xp.logits = sp.logits;
    xp.n_chunks = l.n_chunks;
    xp.stats = stats;
    xp.ghist = ghist;
    xp.n_lists = l.n_lists;
    xp.q_last = q_last;
    xp.K = K;
    xp.ks_problem = d->k_stride_problem;
    xp.ks_head = d->k_stride_head;
    xp.ks_token = d->k_stride_token;
    xp.pm = pm;
    t.begin(SAGEKV_STAGE_STATS);
    e = launch_stats_exact(xp, s);
    t.end(SAGEKV_STAGE_STATS);
    if (e != hipSuccess) return SAGEKV_ERR_DEVICE;
    CombineParams cp = {};
    cp.geo = geo;
    cp.logits = sp.logits;
    cp.n_chunks = l.n_chunks;
    cp.stats = stats;
    cp.scores = scores;
    cp.pitch = pitch;
    cp.ghist = ghist;
    cp.S = d->n_sink;
    cp.W = d->n_recent;
    cp.n_lists = l.n_lists;
    t.begin(SAGEKV_STAGE_COMBINE);
    e = launch_combine(cp, s);
    t.end(SAGEKV_STAGE_COMBINE);
    if (e != hipSuccess) return SAGEKV_ERR_DEVICE;
    t.begin(SAGEKV_STAGE_TOPK);
    e = launch_topk(kp, s);
    t.end(SAGEKV_STAGE_TOPK);
    if (e != hipSuccess) return SAGEKV_ERR_DEVICE;
  }

  GatherParams gp = {};
  gp.geo = geo;
  gp.K = K;
  gp.V = V;
  gp.ks_problem = d->k_stride_problem;
  gp.ks_head = d->k_stride_head;
  gp.ks_token = d->k_stride_token;
  gp.vs_problem = d->v_stride_problem;
  gp.vs_head = d->v_stride_head;
  gp.vs_token = d->v_stride_token;
  gp.pm = pm;
  gp.kept_idx = kept_idx;
  gp.Kc = Kc;
  gp.Vc = Vc;
  gp.n_kept = d->n_sink + l.n_lists * d->k + d->n_recent;
  gp.cap = d->compact_capacity;
  if (out_pm) gp.cpm = *out_pm;
  t.begin(SAGEKV_STAGE_GATHER);
  e = launch_gather(gp, s);
  t.end(SAGEKV_STAGE_GATHER);
  return dev(e);
}

}  // namespace

extern "C" {

sagekv_status sagekv_select(const sagekv_select_desc* d, const void* q_last, const void* K, const void* V, void* Kc,
                            void* Vc, int32_t* kept_idx, float* scores_out, void* workspace, size_t workspace_bytes,
                            void* hip_stream) {
  const PageMap none = {nullptr, 0, 0, 0, 0, 0};
  return select_impl(d, none, q_last, K, V, Kc, Vc, kept_idx, scores_out, workspace, workspace_bytes, hip_stream);
}

}  // extern "C"

namespace {
// Page map of a paged FULL cache (the strides inside a page come from the select descriptor).
sagekv_status input_page_map(const sagekv_select_desc* d, const sagekv_paged_kv* pg, PageMap* pm) {
  if (!pg || !pg->block_table || pg->n_pages < 1) return SAGEKV_ERR_INVALID_ARG;
  if ((uintptr_t)pg->block_table & 3u) return SAGEKV_ERR_UNSUPPORTED;
  const int ps = pg->page_size;
  if (ps < 16 || (ps & (ps - 1))) return SAGEKV_ERR_INVALID_ARG;
  if (pg->table_pitch < (d->L + ps - 1) / ps) return SAGEKV_ERR_INVALID_ARG;
  const int epl = d->dtype == SAGEKV_BF16 ? 8 : 4;
  if (pg->k_stride_page < 0 || pg->v_stride_page < 0 || pg->k_stride_page % epl || pg->v_stride_page % epl)
    return SAGEKV_ERR_UNSUPPORTED;
  pm->table = pg->block_table;
  pm->pitch = pg->table_pitch;
  pm->ks_page = pg->k_stride_page;
  pm->vs_page = pg->v_stride_page;
  pm->shift = __builtin_ctz((unsigned)ps);
  pm->n_pages = pg->n_pages;
  return SAGEKV_OK;
}
}  // namespace

extern "C" {

sagekv_status sagekv_select_paged(const sagekv_select_desc* d, const sagekv_paged_kv* pg, const void* q_last,
                                  const void* K_pool, const void* V_pool, void* Kc, void* Vc, int32_t* kept_idx,
                                  float* scores_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  sagekv_status st;
  if (!check_select(d, &st)) return st;
  PageMap pm;
  st = input_page_map(d, pg, &pm);
  if (st != SAGEKV_OK) return st;
  return select_impl(d, pm, q_last, K_pool, V_pool, Kc, Vc, kept_idx, scores_out, workspace, workspace_bytes,
                     hip_stream);
}

sagekv_status sagekv_select_into_pages(const sagekv_select_desc* d, const sagekv_paged_kv* in_pages,
                                       const sagekv_paged_kv* out_pages, const void* q_last, const void* K,
                                       const void* V, void* Kc_pool, void* Vc_pool, int32_t* kept_idx,
                                       float* scores_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  sagekv_status st;
  if (!check_select(d, &st)) return st;
  PageMap in_pm = {nullptr, 0, 0, 0, 0, 0}, out_pm;
  if (in_pages) {
    st = input_page_map(d, in_pages, &in_pm);
    if (st != SAGEKV_OK) return st;
  }
  st = compact_page_map(out_pages, d->dtype, d->n_kv_heads, d->head_dim, d->compact_capacity, &out_pm);
  if (st != SAGEKV_OK) return st;
  return select_impl(d, in_pm, q_last, K, V, Kc_pool, Vc_pool, kept_idx, scores_out, workspace, workspace_bytes,
                     hip_stream, &out_pm);
}

sagekv_status sagekv_select_redone_rows(const sagekv_select_desc* d, const void* workspace, size_t workspace_bytes,
                                        void* hip_stream, int32_t* n_rows) {
  sagekv_status st;
  if (!check_select(d, &st)) return st;
  if (!n_rows) return SAGEKV_ERR_INVALID_ARG;
  const SelectLayout l = select_layout(d, true);
  if (!workspace || workspace_bytes < l.total) return SAGEKV_ERR_WORKSPACE;
  *n_rows = -1;
  if (!l.small) return SAGEKV_OK;
  hipStream_t s = (hipStream_t)hip_stream;
  if (hipStreamSynchronize(s) != hipSuccess) return SAGEKV_ERR_DEVICE;
  int n = 0;  // -1: the last call went through the dense stages for every row
  if (hipMemcpy(&n, (const char*)workspace + l.n_fail, sizeof(int), hipMemcpyDeviceToHost) != hipSuccess)
    return SAGEKV_ERR_DEVICE;
  *n_rows = n;
  return SAGEKV_OK;
}

sagekv_status sagekv_append(const sagekv_decode_desc* d, const void* k_new, const void* v_new, void* Kc, void* Vc,
                            int32_t n_appended, void* hip_stream) {
  sagekv_status st;
  if (!check_decode(d, &st)) return st;
  if (!k_new || !v_new || !Kc || !Vc || n_appended < 0) return SAGEKV_ERR_INVALID_ARG;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(Kc) || !aligned16(Vc)) return SAGEKV_ERR_UNSUPPORTED;
  const int base = d->n_sink + decode_lists(d) * d->k;
  const int64_t slot = d->grow_recent ? (int64_t)base + d->n_recent + n_appended : base + n_appended % d->n_recent;
  if (slot >= d->compact_capacity) return SAGEKV_ERR_INVALID_ARG;
  DecodeParams p = {};
  p.n_problems = d->n_problems;
  p.Hkv = d->n_kv_heads;
  p.D = d->head_dim;
  p.dtype = d->dtype;
  p.Kc = Kc;
  p.Vc = Vc;
  p.k_new = k_new;
  p.v_new = v_new;
  p.slot = (int)slot;
  p.cap = d->compact_capacity;
  return dev(launch_append(p, (hipStream_t)hip_stream));
}

size_t sagekv_decode_workspace_bytes(const sagekv_decode_desc* desc) {
  sagekv_status st;
  if (!check_decode(desc, &st)) return 0;
  return decode_layout(desc).total;
}

sagekv_status sagekv_decode_attn(const sagekv_decode_desc* d, const void* q, const void* Kc, const void* Vc,
                                 int32_t len, float* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  sagekv_status st;
  if (!check_decode(d, &st)) return st;
  if (!q || !Kc || !Vc || !out || len < 1 || len > d->compact_capacity) return SAGEKV_ERR_INVALID_ARG;
  return run_decode(d, q, nullptr, nullptr, nullptr, const_cast<void*>(Kc), const_cast<void*>(Vc), -1, len, nullptr, out,
                    workspace, workspace_bytes, (hipStream_t)hip_stream);
}

sagekv_status sagekv_decode_attn_window(const sagekv_decode_desc* d, const void* q, const void* q_sink, const void* Kc,
                                        const void* Vc, int32_t len, float* out, void* workspace,
                                        size_t workspace_bytes, void* hip_stream) {
  sagekv_status st;
  if (!check_decode(d, &st)) return st;
  if (!q || !q_sink || !Kc || !Vc || !out || len < 1 || len > d->compact_capacity) return SAGEKV_ERR_INVALID_ARG;
  return run_decode(d, q, q_sink, nullptr, nullptr, const_cast<void*>(Kc), const_cast<void*>(Vc), -1, len, nullptr, out,
                    workspace, workspace_bytes, (hipStream_t)hip_stream);
}

sagekv_status sagekv_decode_step(const sagekv_decode_desc* d, const void* q, const void* k_new, const void* v_new,
                                 void* Kc, void* Vc, int32_t n_appended, float* out, void* workspace,
                                 size_t workspace_bytes, void* hip_stream) {
  sagekv_status st;
  if (!check_decode(d, &st)) return st;
  if (!q || !k_new || !v_new || !Kc || !Vc || !out || n_appended < 0) return SAGEKV_ERR_INVALID_ARG;
  const int base = d->n_sink + decode_lists(d) * d->k;
  const int64_t slot = d->grow_recent ? (int64_t)base + d->n_recent + n_appended : base + n_appended % d->n_recent;
  const int64_t len = d->grow_recent ? slot + 1 : (int64_t)base + d->n_recent;
  if (slot >= d->compact_capacity) return SAGEKV_ERR_INVALID_ARG;
  return run_decode(d, q, nullptr, k_new, v_new, Kc, Vc, (int)slot, (int)len, nullptr, out, workspace, workspace_bytes,
                    (hipStream_t)hip_stream);
}

sagekv_status sagekv_decode_step_static(const sagekv_decode_desc* d, const void* q, const void* k_new, const void* v_new,
                                        void* Kc, void* Vc, int32_t n_appended, float* out, void* hip_stream) {
  sagekv_status st;
  if (!check_decode(d, &st)) return st;
  if (!q || !k_new || !v_new || !Kc || !Vc || !out || n_appended < 0) return SAGEKV_ERR_INVALID_ARG;
  const int base = d->n_sink + decode_lists(d) * d->k;
  const int64_t slot = d->grow_recent ? (int64_t)base + d->n_recent + n_appended : base + n_appended % d->n_recent;
  const int64_t len = d->grow_recent ? slot + 1 : (int64_t)base + d->n_recent;
  if (slot >= d->compact_capacity) return SAGEKV_ERR_INVALID_ARG;
  if (decode_layout(d).total > (size_t)SAGEKV_STATIC_SCRATCH_BYTES) return SAGEKV_ERR_SCRATCH_LIMIT;
  void* ws = nullptr;
  st = static_scratch(&ws);
  if (st != SAGEKV_OK) return st;
  return run_decode(d, q, nullptr, k_new, v_new, Kc, Vc, (int)slot, (int)len, nullptr, out, ws,
                    (size_t)SAGEKV_STATIC_SCRATCH_BYTES, (hipStream_t)hip_stream);
}

sagekv_status sagekv_decode_attn_paged(const sagekv_decode_desc* d, const sagekv_paged_kv* pages, const void* q,
                                       const void* Kc_pool, const void* Vc_pool, int32_t len, float* out,
                                       void* workspace, size_t workspace_bytes, void* hip_stream) {
  sagekv_status st;
  if (!check_decode(d, &st)) return st;
  if (!q || !Kc_pool || !Vc_pool || !out || len < 1 || len > d->compact_capacity) return SAGEKV_ERR_INVALID_ARG;
  PageMap cpm;
  st = compact_page_map(pages, d->dtype, d->n_kv_heads, d->head_dim, d->compact_capacity, &cpm);
  if (st != SAGEKV_OK) return st;
  return run_decode(d, q, nullptr, nullptr, nullptr, const_cast<void*>(Kc_pool), const_cast<void*>(Vc_pool), -1, len,
                    nullptr, out, workspace, workspace_bytes, (hipStream_t)hip_stream, &cpm);
}

sagekv_status sagekv_decode_step_paged(const sagekv_decode_desc* d, const sagekv_paged_kv* pages, const void* q,
                                       const void* k_new, const void* v_new, void* Kc_pool, void* Vc_pool,
                                       int32_t n_appended, int32_t* ring_state, float* out, void* workspace,
                                       size_t workspace_bytes, void* hip_stream) {
  sagekv_status st;
  if (!check_decode(d, &st)) return st;
  if (!q || !k_new || !v_new || !Kc_pool || !Vc_pool || !out || (!ring_state && n_appended < 0))
    return SAGEKV_ERR_INVALID_ARG;
  PageMap cpm;
  st = compact_page_map(pages, d->dtype, d->n_kv_heads, d->head_dim, d->compact_capacity, &cpm);
  if (st != SAGEKV_OK) return st;
  const int base = d->n_sink + decode_lists(d) * d->k;
  if (ring_state) {
    const int len = d->grow_recent ? d->compact_capacity : base + d->n_recent;
    return run_decode(d, q, nullptr, k_new, v_new, Kc_pool, Vc_pool, 0, len, ring_state, out, workspace,
                      workspace_bytes, (hipStream_t)hip_stream, &cpm);
  }
  const int64_t slot = d->grow_recent ? (int64_t)base + d->n_recent + n_appended : base + n_appended % d->n_recent;
  const int64_t len = d->grow_recent ? slot + 1 : (int64_t)base + d->n_recent;
  if (slot >= d->compact_capacity) return SAGEKV_ERR_INVALID_ARG;
  return run_decode(d, q, nullptr, k_new, v_new, Kc_pool, Vc_pool, (int)slot, (int)len, nullptr, out, workspace,
                    workspace_bytes, (hipStream_t)hip_stream, &cpm);
}

sagekv_status sagekv_decode_step_ring(const sagekv_decode_desc* d, const void* q, const void* k_new, const void* v_new,
                                      void* Kc, void* Vc, int32_t* ring_state, float* out, void* workspace,
                                      size_t workspace_bytes, void* hip_stream) {
  sagekv_status st;
  if (!check_decode(d, &st)) return st;
  if (!q || !k_new || !v_new || !Kc || !Vc || !out || !ring_state) return SAGEKV_ERR_INVALID_ARG;
  const int base = d->n_sink + decode_lists(d) * d->k;
  // the longest row this step can attend (a growing row's length is only known on the device)
  const int len = d->grow_recent ? d->compact_capacity : base + d->n_recent;
  return run_decode(d, q, nullptr, k_new, v_new, Kc, Vc, 0, len, ring_state, out, workspace,
                    workspace_bytes, (hipStream_t)hip_stream);
}

sagekv_status sagekv_decode_step_window(const sagekv_decode_desc* d, const void* q, const void* q_sink,
                                        const void* k_new, const void* v_new, void* Kc, void* Vc, int32_t n_appended,
                                        float* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  sagekv_status st;
  if (!check_decode(d, &st)) return st;
  if (!q || !q_sink || !k_new || !v_new || !Kc || !Vc || !out || n_appended < 0) return SAGEKV_ERR_INVALID_ARG;
  const int base = d->n_sink + decode_lists(d) * d->k;
  const int64_t slot = d->grow_recent ? (int64_t)base + d->n_recent + n_appended : base + n_appended % d->n_recent;
  const int64_t len = d->grow_recent ? slot + 1 : (int64_t)base + d->n_recent;
  if (slot >= d->compact_capacity) return SAGEKV_ERR_INVALID_ARG;
  return run_decode(d, q, q_sink, k_new, v_new, Kc, Vc, (int)slot, (int)len, nullptr, out, workspace, workspace_bytes,
                    (hipStream_t)hip_stream);
}

sagekv_status sagekv_stage_timing_enable(int32_t n_calls) {
  for (hipEvent_t e : g_timing.sel) (void)hipEventDestroy(e);
  for (hipEvent_t e : g_timing.dec) (void)hipEventDestroy(e);
  g_timing.sel.clear();
  g_timing.dec.clear();
  g_timing.sel_mask.clear();
  g_timing.n_calls = 0;
  g_timing.next_select = g_timing.next_decode = 0;
  if (n_calls <= 0) return SAGEKV_OK;
  g_timing.sel.resize((size_t)n_calls * SAGEKV_N_STAGES * 2);
  g_timing.dec.resize((size_t)n_calls * 2);
  g_timing.sel_mask.assign((size_t)n_calls, 0u);
  for (hipEvent_t& e : g_timing.sel)
    if (hipEventCreate(&e) != hipSuccess) return SAGEKV_ERR_DEVICE;
  for (hipEvent_t& e : g_timing.dec)
    if (hipEventCreate(&e) != hipSuccess) return SAGEKV_ERR_DEVICE;
  g_timing.n_calls = n_calls;
  return SAGEKV_OK;
}

sagekv_status sagekv_stage_timing_stages(uint32_t select_stage_mask, int32_t decode) {
  g_timing.stages = select_stage_mask;
  g_timing.decode = decode != 0;
  return SAGEKV_OK;
}

sagekv_status sagekv_stage_timing_read(int32_t which, int32_t call, float* ms) {
  if (!ms || call < 0) return SAGEKV_ERR_INVALID_ARG;
  if (which == 0) {
    if (call >= g_timing.next_select) return SAGEKV_ERR_INVALID_ARG;
    hipEvent_t* ev = &g_timing.sel[(size_t)call * SAGEKV_N_STAGES * 2];
    for (int i = 0; i < SAGEKV_N_STAGES; ++i) {
      ms[i] = 0.f;
      if (!(g_timing.sel_mask[call] & (1u << i))) continue;
      if (hipEventSynchronize(ev[2 * i + 1]) != hipSuccess) return SAGEKV_ERR_DEVICE;
      if (hipEventElapsedTime(&ms[i], ev[2 * i], ev[2 * i + 1]) != hipSuccess) return SAGEKV_ERR_DEVICE;
    }
    return SAGEKV_OK;
  }
  if (which == 1) {
    if (call >= g_timing.next_decode) return SAGEKV_ERR_INVALID_ARG;
    hipEvent_t* ev = &g_timing.dec[(size_t)call * 2];
    if (hipEventSynchronize(ev[1]) != hipSuccess) return SAGEKV_ERR_DEVICE;
    if (hipEventElapsedTime(&ms[0], ev[0], ev[1]) != hipSuccess) return SAGEKV_ERR_DEVICE;
    return SAGEKV_OK;
  }
  return SAGEKV_ERR_INVALID_ARG;
}

}  // extern "C"
