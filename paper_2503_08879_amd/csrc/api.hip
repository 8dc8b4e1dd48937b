// C ABI of the library: argument checks, workspace layout, launch order.
#include "../../include/sagekv.h"

#include <math.h>
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

struct SelectLayout {
  size_t logits, scores, partials, stats, ghist, total;
  int64_t Lp;
  int n_chunks, rows, G;
};

bool check_select(const sagekv_select_desc* d, sagekv_status* st) {
  *st = SAGEKV_ERR_INVALID_ARG;
  if (!d) return false;
  if (d->n_problems < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->n_q_heads % d->n_kv_heads) return false;
  if (d->L < 1 || d->L > 0x7FFFFFF0ll) return false;
  if (d->n_sink < 0 || d->n_recent < 1 || d->k < 0) return false;
  if ((int64_t)d->n_sink + d->n_recent + d->k > d->L) return false;
  if ((int64_t)d->compact_capacity < (int64_t)d->n_sink + d->n_recent + d->k) return false;
  if ((int64_t)d->n_problems * d->n_kv_heads > 65535) return false;
  *st = SAGEKV_ERR_UNSUPPORTED;
  if (d->dtype != SAGEKV_BF16 && d->dtype != SAGEKV_F32) return false;
  if (d->head_dim != 64 && d->head_dim != 128) return false;
  if (d->head_mode != SAGEKV_HEADS_GROUP_SUM) return false;
  if (d->n_q_heads / d->n_kv_heads > 64) return false;
  const int epl = d->dtype == SAGEKV_BF16 ? 8 : 4;  // 16-byte alignment of every token row
  const int64_t strides[6] = {d->k_stride_problem, d->k_stride_head, d->k_stride_token,
                              d->v_stride_problem, d->v_stride_head, d->v_stride_token};
  for (int i = 0; i < 6; ++i)
    if (strides[i] < 0 || strides[i] % epl) return false;
  if (d->k_stride_token < d->head_dim || d->v_stride_token < d->head_dim) return false;
  *st = SAGEKV_OK;
  return true;
}

SelectLayout select_layout(const sagekv_select_desc* d, bool own_scores) {
  SelectLayout l;
  l.rows = d->n_problems * d->n_kv_heads;
  l.G = d->n_q_heads / d->n_kv_heads;
  l.Lp = (d->L + 3) / 4 * 4;
  l.n_chunks = (int)((d->L + kScoreChunk - 1) / kScoreChunk);
  size_t off = 0;
  l.logits = off;
  off = align_up(off + (size_t)l.rows * l.n_chunks * l.G * kScoreChunk * sizeof(float));
  l.scores = off;
  if (own_scores) off = align_up(off + (size_t)l.rows * l.Lp * sizeof(float));
  l.partials = off;
  off = align_up(off + (size_t)l.rows * l.G * l.n_chunks * sizeof(float2));
  l.stats = off;
  off = align_up(off + (size_t)l.rows * l.G * sizeof(RowStat));
  l.ghist = off;
  off = align_up(off + (size_t)l.rows * kHistBins * sizeof(int));
  l.total = off;
  return l;
}

bool check_decode(const sagekv_decode_desc* d, sagekv_status* st) {
  *st = SAGEKV_ERR_INVALID_ARG;
  if (!d) return false;
  if (d->n_problems < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->n_q_heads % d->n_kv_heads) return false;
  if (d->n_sink < 0 || d->n_recent < 1 || d->k < 0) return false;
  if ((int64_t)d->compact_capacity < (int64_t)d->n_sink + d->n_recent + d->k) return false;
  if ((int64_t)d->n_problems * d->n_kv_heads > 65535) return false;
  *st = SAGEKV_ERR_UNSUPPORTED;
  if (d->dtype != SAGEKV_BF16 && d->dtype != SAGEKV_F32) return false;
  if (d->head_dim != 64 && d->head_dim != 128) return false;
  if (d->head_mode != SAGEKV_HEADS_GROUP_SUM) return false;
  *st = SAGEKV_OK;
  return true;
}

struct DecodeLayout {
  size_t part_ml, part_acc, total;
  int max_splits, rows, G;
};

// Splits per row.  With about one row per CU or more, a single 16-wave workgroup per row fills
// the chip and needs no merge launch; otherwise enough workgroups to fill 256 CUs several times
// over, at least 256 tokens each.
int splits_for(int rows, int len) {
  if (rows >= 192) return 1;
  int want = (2048 + rows - 1) / rows;
  int most = (len + 255) / 256;
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
} g_timing;

struct StageTimer {
  hipEvent_t* ev = nullptr;
  hipStream_t s;
  StageTimer(int which, hipStream_t stream) : s(stream) {
    if (g_timing.n_calls == 0) return;
    if (which == 0 && g_timing.next_select < g_timing.n_calls)
      ev = &g_timing.sel[(size_t)g_timing.next_select++ * SAGEKV_N_STAGES * 2];
    if (which == 1 && g_timing.next_decode < g_timing.n_calls) ev = &g_timing.dec[(size_t)g_timing.next_decode++ * 2];
  }
  void begin(int stage) {
    if (ev) (void)hipEventRecord(ev[stage * 2], s);
  }
  void end(int stage) {
    if (ev) (void)hipEventRecord(ev[stage * 2 + 1], s);
  }
};

sagekv_status dev(hipError_t e) { return e == hipSuccess ? SAGEKV_OK : SAGEKV_ERR_DEVICE; }

sagekv_status run_decode(const sagekv_decode_desc* d, const void* q, const void* k_new, const void* v_new,
                         void* Kc, void* Vc, int slot, int len, float* out, void* ws, size_t ws_bytes,
                         hipStream_t s) {
  const DecodeLayout l = decode_layout(d);
  if (l.total > 0 && (!ws || ws_bytes < l.total)) return SAGEKV_ERR_WORKSPACE;
  DecodeParams p;
  p.n_problems = d->n_problems;
  p.Hq = d->n_q_heads;
  p.Hkv = d->n_kv_heads;
  p.G = l.G;
  p.D = d->head_dim;
  p.dtype = d->dtype;
  p.q = q;
  p.Kc = Kc;
  p.Vc = Vc;
  p.k_new = k_new;
  p.v_new = v_new;
  p.slot = slot;
  p.len = len;
  p.cap = d->compact_capacity;
  p.n_splits = splits_for(l.rows, len);
  if (p.n_splits > l.max_splits) p.n_splits = l.max_splits;
  const int tps = (len + p.n_splits - 1) / p.n_splits;
  p.tokens_per_split = (tps + 63) / 64 * 64;
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

const char* sagekv_status_string(sagekv_status s) {
  switch (s) {
    case SAGEKV_OK: return "ok";
    case SAGEKV_ERR_INVALID_ARG: return "invalid argument";
    case SAGEKV_ERR_UNSUPPORTED: return "unsupported configuration";
    case SAGEKV_ERR_WORKSPACE: return "workspace missing or too small";
    case SAGEKV_ERR_DEVICE: return "HIP launch failed";
  }
  return "unknown status";
}

size_t sagekv_select_workspace_bytes(const sagekv_select_desc* desc) {
  sagekv_status st;
  if (!check_select(desc, &st)) return 0;
  return select_layout(desc, true).total;
}

sagekv_status sagekv_select(const sagekv_select_desc* d, const void* q_last, const void* K, const void* V, void* Kc,
                            void* Vc, int32_t* kept_idx, float* scores_out, void* workspace, size_t workspace_bytes,
                            void* hip_stream) {
  sagekv_status st;
  if (!check_select(d, &st)) return st;
  if (!q_last || !K || !V || !Kc || !Vc || !kept_idx) return SAGEKV_ERR_INVALID_ARG;
  const SelectLayout l = select_layout(d, scores_out == nullptr);
  if (!workspace || workspace_bytes < l.total) return SAGEKV_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;

  RowGeom geo;
  geo.n_problems = d->n_problems;
  geo.Hq = d->n_q_heads;
  geo.Hkv = d->n_kv_heads;
  geo.G = l.G;
  geo.D = d->head_dim;
  geo.dtype = d->dtype;
  geo.L = d->L;
  geo.Lp = l.Lp;

  float* logits = (float*)(ws + l.logits);
  float* scores = scores_out ? scores_out : (float*)(ws + l.scores);
  const int64_t pitch = scores_out ? d->L : l.Lp;
  float2* partials = (float2*)(ws + l.partials);
  RowStat* stats = (RowStat*)(ws + l.stats);
  int* ghist = (int*)(ws + l.ghist);

  StageTimer t(0, s);
  hipError_t e;

  ScoreParams sp;
  sp.geo = geo;
  sp.q_last = q_last;
  sp.K = K;
  sp.ks_problem = d->k_stride_problem;
  sp.ks_head = d->k_stride_head;
  sp.ks_token = d->k_stride_token;
  sp.logits = logits;
  sp.partials = partials;
  sp.n_chunks = l.n_chunks;
  sp.g0 = 0;
  sp.scale = (float)(1.0 / sqrt((double)d->head_dim));
  t.begin(SAGEKV_STAGE_SCORE);
  e = launch_score(sp, s);
  t.end(SAGEKV_STAGE_SCORE);
  if (e != hipSuccess) return SAGEKV_ERR_DEVICE;

  StatsParams tp;
  tp.partials = partials;
  tp.stats = stats;
  tp.ghist = ghist;
  tp.G = l.G;
  tp.n_chunks = l.n_chunks;
  t.begin(SAGEKV_STAGE_STATS);
  e = launch_stats(tp, l.rows, s);
  t.end(SAGEKV_STAGE_STATS);
  if (e != hipSuccess) return SAGEKV_ERR_DEVICE;

  CombineParams cp;
  cp.geo = geo;
  cp.logits = logits;
  cp.n_chunks = l.n_chunks;
  cp.stats = stats;
  cp.scores = scores;
  cp.pitch = pitch;
  cp.ghist = ghist;
  cp.S = d->n_sink;
  cp.W = d->n_recent;
  t.begin(SAGEKV_STAGE_COMBINE);
  e = launch_combine(cp, s);
  t.end(SAGEKV_STAGE_COMBINE);
  if (e != hipSuccess) return SAGEKV_ERR_DEVICE;

  TopkParams kp;
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
  kp.kept_idx = kept_idx;
  kp.S = d->n_sink;
  kp.W = d->n_recent;
  kp.k = d->k;
  kp.band = kBand;
  t.begin(SAGEKV_STAGE_TOPK);
  e = launch_topk(kp, s);
  t.end(SAGEKV_STAGE_TOPK);
  if (e != hipSuccess) return SAGEKV_ERR_DEVICE;

  GatherParams gp;
  gp.geo = geo;
  gp.K = K;
  gp.V = V;
  gp.ks_problem = d->k_stride_problem;
  gp.ks_head = d->k_stride_head;
  gp.ks_token = d->k_stride_token;
  gp.vs_problem = d->v_stride_problem;
  gp.vs_head = d->v_stride_head;
  gp.vs_token = d->v_stride_token;
  gp.kept_idx = kept_idx;
  gp.Kc = Kc;
  gp.Vc = Vc;
  gp.n_kept = d->n_sink + d->k + d->n_recent;
  gp.cap = d->compact_capacity;
  t.begin(SAGEKV_STAGE_GATHER);
  e = launch_gather(gp, s);
  t.end(SAGEKV_STAGE_GATHER);
  return dev(e);
}

sagekv_status sagekv_append(const sagekv_decode_desc* d, const void* k_new, const void* v_new, void* Kc, void* Vc,
                            int32_t n_appended, void* hip_stream) {
  sagekv_status st;
  if (!check_decode(d, &st)) return st;
  if (!k_new || !v_new || !Kc || !Vc || n_appended < 0) return SAGEKV_ERR_INVALID_ARG;
  const int base = d->n_sink + d->k;
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
  return run_decode(d, q, nullptr, nullptr, const_cast<void*>(Kc), const_cast<void*>(Vc), -1, len, out, workspace,
                    workspace_bytes, (hipStream_t)hip_stream);
}

sagekv_status sagekv_decode_step(const sagekv_decode_desc* d, const void* q, const void* k_new, const void* v_new,
                                 void* Kc, void* Vc, int32_t n_appended, float* out, void* workspace,
                                 size_t workspace_bytes, void* hip_stream) {
  sagekv_status st;
  if (!check_decode(d, &st)) return st;
  if (!q || !k_new || !v_new || !Kc || !Vc || !out || n_appended < 0) return SAGEKV_ERR_INVALID_ARG;
  const int base = d->n_sink + d->k;
  const int64_t slot = d->grow_recent ? (int64_t)base + d->n_recent + n_appended : base + n_appended % d->n_recent;
  const int64_t len = d->grow_recent ? slot + 1 : (int64_t)base + d->n_recent;
  if (slot >= d->compact_capacity) return SAGEKV_ERR_INVALID_ARG;
  return run_decode(d, q, k_new, v_new, Kc, Vc, (int)slot, (int)len, out, workspace, workspace_bytes,
                    (hipStream_t)hip_stream);
}

sagekv_status sagekv_stage_timing_enable(int32_t n_calls) {
  for (hipEvent_t e : g_timing.sel) (void)hipEventDestroy(e);
  for (hipEvent_t e : g_timing.dec) (void)hipEventDestroy(e);
  g_timing.sel.clear();
  g_timing.dec.clear();
  g_timing.n_calls = 0;
  g_timing.next_select = g_timing.next_decode = 0;
  if (n_calls <= 0) return SAGEKV_OK;
  g_timing.sel.resize((size_t)n_calls * SAGEKV_N_STAGES * 2);
  g_timing.dec.resize((size_t)n_calls * 2);
  for (hipEvent_t& e : g_timing.sel)
    if (hipEventCreate(&e) != hipSuccess) return SAGEKV_ERR_DEVICE;
  for (hipEvent_t& e : g_timing.dec)
    if (hipEventCreate(&e) != hipSuccess) return SAGEKV_ERR_DEVICE;
  g_timing.n_calls = n_calls;
  return SAGEKV_OK;
}

sagekv_status sagekv_stage_timing_read(int32_t which, int32_t call, float* ms) {
  if (!ms || call < 0) return SAGEKV_ERR_INVALID_ARG;
  if (which == 0) {
    if (call >= g_timing.next_select) return SAGEKV_ERR_INVALID_ARG;
    hipEvent_t* ev = &g_timing.sel[(size_t)call * SAGEKV_N_STAGES * 2];
    for (int i = 0; i < SAGEKV_N_STAGES; ++i) {
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
