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

struct ScoreParams {
  RowGeom geo;
  const void* q_last;
  const void* K;
  int64_t ks_problem, ks_head, ks_token;  // elements
  float* logits;                          // [rows][n_chunks][G][kScoreChunk]
  float2* partials;                       // [rows][G][n_chunks]  (max, sum exp(x - max))
  int n_chunks;
  int g0;  // first head of the group handled by this launch
  float scale;
};

struct StatsParams {
  const float2* partials;
  RowStat* stats;  // [rows][G]
  int* ghist;      // [rows][kHistBins], zeroed here
  int G, n_chunks;
};

struct CombineParams {
  RowGeom geo;
  const float* logits;
  int n_chunks;  // score chunks per row (logit scratch layout)
  const RowStat* stats;
  float* scores;  // [rows][pitch]
  int64_t pitch;
  int* ghist;
  int S, W;
};

struct TopkParams {
  RowGeom geo;
  float* scores;
  int64_t pitch;
  const int* ghist;
  const RowStat* stats;
  const void* q_last;
  const void* K;
  int64_t ks_problem, ks_head, ks_token;
  int32_t* kept_idx;  // [rows][S + k + W]
  int S, W, k;
  float band;  // relative half-width of the fp64 re-evaluation band around the k-th score
};

struct GatherParams {
  RowGeom geo;
  const void* K;
  const void* V;
  int64_t ks_problem, ks_head, ks_token, vs_problem, vs_head, vs_token;
  const int32_t* kept_idx;
  void* Kc;
  void* Vc;
  int n_kept, cap;
};

struct DecodeParams {
  int n_problems, Hq, Hkv, G, D, dtype;
  const void* q;       // [P][Hq][D]
  void* Kc;            // [rows][cap][D]
  void* Vc;
  const void* k_new;   // nullable: [rows][D]
  const void* v_new;
  int slot;            // row position the new token takes, -1 = no append
  int len, cap;
  int n_splits, tokens_per_split;
  float* part_acc;     // [rows][n_splits][G][D]
  float2* part_ml;     // [rows][n_splits][G]   (max, sum)
  float* out;          // [P][Hq][D]
  float scale;
};

hipError_t launch_score(const ScoreParams& p, hipStream_t s);
hipError_t launch_stats(const StatsParams& p, int rows, hipStream_t s);
hipError_t launch_combine(const CombineParams& p, hipStream_t s);
hipError_t launch_topk(const TopkParams& p, hipStream_t s);
hipError_t launch_gather(const GatherParams& p, hipStream_t s);
hipError_t launch_decode(const DecodeParams& p, hipStream_t s);
hipError_t launch_append(const DecodeParams& p, hipStream_t s);
hipError_t launch_fill_zero(void* ptr, size_t bytes, hipStream_t s);

int max_group_per_launch();  // heads of a group one score / decode launch can hold in registers

}  // namespace sagekv
