/* sagekv.h - C ABI of the MI355X (gfx950) SAGE-KV hot path.
 *
 * SAGE-KV (arXiv 2503.08879, Sec. 2) compresses a model's KV cache once, after
 * prefill: per layer and head it keeps the first tokens (sink), the most recent
 * tokens and the top-k of the tokens in between, ranked by the attention score
 * of the LAST token's query; decoding then attends over that reduced cache, and
 * every generated token enters the recent window, which evicts its oldest entry.
 *
 * Conventions
 *   - Every data pointer is DEVICE memory owned by the caller (unless a comment
 *     says host).  Descriptors are host structs, read during the call only.
 *   - All work is enqueued on `hip_stream` (a hipStream_t passed as void*, null =
 *     the default stream).  No call allocates, frees or synchronises (the benchmark aids of
 *     sagekv_bench.h that wait for the stream say so).
 *   - Indices are 0-based.  A "problem" is one layer of one sequence; problems are
 *     independent (Sec. 2: selection is done "for each layer").  A "row" is one
 *     (problem, KV head).  G = n_q_heads / n_kv_heads consecutive query heads share
 *     KV head c = h / G (App. A.2's query group number).
 *   - n_recent counts the last prompt token: in the paper's Step 1 notation
 *     n_recent = R + 1, n_sink = S, and L = N.  Candidates for eviction are the
 *     positions [n_sink, L - n_recent).
 *   - Errors are return codes.  Arguments are checked before anything is launched:
 *     on SAGEKV_ERR_INVALID_ARG / _UNSUPPORTED / _WORKSPACE nothing was written.
 *   - One call handles at most 65535 rows (n_problems * n_kv_heads; times G in PER_QUERY selection):
 *     more is SAGEKV_ERR_UNSUPPORTED, split the problems over several calls.
 *   - Element types: bf16 (raw 16-bit patterns) or fp32; head_dim 64 or 128; the
 *     innermost (head_dim) stride is 1 and rows must be 16-byte aligned: base pointers of
 *     caches, queries and workspaces on 16 bytes (else SAGEKV_ERR_UNSUPPORTED), strides in
 *     multiples of 16 bytes.
 */
#ifndef SAGEKV_H
#define SAGEKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SAGEKV_OK = 0,
  SAGEKV_ERR_INVALID_ARG = 1,
  SAGEKV_ERR_UNSUPPORTED = 2,
  SAGEKV_ERR_WORKSPACE = 3,
  SAGEKV_ERR_DEVICE = 4,
  SAGEKV_ERR_SCRATCH_LIMIT = 5 /* sagekv_decode_step_static: the problem needs more than the built-in scratch */
} sagekv_status;

typedef enum { SAGEKV_BF16 = 0, SAGEKV_F32 = 1 } sagekv_dtype;

/* How the G query heads of a KV head are combined before the top-k (Sec. 2 Step 2,
 * "Hq groups of the top-k"; App. A.2).
 *   GROUP_SUM: the heads' softmax probabilities are added and the KV head takes ONE
 *              top-k (the paper prints no operator for this; it is this library's
 *              primary, fastest mode).
 *   PER_QUERY: the paper's literal rule: every query head takes its own top-k of k tokens by
 *              its own probabilities, the KV head stores G lists.  A reduced row is then
 *              [sink | list of head 0 | ... | list of head G-1 | recent], S + G*k + W tokens
 *              (compact_capacity and kept_idx are sized for that; scores_out is
 *              [n_problems, Hq, L]); at decode, head g attends sink + its own list + recent. */
typedef enum { SAGEKV_HEADS_GROUP_SUM = 0, SAGEKV_HEADS_PER_QUERY = 1 } sagekv_head_mode;

/* ---- eviction pass ------------------------------------------------------------------ */
typedef struct {
  int32_t n_problems;          /* layers x sequences                                       */
  int32_t n_q_heads;           /* Hq                                                       */
  int32_t n_kv_heads;          /* Hkv, divides Hq                                          */
  int32_t head_dim;            /* 64 or 128                                                */
  int32_t dtype;               /* sagekv_dtype of q_last, K, V, Kc, Vc                     */
  int32_t head_mode;           /* sagekv_head_mode                                         */
  int64_t L;                   /* cache length, last prompt token included                 */
  int64_t k_stride_problem;    /* strides of K in ELEMENTS: K[p][c][i][j] is at            */
  int64_t k_stride_head;       /*   p*stride_problem + c*stride_head + i*stride_token + j  */
  int64_t k_stride_token;
  int64_t v_stride_problem;    /* the same three for V                                     */
  int64_t v_stride_head;
  int64_t v_stride_token;
  int32_t n_sink;              /* S >= 0                                                   */
  int32_t n_recent;            /* W >= 1, includes the last token                          */
  int32_t k;                   /* middle tokens kept per list, 0 <= k <= L - S - W         */
  int32_t compact_capacity;    /* row pitch (tokens) of Kc / Vc, >= S + lists*k + W        */
  uint32_t flags;              /* 0, or SAGEKV_SELECT_DENSE                                */
} sagekv_select_desc;

/* sagekv_select normally pre-filters: a strided sample of each row gives a conservative score
 * threshold, the pass over K keeps only the tokens that reach it, and the top-k is taken among
 * those; a row whose result cannot be proven equal to the top-k over ALL its candidates is redone
 * by the dense path (every token's score is materialised).  The kept set is the same either way.
 * SAGEKV_SELECT_DENSE forces the dense path for every row; so does a non-null scores_out, an
 * fp32 cache, G > 16, more than 1048576 tokens per row, or a k so large that the pre-filter
 * would have to keep about half of the row (roughly 5 k lists + 8192 > L - S - W). */
enum { SAGEKV_SELECT_DENSE = 1u };

/* Bytes of device scratch sagekv_select needs for this descriptor (0 if it is invalid). */
size_t sagekv_select_workspace_bytes(const sagekv_select_desc* desc);

/* Sec. 2 Steps 1-3.  For every row:
 *   score[i] = sum over the row's G query heads of softmax_i( q_last[h] . K[i] / sqrt(head_dim) ),
 *              the softmax taken over the whole row i in [0, L);
 *   sel      = the k candidates with the largest score (equal scores: lower index first),
 *              in ascending position;
 *   kept     = [0, S) ++ sel ++ [L - W, L);     Kc[t] = K[kept[t]],  Vc[t] = V[kept[t]].
 * In:  q_last [n_problems, Hq, head_dim] contiguous; K, V strided as described above (read only).
 * Out: Kc, Vc [n_problems, Hkv, compact_capacity, head_dim] contiguous, rows [0, S+k+W) written;
 *      kept_idx [n_problems, Hkv, S+k+W] int32;
 *      scores_out (nullable) [n_problems, Hkv, L] fp32 (the scores the selection used).
 * Scores are computed in fp32; the candidates close to the k-th score are re-evaluated in
 * fp64 before the final decision, so the kept set does not depend on fp32 summation order. */
sagekv_status sagekv_select(const sagekv_select_desc* desc, const void* q_last, const void* K, const void* V,
                            void* Kc, void* Vc, int32_t* kept_idx, float* scores_out, void* workspace,
                            size_t workspace_bytes, void* hip_stream);

/* Paged caches (the block-table layout of serving engines; Sec. 2 Step 1 only fixes WHICH tokens
 * form the cache, not where they live).  The tokens of a problem are cut into logical pages of
 * page_size tokens; logical page j of problem p is physical page block_table[p * table_pitch + j]
 * of a pool, and token t of KV head c sits at
 *   pool + page * k_stride_page + c * k_stride_head + (t mod page_size) * k_stride_token   (elements),
 * with desc->k_stride_head / k_stride_token (v_*) now meaning the strides INSIDE a page;
 * desc->k_stride_problem / v_stride_problem are ignored.  All pointers are device pointers. */
typedef struct sagekv_paged_kv {
  const int32_t* block_table; /* [n_problems][table_pitch], entries in [0, n_pages) (clamped to it) */
  int64_t table_pitch;        /* >= ceil(L / page_size) */
  int32_t page_size;          /* tokens per page: a power of two, >= 16 */
  int32_t n_pages;            /* pages in the pool */
  int64_t k_stride_page;      /* elements, multiple of 16 bytes */
  int64_t v_stride_page;
} sagekv_paged_kv;

/* sagekv_select over a paged cache: same selection, same outputs (Kc, Vc dense as above), same
 * workspace size.  K_pool / V_pool are the page pools. */
sagekv_status sagekv_select_paged(const sagekv_select_desc* desc, const sagekv_paged_kv* pages, const void* q_last,
                                  const void* K_pool, const void* V_pool, void* Kc, void* Vc, int32_t* kept_idx,
                                  float* scores_out, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Interval refresh (Sec. 4, future work: "the model periodically refreshes the selected tokens
 * during generation").  The library keeps no state between calls, so a refresh is a second
 * sagekv_select with the CURRENT token's query over the full cache as it stands now.  Contract:
 *   - the caller keeps the full cache (K, V with spare capacity behind L; the stride fields address
 *     it) and stores every generated token's (k, v) at positions L0, L0+1, ... itself: decode calls
 *     only write the reduced cache;
 *   - after T generated tokens, call sagekv_select with L = L0 + T, the query of the newest token
 *     (the one at position L - 1) and the SAME Kc, Vc, kept_idx as before: rows [0, S+lists*k+W) of
 *     every reduced row and of kept_idx are rewritten in full, on the stream, after the decode
 *     steps already enqueued there;
 *   - the recent window is then again positions [L - W, L) in ascending order in slots
 *     [S+lists*k, S+lists*k+W): restart the append count (n_appended = 0 for the next
 *     sagekv_decode_step; with sagekv_decode_step_ring set ring_state[0] = 0 on the
 *     stream);
 *   - a grown row (grow_recent) starts again at length S+lists*k+W. */

/* ---- decoding over the reduced cache -------------------------------------------------- */
typedef struct {
  int32_t n_problems, n_q_heads, n_kv_heads, head_dim;
  int32_t dtype;               /* of q, k_new, v_new, Kc, Vc                                */
  int32_t head_mode;           /* as in the eviction pass that built the cache              */
  int32_t n_sink, k, n_recent; /* layout of a reduced row: [sink | selected | recent window] */
  int32_t compact_capacity;    /* row pitch of Kc / Vc                                      */
  int32_t grow_recent;         /* 0: the paper's fixed-size FIFO window (Step 4)            */
                               /* 1: nothing is evicted, new tokens go to rows S+k+W, ...   */
} sagekv_decode_desc;

/* Step 4's cache update: put (k_new, v_new) [n_problems, Hkv, head_dim] into every reduced row.
 * `n_appended` = how many tokens were appended to this cache before this call (host counter).
 * FIFO: the window is a ring; the new token overwrites its oldest entry, physical slot
 *       S + k + (n_appended mod W).  Attention does not depend on the physical order.
 * grow: slot S + k + W + n_appended, which must be < compact_capacity. */
sagekv_status sagekv_append(const sagekv_decode_desc* desc, const void* k_new, const void* v_new, void* Kc,
                            void* Vc, int32_t n_appended, void* hip_stream);

/* Bytes of device scratch the decode calls need (may be 0: then `workspace` may be null).
 * The scratch needs no initialisation and carries no state between calls. */
size_t sagekv_decode_workspace_bytes(const sagekv_decode_desc* desc);

/* Step 4's attention: out[h] = sum_t softmax_t( q[h] . Kc[c][t] / sqrt(head_dim) ) Vc[c][t],
 * t in [0, len), c = h / G.   q [n_problems, Hq, head_dim]; out [n_problems, Hq, head_dim] fp32.
 * 1 <= len <= compact_capacity.  Logits, softmax and the weighted sum are fp32; with a bf16 cache
 * and more than 4 heads per KV head, or a row split over several workgroups, the softmax weights
 * are rounded to bf16 (like the values they multiply) and the sum runs on the matrix cores. */
sagekv_status sagekv_decode_attn(const sagekv_decode_desc* desc, const void* q, const void* Kc, const void* Vc,
                                 int32_t len, float* out, void* workspace, size_t workspace_bytes,
                                 void* hip_stream);

/* One whole decode step in a single launch: sagekv_append(k_new, v_new, n_appended) followed by
 * sagekv_decode_attn over the updated cache (the new token attends to itself).  The length
 * attended is S+k+W (FIFO) or S+k+W+n_appended+1 (grow). */
sagekv_status sagekv_decode_step(const sagekv_decode_desc* desc, const void* q, const void* k_new,
                                 const void* v_new, void* Kc, void* Vc, int32_t n_appended, float* out,
                                 void* workspace, size_t workspace_bytes, void* hip_stream);

/* sagekv_decode_step with the append count kept ON THE DEVICE (Step 4's FIFO position), so that one
 * recorded launch sequence (a HIP graph of a decode step) serves every generated token.
 * ring_state: device int32[2], owned by the caller.  ring_state[0] = tokens appended so far, read by
 * the launch in place of `n_appended` and increased by one when the step is done; ring_state[1] is
 * the library's arrival counter (it is 0 between calls).  Set both to 0 before the first step;
 * after every sagekv_select into this reduced cache set ring_state[0] to 0 again (stream-ordered,
 * e.g. a fill kernel: a memset node must not be recorded into a graph).  Calls on one ring_state
 * must not overlap.
 * grow_recent: a row that has reached compact_capacity stays as it is (the token is dropped and the
 * count still moves on); the caller sizes compact_capacity for the tokens it will generate. */
sagekv_status sagekv_decode_step_ring(const sagekv_decode_desc* desc, const void* q, const void* k_new,
                                      const void* v_new, void* Kc, void* Vc, int32_t* ring_state, float* out,
                                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* For callers that cannot provide device scratch (code under HIP graph capture that may not call
 * hipMalloc, tight serving loops, harnesses that forbid allocation): sagekv_decode_step with the
 * split partials of a row kept in a scratch array built into the library (device memory that every
 * GPU the library runs on holds until the process ends), SAGEKV_STATIC_SCRATCH_BYTES of it.
 * Allocates nothing and takes no workspace.  A descriptor whose
 * sagekv_decode_workspace_bytes exceeds that size is rejected with SAGEKV_ERR_SCRATCH_LIMIT before
 * anything is launched.  All calls on one GPU share the array: calls that overlap there (two
 * streams, two threads) race; calls on one stream are safe.  The array needs no clearing: every
 * partial a step reads was written by that step. */
enum { SAGEKV_STATIC_SCRATCH_BYTES = 4 * 1024 * 1024 };
sagekv_status sagekv_decode_step_static(const sagekv_decode_desc* desc, const void* q, const void* k_new,
                                        const void* v_new, void* Kc, void* Vc, int32_t n_appended, float* out,
                                        void* hip_stream);

/* ---- reduced cache in pages ------------------------------------------------------------------
 * A serving engine keeps its caches in pages, the reduced one too (Sec. 4: the method plugs into
 * existing inference stacks; Sec. 2 Step 3 only fixes WHICH tokens the reduced cache holds and their
 * order).  With a sagekv_paged_kv for the reduced cache, Kc and Vc are page pools: a page holds
 * [n_kv_heads][page_size][head_dim] elements (contiguous), pages are k_stride_page / v_stride_page
 * elements apart, and token t of a reduced row of problem p, KV head c, sits at
 *   pool + block_table[p * table_pitch + t / page_size] * stride_page + (c * page_size + t % page_size) * head_dim.
 * table_pitch >= ceil(compact_capacity / page_size); page_size a power of two >= 16; the pages of
 * different problems must be distinct.  Everything else is as in the dense calls of the same name. */

/* sagekv_select (in_pages == NULL: K, V strided as in sagekv_select; else pools as in
 * sagekv_select_paged) gathering into a paged reduced cache. */
sagekv_status sagekv_select_into_pages(const sagekv_select_desc* desc, const sagekv_paged_kv* in_pages,
                                       const sagekv_paged_kv* out_pages, const void* q_last, const void* K,
                                       const void* V, void* Kc_pool, void* Vc_pool, int32_t* kept_idx,
                                       float* scores_out, void* workspace, size_t workspace_bytes, void* hip_stream);

/* sagekv_decode_attn over a paged reduced cache. */
sagekv_status sagekv_decode_attn_paged(const sagekv_decode_desc* desc, const sagekv_paged_kv* pages, const void* q,
                                       const void* Kc_pool, const void* Vc_pool, int32_t len, float* out,
                                       void* workspace, size_t workspace_bytes, void* hip_stream);

/* sagekv_decode_step over a paged reduced cache: the new token is stored in the page that holds its
 * ring slot.  ring_state == NULL: `n_appended` counts the appended tokens (as in sagekv_decode_step);
 * else the count lives on the device (as in sagekv_decode_step_ring) and n_appended is ignored. */
sagekv_status sagekv_decode_step_paged(const sagekv_decode_desc* desc, const sagekv_paged_kv* pages, const void* q,
                                       const void* k_new, const void* v_new, void* Kc_pool, void* Vc_pool,
                                       int32_t n_appended, int32_t* ring_state, float* out, void* workspace,
                                       size_t workspace_bytes, void* hip_stream);

/* Window-relative rotary positions (the StreamLLM_R cache mode of Sec. 3.1, baseline (3a), App. A.1:
 * the entry at index i of a window of n entries has position i, the query position n-1, so
 * positions stay bounded however long the generation runs).  Rotary attention depends on position
 * differences only, so the mode needs no re-rotation of the cache when the window slides: keep the
 * keys rotated at their ABSOLUTE positions (the usual cache), pass
 *   q      = the query rotated at its absolute position (recent tokens: the distance to a recent
 *            token is the same in window and in absolute positions), and
 *   q_sink = the query rotated at position n-1 = S+k+W-1 (a sink token's absolute position IS its
 *            window position, so only the query's position differs),
 * and the sink tokens [0, n_sink) are scored with q_sink, every other token with q.  The rotation
 * itself belongs to the model around the cache and is not done here.  Everything else is as in
 * sagekv_decode_attn / sagekv_decode_step; q_sink [n_problems, Hq, head_dim] must not be null. */
sagekv_status sagekv_decode_attn_window(const sagekv_decode_desc* desc, const void* q, const void* q_sink,
                                        const void* Kc, const void* Vc, int32_t len, float* out, void* workspace,
                                        size_t workspace_bytes, void* hip_stream);
sagekv_status sagekv_decode_step_window(const sagekv_decode_desc* desc, const void* q, const void* q_sink,
                                        const void* k_new, const void* v_new, void* Kc, void* Vc,
                                        int32_t n_appended, float* out, void* workspace, size_t workspace_bytes,
                                        void* hip_stream);

/* ---- misc ---------------------------------------------------------------------------------- */
const char* sagekv_status_string(sagekv_status s); /* host string, static storage */

/* The paper's split of a per-KV-head budget of B tokens for PER_QUERY selection (App. A.2):
 * n_sink = B/4, k per query head = B/(2G) rounded down to a power of two (the two cases the
 * appendix prints, G = 4 -> 1024 and G = 7 -> 512 at B = 8192, fix the rounding), n_recent =
 * what is left, so that n_sink + G*k + n_recent = B.  Host only, touches no device.  G = query
 * heads per KV head.  INVALID_ARG (outputs untouched) for null outputs, G < 1 or B < 4*G (no room
 * for one token per head). */
sagekv_status sagekv_paper_budget(int32_t B, int32_t G, int32_t* n_sink, int32_t* k, int32_t* n_recent);

#ifdef __cplusplus
}
#endif
#endif
