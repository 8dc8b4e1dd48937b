/* sagekv_bench.h - measurement aids of libsagekv.so, apart from the method's calls (sagekv.h).
 *
 * Nothing here belongs in a serving loop: the calls keep process-wide host state (not thread safe)
 * or wait for the stream.  bench.py and the tests use them to time single stages with HIP events
 * recorded on the call's own stream and to see how many rows the pre-filtered eviction path had to
 * hand to the dense path.
 */
#ifndef SAGEKV_BENCH_H
#define SAGEKV_BENCH_H

#include "sagekv.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Waits for the stream, then reports how many rows of the LAST sagekv_select
 * call that used this workspace were redone by the dense path (-1 if the call was dense anyway).
 * `n_rows` is a host pointer. */
sagekv_status sagekv_select_redone_rows(const sagekv_select_desc* desc, const void* workspace,
                                        size_t workspace_bytes, void* hip_stream, int32_t* n_rows);

/* Stage timing for benchmarks (host-side state, per process; not thread safe).
 * sagekv_stage_timing_enable(n) creates HIP events for the next n instrumented calls of
 * sagekv_select and n of sagekv_decode_attn / sagekv_decode_step (n = 0 switches it off and
 * destroys the events).  While enabled, each call records an event pair around every stage's
 * launches on the call's own stream.  sagekv_stage_timing_read(which, call, ms) waits for that
 * call's events and returns the elapsed milliseconds per stage: which = 0 reads a select call
 * (ms[0 .. SAGEKV_N_STAGES), 0 for a stage the call did not run), which = 1 a decode call (ms[0] only). */
enum { SAGEKV_STAGE_SAMPLE = 0, SAGEKV_STAGE_SCORE = 1, SAGEKV_STAGE_STATS = 2, SAGEKV_STAGE_COMBINE = 3,
       SAGEKV_STAGE_TOPK = 4, SAGEKV_STAGE_REDO = 5, SAGEKV_STAGE_GATHER = 6, SAGEKV_N_STAGES = 7 };
sagekv_status sagekv_stage_timing_enable(int32_t n_calls);
sagekv_status sagekv_stage_timing_read(int32_t which, int32_t call, float* ms /* host */);
/* Every event record leaves the GPU idle for some microseconds between two kernels (measured ~10 us
 * on MI355X), so a fully instrumented eviction pass is ~3 % slower than a plain one.  This restricts
 * the stages of sagekv_select that are bracketed (bit i = stage i; default: all) and says whether
 * decode calls are (decode != 0; default: yes).  Takes effect for the calls that follow. */
sagekv_status sagekv_stage_timing_stages(uint32_t select_stage_mask, int32_t decode);

#ifdef __cplusplus
}
#endif
#endif
