/* freekv_instrument.h -- measurement and test hooks of libfreekv.so.
 *
 * Not part of the retrieval-decode interface (freekv.h): these entry points exist for the benchmark
 * (kernel timers on the launch stream, the cost of an empty launch) and for one test of failure
 * handling (a bounded in-kernel wait that the host makes run out).  A serving loop needs none of them.
 * Same conventions as freekv.h: 0 or a negative FKV_E* code, nothing throws.
 */
#ifndef FREEKV_INSTRUMENT_H
#define FREEKV_INSTRUMENT_H

#include "freekv.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Time the split attention kernel (the dominant HBM reader of the step) with a
 * HIP event pair around each of the next max_launches launches, on the stream it
 * is launched on.  max_launches = 0 switches the timers off.  Blocking. */
int fkv_profile_enable(fkv_ctx* ctx, int32_t max_launches);
/* Sum of the recorded durations (ms) and their number; resets the timers.  Blocking. */
int fkv_profile_read(fkv_ctx* ctx, double* total_ms, int32_t* launches);

/* Launch the attention kernel `reps` times for every layer in turn (ACTIVE selection, the
 * state is not changed), back to back on `stream` between one HIP event pair, and return
 * the elapsed time and the number of launches.  q_dev: layer l's queries at
 * q_dev + l * q_layer_stride bytes.  out_dev: [batch, n_q, d] fp32 scratch output.  Blocking. */
int fkv_profile_attn(fkv_ctx* ctx, const void* q_dev, size_t q_layer_stride, float* out_dev, int32_t reps,
                     void* stream, double* total_ms, int32_t* launches);

/* The same for the page-weight scan and the selection (Sec. 3.2) as fkv_page_select launches them: `reps`
 * times for every layer in turn between one HIP event pair; `launches` receives the kernel launches made
 * (one per call when the selection rides in the scoring launch, more otherwise).  The layers' PENDING id
 * buffers are overwritten; no other state changes.  Blocking. */
int fkv_profile_select(fkv_ctx* ctx, const void* q_dev, size_t q_layer_stride, int32_t reps, void* stream,
                       double* total_ms, int32_t* launches);

/* The cost of a launch as such: `reps` launches, back to back on `stream` between one HIP event
 * pair, of a kernel with the grid, block size and dynamic LDS of `layer`'s last one-launch
 * layer-step whose blocks return at once.  FKV_ESTATE if that step took several launches.
 * grid / lds_bytes (may be NULL) receive the shape.  Blocking. */
int fkv_profile_launch_floor(fkv_ctx* ctx, int32_t layer, int32_t reps, void* stream, double* total_ms,
                             int32_t* grid, int32_t* lds_bytes);

/* Test hook for the bounded wait of the one-launch layer-step: while on, the attention waves of a
 * corrected head wait for picked page ids tagged with an epoch that never comes (the host asks them to
 * wait for the wrong one).  Every kernel still ends; the wait runs out after about 0.1 s, the head's
 * output rows are NaN and fkv_health reports FKV_ETIMEOUT.  Host-side switch, no GPU work. */
int fkv_test_lose_selection(fkv_ctx* ctx, int32_t on);

/* While on, kernels record 100 MHz phase timestamps of head 0 (read with FKV_DBG_TSTAMP). */
int fkv_instrument_timestamps(fkv_ctx* ctx, int32_t on);

#ifdef __cplusplus
}
#endif
#endif /* FREEKV_INSTRUMENT_H */
