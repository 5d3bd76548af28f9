/*
 * libdmmv - measurement hooks.  Not part of the library's functional surface (include/dmmv.h):
 * the benchmark uses them to time a kernel of the hot path in isolation with HIP events on the
 * handle's own stream.
 */
#ifndef DMMV_BENCH_H
#define DMMV_BENCH_H

#include "dmmv.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Enqueue the evaluation step of the descent (every kernel of it: the step that streams all of A
 * and leaves the arg-min records, the "evaluate all candidates in bulk" step of the paper's
 * section "GPU Acceleration") `reps` times back to back between two HIP events on the handle's
 * stream and return the elapsed time in milliseconds in *ms_out (HOST).  One untimed launch
 * precedes the timed ones.  reps < 0: -reps timed launches WITHOUT the untimed one, for a
 * measurement that starts from whatever the caller left in the caches (say, after a large copy).
 * The state is not changed.  Needs a residual.  Waits for the stream. */
dmmv_status dmmv_time_eval(dmmv_handle h, int32_t reps, float* ms_out);

/* The same for the contraction g = A^T r behind dmmv_l2_changes (for a batch G = X^T R_mat, on the
 * matrix cores for fp32): `reps` launches between two events after one untimed launch.  The handle
 * must have been created with options.l2_rule != 0 and needs a residual.  Waits for the stream. */
dmmv_status dmmv_time_l2(dmmv_handle h, int32_t reps, float* ms_out);

/* Which loop dmmv_solve runs on this handle: 1 = launches per iteration, 2 = all iterations in one
 * launch (options.dense_loop, resolved: the automatic choice depends on the instance and on the
 * device's number of compute units; a handle on a batch with options.prune in effect also
 * answers 2).  HOST query, no GPU work. */
int32_t dmmv_loop_in_use(dmmv_handle h);

#ifdef __cplusplus
}
#endif
#endif /* DMMV_BENCH_H */
