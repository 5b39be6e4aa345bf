/*
 * so_adam_aux.h -- measurement and testing aids of the Adam(W) bucket-step library.
 *
 * Nothing here is part of the optimizer path declared in so_adam.h: these calls only time the
 * step kernels on the stream they are launched on (the benchmark's roofline figure) and let a
 * test exercise the code that cuts one step into several launches without allocating
 * 17 billion elements.  Same conventions as so_adam.h.
 */
#ifndef SO_ADAM_AUX_H
#define SO_ADAM_AUX_H

#include "so_adam.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Measurement aid: with profiling enabled every step-kernel launch (so_adam_step,
 * so_adam_step_multi, so_adam_step_guarded) is bracketed by a HIP event pair on the context's
 * stream.  so_read_step_kernel_ms waits for the recorded launches, writes their durations in
 * milliseconds (launch order) to ms_out[0..cap), the count to *n_out, and starts over. */
so_status so_set_profiling(so_ctx* ctx, int enable);
so_status so_read_step_kernel_ms(so_ctx* ctx, double* ms_out, size_t cap, size_t* n_out);

/* Testing aid: lower the size of one step launch -- workgroups (256-element tiles) per grid
 * row and rows (buckets) per two-dimensional grid -- so that the paths which cut a step into
 * several launches run at small sizes.  0 restores a limit to the hardware's; values above
 * it are SO_ERR_INVALID_ARG.  The state a step produces never depends on these limits. */
so_status so_set_limits(so_ctx* ctx, uint64_t max_grid_workgroups, uint32_t max_grid_rows);

#ifdef __cplusplus
}
#endif
#endif /* SO_ADAM_AUX_H */
