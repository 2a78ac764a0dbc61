/*
 * lasp_profile.h -- per-kernel timing of the calls of lasp.h, for benchmarks.
 *
 * A diagnostic beside the method's entry points (lasp.h), kept apart from them:
 * it measures, it computes nothing of the method. It keeps one process-wide
 * recording state, so it is NOT thread-safe and at most one recording can be
 * open at a time; the entry points of lasp.h themselves keep no state.
 */
#ifndef LASP_PROFILE_H
#define LASP_PROFILE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Between lasp_profile_begin and lasp_profile_end every
 * lasp_fwd / lasp_bwd call records HIP events around its three kernels on the
 * stream it launches on (no synchronisation is added), for at most max_calls
 * calls of each kind. lasp_profile_end waits for the recorded events, writes
 * the summed milliseconds per kernel
 *     ms_sum[0..2] = forward  {local pass, scan, tile walk}
 *     ms_sum[3..5] = backward {local pass, scan, tile walk}
 * and the number of recorded calls, and releases the events. The bidirectional
 * calls record too: lasp_bidir_state as a forward call (reduction under "local
 * pass", sum of the partials under "scan"), lasp_bidir_fwd as a forward call and
 * lasp_bidir_bwd as a backward call (their one kernel under "tile walk").
 * begin: LASP_ERR_SHAPE if max_calls <= 0 or profiling is already on,
 * LASP_ERR_HIP if events cannot be created. end: LASP_ERR_NULL on NULL
 * arguments, LASP_ERR_SHAPE if profiling is off.
 */
int lasp_profile_begin(int32_t max_calls);
int lasp_profile_end(double ms_sum[6], int32_t *fwd_calls, int32_t *bwd_calls);

#ifdef __cplusplus
}
#endif
#endif /* LASP_PROFILE_H */
