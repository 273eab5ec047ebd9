/*
 * mtfm_hta_timing.h -- optional instrumentation of libmtfm_hta.so for benchmarks and profiling: HIP event pairs
 * recorded by the library around each kernel it enqueues.  Not part of the attention interface (mtfm_hta.h) and not
 * bound by its contract: mtfm_hta_timing_read() blocks on its events, and the state is process-wide.  Off unless
 * switched on; while off, the attention calls record nothing.
 */
#ifndef MTFM_HTA_TIMING_H
#define MTFM_HTA_TIMING_H

#include "mtfm_hta.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Per-kernel timing.  mtfm_hta_timing_enable(slots) creates `slots`
 * HIP event pairs per kernel kind (slots <= 0: destroy them and switch timing off, the default).  While
 * on, every call records an event pair on its stream around each kernel it enqueues, into a ring of
 * `slots` entries per kind.  mtfm_hta_timing_read() waits for the recorded events of one kind (this is
 * the only blocking call of the library), writes up to `capacity` durations in milliseconds to the HOST
 * array `ms`, oldest first, empties that ring and returns how many it wrote (or a negative status).
 * Process-wide state; not meant to be toggled while another thread is inside a call.
 */
enum { MTFM_HTA_KERNEL_FWD = 0,      /* forward attention kernel */
       MTFM_HTA_KERNEL_BWD_SELF = 1, /* dk/dv of the target tokens' own keys: no launch of its own any more (its blocks
                                        ride at the end of the BWD_DQ grid), never recorded */
       MTFM_HTA_KERNEL_BWD_DQ = 2,   /* dq (row-stationary pass; the whole backward of the fp32 path) */
       MTFM_HTA_KERNEL_BWD_DKDV = 3, /* dk, dv of the history keys (key-stationary pass) */
       MTFM_HTA_N_KERNELS = 7        /* kinds 4..6 belong to mtfm_gln.h */ };
MTFM_HTA_API int mtfm_hta_timing_enable(int slots);
MTFM_HTA_API int mtfm_hta_timing_read(int kernel, float* ms, int capacity);

#ifdef __cplusplus
}
#endif
#endif /* MTFM_HTA_TIMING_H */
