/*
 * flowmm_profile.h - measurement support of libflowmm.so (no part of the method; the benchmark
 * uses it to time single kernels inside a pass).
 *
 * The library can bracket chosen kernels with HIP events on the launch stream.
 * flowmm_profile_select: names = "all", "" / NULL (off, the default) or a comma-separated list
 *   of kernel names as returned by flowmm_profile_kernel_name(0 .. count-1).  Process-wide.
 * flowmm_profile_collect: waits for the recorded events (host-side wait on those events only),
 *   adds up milliseconds and launch counts per kernel id into the two host arrays (each
 *   flowmm_profile_kernel_count() long, either may be NULL) and forgets the records.
 * While any kernel is selected the library creates HIP events; do not select kernels around
 * calls that are being captured into a HIP graph.
 */
#ifndef FLOWMM_PROFILE_H
#define FLOWMM_PROFILE_H

#include "flowmm.h"

#ifdef __cplusplus
extern "C" {
#endif

int flowmm_profile_kernel_count(void);
const char *flowmm_profile_kernel_name(int id);
void flowmm_profile_select(const char *names);
flowmm_status flowmm_profile_collect(double *total_ms, long long *launches);

#ifdef __cplusplus
}
#endif
#endif /* FLOWMM_PROFILE_H */
