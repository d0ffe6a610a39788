/*
 * flare_profile.h -- per-kernel timing hooks of libflare.so, for measurement (bench.py); not part of the
 * operator's interface in flare.h.
 */
#ifndef FLARE_PROFILE_H
#define FLARE_PROFILE_H

#ifdef __cplusplus
extern "C" {
#endif

/*
 * While enabled, every kernel
 * the library launches is bracketed by a pair of HIP events recorded on the launch stream.
 * flare_profile_enable(1) creates the event pool (the only allocation this library makes) and
 * clears the totals; flare_profile_enable(0) stops recording.  flare_profile_kernels() returns
 * how many kernel ids exist; flare_profile_name(id) names one; flare_profile_read(id, ...)
 * waits for the recorded events and returns the summed duration in milliseconds and the
 * number of launches since enabling.  At most 8192 launches are recorded; later ones run
 * untimed.  Not thread-safe.
 */
int flare_profile_enable(int on);
int flare_profile_kernels(void);
const char *flare_profile_name(int kernel_id);
int flare_profile_read(int kernel_id, double *total_ms, int *launches);

#ifdef __cplusplus
}
#endif
#endif /* FLARE_PROFILE_H */
