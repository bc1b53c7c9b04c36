/*
 * lss_timing.h -- benchmark-only instrumentation of liblss_attn.so; not part of the
 * library's product interface (include/lss_attn.h) and not part of the paper's method.
 *
 * While enabled, every kernel the library launches is bracketed by a pair of HIP events
 * on its launch stream.  Kernel ids are small integers; lss_timing_kernel_name(id) is the
 * base name of the __global__ function that id stands for, as a profiler prints it
 * (without namespace and template arguments).
 *   lss_timing_enable(on)   switch recording on (1) or off (0) for every kernel; off by default
 *   lss_timing_select(mask) record only the kernels whose id bit is set in `mask` (0 = none)
 *   lss_timing_reset()      wait for outstanding events and zero the totals
 *   lss_timing_read(id, &total_ms, &launches)
 *                           wait for outstanding events (blocks the host until those kernels
 *                           are done), then return the summed duration and launch count of
 *                           kernel `id` since the last reset; host pointers
 *   lss_timing_kernel_name(id)  name of kernel `id` (0, 1, ...), NULL past the last one
 * Not thread-safe against concurrent reads; returns LSS_OK or a negative lss_status.
 */
#ifndef LSS_TIMING_H
#define LSS_TIMING_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

int lss_timing_enable(int on);
int lss_timing_select(uint64_t kernel_mask);
int lss_timing_reset(void);
int lss_timing_read(int kernel_id, double *total_ms, int64_t *launches);
const char *lss_timing_kernel_name(int kernel_id);

#ifdef __cplusplus
}
#endif
#endif /* LSS_TIMING_H */
