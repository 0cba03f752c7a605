/*
 * Development aid, compiled only into trace builds of the library (-DTAPER_WG_TRACE, see
 * build.py and wg_trace.py): per-workgroup clocks of the decode kernel.
 *
 * taper_wg_trace_buffer(ctx, buf): every later launch on ctx writes, for workgroup w of its
 * grid, four 64-bit words at buf[4w..4w+3] (device memory, at least 4 x grid size words,
 * zeroed by the caller before each launch): the 100 MHz wall clock when the workgroup
 * started, when its own share was done (when it first turned to the pool; without a pool: when a
 * shared-prefix share was done, or a private one started), when it
 * left the kernel, and the clock ticks it spent merging.  NULL switches tracing off.
 */
#ifndef TAPER_TRACE_H
#define TAPER_TRACE_H
#include "taper_attn.h"
#ifdef __cplusplus
extern "C" {
#endif
__attribute__((visibility("default"))) int taper_wg_trace_buffer(taper_ctx *ctx, long long *buf /* device */);
#ifdef __cplusplus
}
#endif
#endif
