/*
 * shadow_measure.h -- measurement aids of the shadow-update library.  Nothing
 * here is part of the method: these calls exist so that a benchmark can time
 * the library's kernels on their own streams and scale hardware byte counters
 * against a kernel of known traffic.
 */
#ifndef SHADOW_MEASURE_H
#define SHADOW_MEASURE_H

#include "shadow.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-kernel timing with HIP events on the streams the kernels run on.
 * kind: 0 fused fold + optimizer, 1 fold + sum of squares, 2 norm finalize, 3 optimizer sweep,
 * 4 snapshot copies. */
enum { SHADOW_K_FOLD_ADAMW = 0, SHADOW_K_FOLD_SUMSQ = 1, SHADOW_K_NORM = 2, SHADOW_K_ADAMW = 3, SHADOW_K_SNAPSHOT = 4,
       SHADOW_K_COUNT = 5 };
/* While enabled every launch is bracketed by two events; at most 65,536 spans are kept per kind
 * between reads (later launches are not recorded). */
int32_t shadow_profile_enable(shadow_ctx* ctx, int32_t on);
/* Synchronizes, returns and resets the launches and summed duration of one kind. */
int32_t shadow_profile_read(shadow_ctx* ctx, uint32_t kind, uint64_t* launches, double* total_ms);

/* Plain device-to-device copy kernel of `bytes` (multiple of 16) on `stream`
 * (NULL = default): a known-traffic yardstick for bandwidth counters.
 * max_launch_threads: 0 = one launch per 2^31 threads, else as in shadow_launch_shape. */
int32_t shadow_copy_probe(void* d_dst, const void* d_src, uint64_t bytes, void* stream, uint64_t max_launch_threads);

#ifdef __cplusplus
}
#endif
#endif /* SHADOW_MEASURE_H */
