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
/* Which kinds are bracketed while profiling is enabled: bit k of kind_mask = kind k (default: all).  The two
 * event records around a launch cost a few microseconds on its stream (measured: 54 of them per iteration
 * add 0.19 ms to a 49.4 ms iteration), so a benchmark times the one kernel it reports on. */
int32_t shadow_profile_kinds(shadow_ctx* ctx, uint32_t kind_mask);
/* Synchronizes, returns and resets the launches and summed duration of one kind. */
int32_t shadow_profile_read(shadow_ctx* ctx, uint32_t kind, uint64_t* launches, double* total_ms);

/* Plain device-to-device copy kernel of `bytes` (multiple of 16) on `stream`
 * (NULL = default): a known-traffic yardstick for bandwidth counters.
 * max_launch_threads: 0 = one launch per 2^31 threads, else as in shadow_launch_shape. */
int32_t shadow_copy_probe(void* d_dst, const void* d_src, uint64_t bytes, void* stream, uint64_t max_launch_threads);

/* A kernel that does nothing but stream: n_src device arrays in, n_dst device arrays out, `bytes`
 * (multiple of 16) each, non-temporal 16-byte accesses, one vector per lane and array, every load of
 * a lane issued before its first use -- the access pattern of the update kernels without their
 * arithmetic.  It shows what the chip sustains for a given mix of read and written streams, the
 * ceiling the update kernels are measured against.
 *   n_src in {0, 1, 2, 4, 7, 8, 16}, n_dst in {0, 1, 3}, not both zero; other mixes: SHADOW_EINVAL.
 *   Vector i of destination d becomes the XOR of vector i of all sources with d added to its first
 *   32-bit word (n_src == 0: the words {i mod 2^32, 0, 0, 0} likewise).
 *   n_dst == 0 (reads alone): d_sink names 16 writable device bytes, written only if the four words
 *   of some XOR all equal 0x9E3779B9; otherwise d_sink may be NULL.
 *   block: threads per block (0 = 256); waves_per_cu: bound on the waves a compute unit holds
 *   (0 = none), both as in shadow_launch_shape.  Arrays are the caller's and 16-byte aligned.  A
 *   destination may be one of the sources (an update in place: each lane writes the vectors it has
 *   read); arrays must not overlap in any other way.  Enqueues on `stream` (NULL = default) and returns. */
int32_t shadow_stream_probe(void* const* d_dst, uint32_t n_dst, const void* const* d_src, uint32_t n_src, void* d_sink, uint64_t bytes,
                            void* stream, uint32_t block, uint32_t waves_per_cu);

#ifdef __cplusplus
}
#endif
#endif /* SHADOW_MEASURE_H */
