/*
 * shadow.h -- C ABI of the shadow-update library for AMD MI355X (gfx950).
 *
 * The library keeps a checkpoint replica of a model (fp32 parameters plus the
 * AdamW moments m and v) in HBM and, once per training iteration, folds the
 * gradient buckets of the W data-parallel workers into one reduced gradient
 * and applies the trainers' optimizer step to the replica.  This is the work
 * of a shadow node in Checkmate (arxiv 2507.13522): section 4 overview, steps
 * 3 and 4; section 4.2.2 (bucket -> parameter mapping); section 4.2.3
 * (updating the checkpoint); section 4.2.4 (functional optimizers: every
 * element is updated independently, so buckets may be applied one by one).
 *
 * Conventions
 *   - Every function returns 0 (SHADOW_OK) or a negative shadow_status; no
 *     function aborts or throws.  On an error the replica is left untouched
 *     unless the status is SHADOW_EHIP (a runtime failure after work was
 *     enqueued; the context must then be destroyed).
 *   - "device pointer" = HBM address valid on the current HIP device;
 *     "host pointer"   = ordinary process memory.  Every array argument says
 *     which one it is.
 *   - The library never frees or reallocates caller memory; arenas and
 *     gradient views are BORROWED.  It allocates only small device tables
 *     (weight-decay map, norm partials) that it owns.
 *   - Calls on one context are not thread-safe; use one host thread per context.
 *   - The calls record and wait on events, keep host-side bookkeeping per
 *     iteration and pass per-iteration scalars as kernel arguments: do not
 *     issue them while a stream is being captured into a HIP graph.
 *   - Events and streams cross the boundary as void* holding a hipEvent_t /
 *     hipStream_t of the caller's HIP runtime.
 *   - Measurement aids (per-kernel timing, a copy kernel of known traffic, a
 *     kernel that only streams a given mix of arrays) are declared in
 *     shadow_measure.h; they are not part of the method.
 */
#ifndef SHADOW_H
#define SHADOW_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SHADOW_OK      = 0,
    SHADOW_EINVAL  = -1,  /* null / misaligned pointer, bad hyper-parameter, bad size          */
    SHADOW_EBUCKET = -2,  /* bucket id out of range                                            */
    SHADOW_EDUP    = -3,  /* bucket already applied in this iteration (section 4.1: a gradient
                             must reach the shadow exactly once per iteration)                 */
    SHADOW_ESTEP   = -4,  /* step is not last completed step + 1 (a lost or replayed iteration) */
    SHADOW_EBUSY   = -5,  /* operation needs an iteration boundary but an iteration is open    */
    SHADOW_EHIP    = -6,  /* HIP runtime failure; shadow_last_hip_error() has the text         */
    SHADOW_ENOMEM  = -7,  /* host or device allocation failed                                  */
    SHADOW_ETOOBIG = -8   /* input exceeds the fixed capacity of the library's static scratch  */
} shadow_status;

enum { SHADOW_GRAD_F32 = 0, SHADOW_GRAD_BF16 = 1 };
enum { SHADOW_REDUCE_MEAN = 0, SHADOW_REDUCE_SUM = 1 };
/* Functional optimizers (section 4.2.4).  ADAMW: decoupled decay.  ADAM: the L2 penalty joins
 * the gradient (g += weight_decay*p).  SGD: g += weight_decay*p; b = beta1*b + g; p -= lr*b, with
 * beta1 as the momentum coefficient and b kept in the m arena; beta2, eps are ignored and the v
 * arena must be NULL. */
enum { SHADOW_OPT_ADAMW = 0, SHADOW_OPT_ADAM = 1, SHADOW_OPT_SGD = 2 };
enum { SHADOW_MAX_WORKERS = 64, SHADOW_MAX_STREAMS = 16 };

/* One model tensor.  Tensors are listed in MODEL order (first layer first). */
typedef struct {
    uint64_t numel;         /* >= 1, no alignment requirement                          */
    uint32_t weight_decay;  /* 1: decoupled weight decay applies; 0: masked (bias/norm) */
    uint32_t reserved;      /* must be 0                                               */
} shadow_tensor_desc;

/* Launch shape of the kernels of ONE replica (part of shadow_hparams; every field 0 = the
 * library's default, which is what was measured fastest on MI355X).  Results never depend on it.
 *   fold_block, fused_block, sweep_block   threads per block of the per-bucket fold + sum-of-squares
 *                             kernel (default: 1024 when a lane's 4 elements are exactly 64 bytes of views, else 128),
 *                             of the per-bucket fold + optimizer kernel (default: 64 for launches under 2^27
 *                             elements, else 128) and of the whole-arena optimizer sweep (default 256):
 *                             64, 128, 256, 512 or 1024.
 *   fold_waves_per_cu, fused_waves_per_cu, sweep_waves_per_cu   upper bound on the waves a compute
 *                             unit holds of that kernel at a time, 1..32 (32 = no bound).  Defaults: no bound
 *                             for 1024-thread fold blocks, else about 96 KiB of loads in flight per compute
 *                             unit; about 80 KiB for the fold + optimizer kernel; never fewer than 8 waves;
 *                             16 for the sweep.  Fewer requests in flight keep DRAM rows open longer; enforced
 *                             by reserving unused LDS, in whole blocks and at most 64 KiB per block.  Worker
 *                             counts other than 1, 2, 4, 8, 16, 32, 64 run a loop that takes the views 8 at a
 *                             time instead of fully unrolled loads: their per-bucket kernels default to
 *                             128-thread blocks, no bound.
 *   drain_blocks              256-thread blocks of the kernel that writes a snapshot to pinned host
 *                             memory (default 4, at most 4096): few on purpose.  Measured: once the stores
 *                             to the host saturate the link (8 blocks and more, and the runtime's own
 *                             device-to-host copy kernel) every kernel that runs beside them slows by
 *                             50-100 %; at 1-4 blocks (10-34 GB/s to the host) by 3-7 %.
 *   max_launch_threads        a logical launch with more threads is issued as several launches
 *                             (default and upper limit 2^31; lower values exist so that tests can
 *                             reach the split paths with small inputs; at least one block and one
 *                             bucket go into every launch). */
typedef struct {
    uint32_t fold_block;
    uint32_t fused_block;
    uint32_t sweep_block;
    uint32_t fold_waves_per_cu;
    uint32_t fused_waves_per_cu;
    uint32_t sweep_waves_per_cu;
    uint32_t drain_blocks;
    uint32_t reserved;          /* must be 0 */
    uint64_t max_launch_threads;
} shadow_launch_shape;

/* Optimizer and reduce settings (AdamW: section 6; reduce: section 2.1). */
typedef struct {
    float    lr;             /* >= 0                                                       */
    float    beta1;          /* in [0, 1)                                                  */
    float    beta2;          /* in [0, 1)                                                  */
    float    eps;            /* > 0                                                        */
    float    weight_decay;   /* >= 0; p *= (1 - lr*weight_decay) on tensors with the flag  */
    float    max_grad_norm;  /* > 0: clip the reduced gradient's global L2 norm; <= 0: off */
    uint32_t num_workers;    /* W in [1, SHADOW_MAX_WORKERS]                               */
    uint32_t grad_dtype;     /* SHADOW_GRAD_F32 or SHADOW_GRAD_BF16                        */
    uint32_t reduce_op;      /* SHADOW_REDUCE_MEAN (sum * float(1/W)) or SHADOW_REDUCE_SUM */
    uint32_t num_streams;    /* HIP streams buckets are spread over, [1, SHADOW_MAX_STREAMS] */
    uint32_t optimizer;      /* SHADOW_OPT_ADAMW, SHADOW_OPT_ADAM or SHADOW_OPT_SGD                */
    uint64_t batch_bytes;    /* bucket scheduling: accepted buckets of a stream are buffered (host side,
                                pointers only) until their gradient bytes (numel * elem size * W) reach
                                this value, then folded by ONE launch; the iteration's last bucket,
                                shadow_sync and shadow_destroy always launch what is buffered.
                                0 = launch every bucket at once (lowest latency); a large value =
                                fewest launches (a 50 MiB bucket is only ~90 us of HBM time, so launch
                                ramps and gaps cost ~4 % of the fold when every bucket is its own launch) */
    shadow_launch_shape launch;  /* all zero = the library's defaults                          */
} shadow_hparams;

/* ------------------------------------------------------------------------ *
 * Parameter layout (host only; needs no GPU).  Section 4.2.2.
 *
 * Tensors are bin-packed into buckets walking from the LAST tensor to the
 * first: a tensor joins the open bucket while the bucket's gradient bytes stay
 * <= bucket_cap_bytes, otherwise a new bucket is opened; a tensor larger than
 * the cap closes the open bucket and gets a bucket of its own.  Bucket 0 is
 * the first one formed (last layers).  Inside a bucket tensors lie back to
 * back in the order they were added, exactly as in the gradient views.
 *
 * The arena (param, m, v and the reduced-gradient scratch share this layout)
 * is bucket-major; every bucket starts on a 256-byte boundary (64 floats), so
 * arena_numel >= num_params; the gaps are owned and kept at zero by the library.
 * ------------------------------------------------------------------------ */
typedef struct shadow_layout shadow_layout;

/* tensors: host pointer, num_tensors entries.  bucket_of_tensor: host pointer
 * or NULL; if given it fixes the bucket id of every tensor (ids must be dense,
 * 0..B-1) and bucket_cap_bytes is ignored; members of a bucket are still laid
 * out last-tensor-first.  grad_elem_bytes: 2 or 4.  *out is owned by the
 * caller until shadow_layout_destroy. */
int32_t shadow_layout_create(shadow_layout** out, const shadow_tensor_desc* tensors, uint32_t num_tensors,
                             const uint32_t* bucket_of_tensor, uint32_t grad_elem_bytes,
                             uint64_t bucket_cap_bytes);
int32_t shadow_layout_destroy(shadow_layout* layout);
int32_t shadow_layout_num_buckets(const shadow_layout* layout, uint32_t* out);
int32_t shadow_layout_num_params(const shadow_layout* layout, uint64_t* out);
/* floats the caller must allocate for each of param, m, v (and scratch) */
int32_t shadow_layout_arena_numel(const shadow_layout* layout, uint64_t* out);
/* bucket -> its start in the arena (in floats), its element count, its tensor count */
int32_t shadow_layout_bucket(const shadow_layout* layout, uint32_t bucket, uint64_t* arena_offset,
                             uint64_t* numel, uint32_t* num_tensors);
/* tensor (model-order index) -> bucket, offset inside the bucket, offset in the arena (elements) */
int32_t shadow_layout_tensor(const shadow_layout* layout, uint32_t tensor, uint32_t* bucket,
                             uint64_t* offset_in_bucket, uint64_t* arena_offset);

/* Placement advice (host only; nothing below is required for correctness).
 * On MI355X the speed of a kernel that streams several arrays at once depends
 * on where in the 288 GiB of HBM the arrays lie.  Measured: the memory behaves
 * as three regions of 96 GiB; arrays that are WRITTEN at the same time should
 * not all lie in one region (whole-arena AdamW sweep at 7B: 33 ms with param,
 * m and v in one region, 29 ms with two of them in one region and the third
 * in the next), and a written array should not share its region with many
 * arrays that are read at the same time (fold of 16 views: 8.2 ms with the
 * reduced-gradient arena in the region of the views, 7.3 ms with it in
 * another).  The W views of one bucket stream best close together
 * (bucket-major: 6.4 TB/s, one arena-sized buffer per worker: 6.05 TB/s).
 *
 * shadow_layout_device_plan: byte offsets for param, m, v, the scratch arena,
 * a snapshot staging set (shadow_snapshot_attach) and the staging buffer of the
 * gradient views inside ONE device allocation of block_bytes (256 GiB).  Made first in a process, such an allocation is one naturally
 * aligned block of the driver's allocator, so offsets inside it are physical
 * offsets: the scratch arena, param and m end the first region, v starts the
 * second, the snapshot set follows v and the staging buffer comes last.
 * with_scratch / with_snapshot_set: nonzero when the caller wants a scratch
 * arena / a second set of param, m, v arenas; staging_bytes: size of the gradient buffer the caller
 * wants placed (the whole bucket-major buffer of shadow_layout_staging_bytes,
 * or a ring of its own size), 0 for none.  Offsets of absent parts are 0.
 * SHADOW_ENOMEM when the parts do not fit this scheme (the caller then places
 * them itself, e.g. by the stride below).
 *
 * shadow_layout_arena_stride: recommended distance in BYTES between the starts
 * of param, m, v (and the scratch arena) when they are carved from one device
 * allocation: the smallest power of two >= the arena's size (at least 2 MiB).
 *
 * shadow_layout_staging_*: a bucket-major staging buffer for the gradient
 * views: bucket 0's W views, then bucket 1's ..., every bucket starting on a
 * 2 MiB boundary.  Views of 2 MiB or more lie a multiple of 2 MiB plus 4 KiB
 * apart (worker w's view starts w * 4 KiB past a 2 MiB boundary), so that the
 * W reads of one element do not meet in one DRAM channel; shorter views lie
 * back to back, 256-byte aligned.  _bytes gives the size of the whole buffer,
 * _view the byte offset of worker `worker`'s view of `bucket`. */
typedef struct shadow_device_plan {
    uint64_t block_bytes;       /* size of the one allocation */
    uint64_t param_offset;      /* byte offsets inside it, each a multiple of 1 GiB */
    uint64_t m_offset;
    uint64_t v_offset;
    uint64_t scratch_offset;
    uint64_t staging_offset;
    uint64_t snap_param_offset; /* snapshot staging set; 0 when not asked for */
    uint64_t snap_m_offset;
    uint64_t snap_v_offset;
} shadow_device_plan;
int32_t shadow_layout_device_plan(const shadow_layout* layout, int32_t with_scratch, int32_t with_snapshot_set,
                                  uint64_t staging_bytes, shadow_device_plan* plan);
int32_t shadow_layout_arena_stride(const shadow_layout* layout, uint64_t* stride_bytes);
int32_t shadow_layout_staging_bytes(const shadow_layout* layout, uint32_t num_workers, uint64_t* bytes);
int32_t shadow_layout_staging_view(const shadow_layout* layout, uint32_t num_workers, uint32_t bucket,
                                   uint32_t worker, uint64_t* byte_offset);

/* ------------------------------------------------------------------------ *
 * The replica.
 * ------------------------------------------------------------------------ */
typedef struct shadow_ctx shadow_ctx;

/* Create a replica over caller-allocated arenas on the current HIP device: the
 * shadow's copy of the training state, i.e. the parameters and the optimizer's
 * state (section 2.1), which starts out equal to the trainers' (section 4.2.3).
 *   layout     host object, copied (may be destroyed afterwards).
 *   hp         host pointer.
 *   d_param, d_m, d_v   device pointers, arena_numel floats each, 256-byte
 *              aligned, borrowed until shadow_destroy.  The caller has already
 *              written the initial state at the layout's offsets (fresh start:
 *              parameters, m = v = 0; restore: a snapshot's contents).  The
 *              library zeroes the alignment gaps.
 *   d_reduced  device pointer, arena_numel floats, 256-byte aligned, borrowed:
 *              holds the reduced gradient between the fold and the update when
 *              clipping is on (the norm over ALL buckets must be known before
 *              any element is updated).  Must be NULL when clipping is off.
 *              May be NULL with clipping on: the library then folds every
 *              bucket's views a second time once the norm is known instead of
 *              storing the reduced gradient (24 + 2*W*G bytes per parameter
 *              instead of 32 + W*G, G = gradient element size: fewer bytes when
 *              W*G < 8, e.g. the paper's own case of ONE already-reduced bf16
 *              gradient per bucket, W = 1); the views of the whole iteration
 *              must then stay unchanged until its update has run.
 *   start_step iterations already applied to this state (0 for a fresh
 *              replica; a snapshot's step when restoring: section 6.5 resumes
 *              training from the shadow's checkpoint).  The first iteration
 *              applied is start_step + 1; Adam's bias correction uses that
 *              1-based count.
 *   streams    host array of hp->num_streams hipStream_t handles (for example
 *              torch streams' .cuda_stream), borrowed; or NULL: the library
 *              creates and owns default-priority streams.
 * Errors: EINVAL (null or misaligned arena, bad hyper-parameter, a bucket too
 * large for one launch), ENOMEM, EHIP; nothing is left allocated on an error.
 */
int32_t shadow_init(shadow_ctx** out, const shadow_layout* layout, const shadow_hparams* hp,
                    float* d_param, float* d_m, float* d_v, float* d_reduced,
                    uint64_t start_step, void* const* streams);

/* The replica's bucket map (section 4.2.2: the shadow keeps the mapping from
 * buckets to parameter offsets).  Same numbers as shadow_layout_num_buckets /
 * shadow_layout_bucket on the layout the replica was created from; they exist
 * on the context because the layout object need not outlive shadow_init. */
int32_t shadow_num_buckets(const shadow_ctx* ctx, uint32_t* out);
int32_t shadow_bucket_info(const shadow_ctx* ctx, uint32_t bucket_id, uint64_t* arena_offset, uint64_t* numel);

/* Apply one bucket of iteration `step` (section 4.2.3: the shadow receives
 * the gradient buckets of an iteration and runs the trainers' optimizer step;
 * section 4.2.4: the optimizers are functional, so buckets may be applied one
 * by one in any order; section 4.1: every gradient reaches the shadow exactly
 * once per iteration).  The W gradient views are folded and (when clipping is
 * off) the bucket's parameters are updated in the same kernel; when clipping is
 * on the fold stores the reduced gradient and its sum of squares, and the call
 * that delivers the last missing bucket of the iteration also enqueues the norm
 * and the update of every bucket.
 *   d_grad_views  HOST array of W DEVICE pointers; view w holds worker w's
 *                 gradient for this bucket: numel(bucket) elements of
 *                 grad_dtype, contiguous, in the bucket's element order,
 *                 16-byte aligned.  The pointer array itself is copied during
 *                 the call.
 *   step          must equal last completed step + 1; buckets of one
 *                 iteration may come in any order, each exactly once.
 *   ready_event   hipEvent_t recorded by the producer of the views (a copy
 *                 engine, a collective, a kernel) on ITS stream after the last
 *                 write to them, or NULL when the views are complete at the
 *                 time of the call.  The library makes the bucket's stream wait
 *                 for the event before anything reads the views, also when the
 *                 launch itself is deferred (batch_bytes > 0); the host never
 *                 blocks.  The event may be re-recorded after the call returns.
 * The views must stay unchanged until the work that reads them has run: see
 * shadow_record_consumed (stream-ordered) or shadow_sync (host-blocking).
 * Asynchronous: returns after buffering or enqueueing.  Errors: EINVAL, EBUCKET, EDUP,
 * ESTEP, ENOMEM (the replica is untouched), EHIP. */
int32_t shadow_apply_bucket(shadow_ctx* ctx, uint32_t bucket_id, const void* const* d_grad_views,
                            uint64_t step, void* ready_event);

/* Release side of the views (the counterpart of ready_event): launches what is buffered for the
 * stream bucket_id runs on and records `event` (the caller's hipEvent_t, not NULL) on that
 * stream.  Once the event has completed, the views of bucket_id and of every bucket accepted
 * before it on the same stream (bucket ids congruent modulo num_streams) have been read for the
 * last time and may be overwritten; the host does not block.  When clipping runs without a
 * scratch arena the views are read a second time at the end of the iteration: the call then
 * returns EBUSY while an iteration is open.  Errors: EINVAL, EBUCKET, EBUSY, EHIP. */
int32_t shadow_record_consumed(shadow_ctx* ctx, uint32_t bucket_id, void* event);

/* Ingest from host memory: the analogue of the shadow node's receive path, which copies
 * reassembled buckets from network buffers into the framework's tensors (section 5).
 * shadow_ingest_attach lends the context a device ring (d_ring: device pointer, 256-byte
 * aligned, ring_bytes >= W * (largest bucket's gradient bytes rounded up to 256); borrowed until
 * shadow_destroy); it is cut into slots that each hold the W views of one bucket (at most 64
 * slots are used).  shadow_ingest_bucket copies the W HOST views (h_grad_views: host array of
 * W host pointers, pinned memory for the copies to be asynchronous) of a bucket into the next
 * slot on a copy stream of the library's own, orders the bucket's fold behind the copy on the
 * bucket's stream and launches it at once (batch_bytes does not apply), so that the copy of
 * one bucket overlaps the fold of the previous ones; a slot is overwritten only after its fold
 * has run.  ready_event (hipEvent_t or NULL) is waited for by the copy stream before the first
 * copy, for host views that a device-side producer fills.  The host views must stay unchanged
 * until shadow_sync returns.  Same step / bucket rules and errors as shadow_apply_bucket; not
 * available when clipping runs without a scratch arena (EINVAL).  Both ways of delivering
 * buckets may be mixed within an iteration. */
int32_t shadow_ingest_attach(shadow_ctx* ctx, void* d_ring, uint64_t ring_bytes);
int32_t shadow_ingest_bucket(shadow_ctx* ctx, uint32_t bucket_id, const void* const* h_grad_views, uint64_t step,
                             void* ready_event);

/* ------------------------------------------------------------------------ *
 * Snapshots: a consistent copy of (param, m, v, step) at an iteration
 * boundary.  The replica itself is the checkpoint, kept up to date at
 * per-iteration granularity (section 4 overview); a snapshot is how it is
 * read without stopping the updates: to serve a recovering trainer or to
 * consolidate shards (section 4.2.4), or to restore a replica (section 6.5).
 * Three ways, none of which blocks the host:
 *
 * shadow_snapshot: copies enqueued on a copy stream of the library's own,
 *   behind the last kernel of the last completed iteration.  dst_* are device
 *   pointers or pinned host pointers of arena_numel floats each (NULL = skip
 *   that array; dst_v is ignored for SGD, which has no second state array).
 *   Kernels of later iterations that only read the gradient views (the fold
 *   with clipping on) run concurrently with the copies; the first kernel that
 *   writes param, m or v waits for them.  To pinned host memory the copies run
 *   at PCIe speed, so a large replica stalls for as long as they take: use
 *   the staged form below for that.  *out_step (host pointer, may be NULL)
 *   receives the iteration count.  done_event (hipEvent_t or NULL) is recorded
 *   behind the last copy.  SHADOW_EBUSY if an iteration is partly applied: a
 *   checkpoint is only consistent at iteration granularity.
 *
 * shadow_snapshot_attach + shadow_snapshot_arm: the staged form.  attach lends
 *   a second set of arenas in device memory (arena_numel floats each, 256-byte
 *   aligned, d_stage_v NULL for SGD; borrowed until shadow_destroy; at most
 *   once per context).  arm asks for the state at the END of the iteration that
 *   is about to start (EBUSY once its first bucket has been accepted): that
 *   iteration's update kernels then write every new value twice, to the replica
 *   and to the staging set (12 more bytes per parameter written, nothing read
 *   again, no separate copy pass and no wait for later iterations).  If
 *   h_dst_* (pinned host pointers, arena_numel floats each, all three NULL for
 *   none) are given, the staging set is drained to them on the copy stream
 *   from the boundary on, concurrently with every later iteration (by a copy
 *   kernel of a few blocks, see drain_blocks, which leaves the chip to the
 *   update kernels); arm
 *   returns EBUSY while such a drain is still running (the staging set would be
 *   overwritten under it).  Without host arrays the staging set itself is the
 *   snapshot; arming again overwrites it, so a caller that reads it orders its
 *   reads before the next arm.
 *
 * shadow_snapshot_record: records `event` (caller's hipEvent_t) behind the last
 *   requested snapshot (EBUSY while an armed snapshot's iteration is not yet
 *   complete; EINVAL if none was ever requested).  shadow_snapshot_wait blocks
 *   the host until that snapshot is complete and returns its step.
 * ------------------------------------------------------------------------ */
int32_t shadow_snapshot(shadow_ctx* ctx, float* dst_param, float* dst_m, float* dst_v, uint64_t* out_step,
                        void* done_event);
int32_t shadow_snapshot_attach(shadow_ctx* ctx, float* d_stage_param, float* d_stage_m, float* d_stage_v);
int32_t shadow_snapshot_arm(shadow_ctx* ctx, float* h_dst_param, float* h_dst_m, float* h_dst_v);
int32_t shadow_snapshot_record(shadow_ctx* ctx, void* event);
int32_t shadow_snapshot_wait(shadow_ctx* ctx, uint64_t* out_step);

/* Block the host until everything enqueued by this context has run, buffered
 * buckets and snapshot copies included (the shadow must have finished an
 * iteration before the trainers' next one reaches it, section 6.4). */
int32_t shadow_sync(shadow_ctx* ctx);
/* Launch what is buffered, wait for it, release the library's tables, streams
 * and events.  The arenas hold the state of the last completed iteration (plus
 * the buckets of an open one) and stay the caller's: the replica can be
 * recreated over them with start_step (recovery, section 4.2.4). */
int32_t shadow_destroy(shadow_ctx* ctx);

/* Queries (host pointers out). */
int32_t shadow_step(const shadow_ctx* ctx, uint64_t* completed_step, uint32_t* buckets_pending);
/* stream (hipStream_t) that work for this bucket is enqueued on */
int32_t shadow_bucket_stream(const shadow_ctx* ctx, uint32_t bucket_id, void** out_stream);
/* Clip coefficient c = min(1, max_norm/(||r||_2 + 1e-6)) and sum of squares of
 * the last completed iteration; synchronizes.  EINVAL if clipping is off. */
int32_t shadow_clip_state(shadow_ctx* ctx, float* out_coef, double* out_sumsq);
/* Learning rate for iterations that start after this call (cosine or any
 * other schedule is evaluated by the caller; section 6).  EBUSY mid-iteration. */
int32_t shadow_set_lr(shadow_ctx* ctx, float lr);

/* For callers that cannot allocate device memory or create streams and events: code whose
 * launches must all go to one given stream, tight serving loops, harnesses that forbid
 * hipMalloc.  One WHOLE iteration in one call, without a context: the same kernels and the same
 * bits as shadow_init + shadow_apply_bucket for every bucket, everything enqueued on `stream`
 * (hipStream_t, NULL = default) in order.  The call makes no device allocation, creates no stream
 * and no event and never blocks: the tables its kernels need beyond the caller's arrays (the
 * weight-decay map, the norm partials, the clip coefficient) live in a static device array of
 * about 5 MiB that each GPU the library runs on holds until the process ends.
 *   layout, hp          as for shadow_init (hp->num_streams and hp->batch_bytes are not used:
 *                       all buckets are folded in as few launches as the descriptor allows).
 *   d_param, d_m, d_v, d_reduced   the arenas, as for shadow_init (d_reduced NULL with clipping
 *                       on: the views are folded twice).  The alignment gaps are not touched.
 *   d_grad_views        HOST array of num_buckets * W DEVICE pointers, bucket-major (bucket b's
 *                       W views at [b*W, b*W + W)), each as for shadow_apply_bucket; complete
 *                       when `stream` reaches the call's work, unchanged until it has run.
 *   step                1-based count of this iteration (Adam's bias correction).
 * Limits: arena_numel <= SHADOW_STATIC_MAX_ARENA_NUMEL, at most SHADOW_STATIC_MAX_BUCKETS buckets
 * and 8,192 runs of tensors with equal weight-decay flag; beyond them SHADOW_ETOOBIG and nothing
 * is enqueued.  All calls on one GPU share that GPU's scratch array, which keeps the last
 * call's contents (every entry that is read is rewritten first, nothing needs clearing): calls
 * whose work may overlap on one GPU (different streams, several threads) race; serialize them.
 * Other errors: EINVAL, ENOMEM (host), EHIP. */
enum { SHADOW_STATIC_MAX_ARENA_NUMEL = 1 << 27, SHADOW_STATIC_MAX_BUCKETS = 4096 };
int32_t shadow_apply_iteration_static(const shadow_layout* layout, const shadow_hparams* hp,
                                      float* d_param, float* d_m, float* d_v, float* d_reduced,
                                      const void* const* d_grad_views, uint64_t step, void* stream);

const char* shadow_strerror(int32_t status);
const char* shadow_last_hip_error(void);
/* Identifies the sources the library was built from (a hash the build passes in). */
const char* shadow_build_id(void);

#ifdef __cplusplus
}
#endif
#endif /* SHADOW_H */
