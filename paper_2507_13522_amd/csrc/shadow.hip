// Host side of the shadow-update library: layout (section 4.2.2), exactly-once
// bookkeeping per iteration (section 4.1), scheduling of bucket kernels on HIP
// streams, snapshot at iteration boundaries (section 4, per-iteration
// granularity of the checkpoint).  The C ABI is declared in include/shadow.h.
#include "shadow_kernels.hip.h"

#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/shadow.h"
#include "../../include/shadow_measure.h"

using namespace shadow;

namespace {

thread_local std::string g_hip_error;

constexpr uint64_t kMaxThreadsPerLaunch = 1ull << 31;
// The fold + sum-of-squares kernel streams W arrays in and one out.  Measured: when a lane's one group of 4 elements
// is exactly 64 bytes of views (W = 8 bf16, W = 4 float) 1024-thread blocks without a bound on the waves are fastest;
// when the lane owns several narrow groups (W = 1, 2, 4 bf16; W = 1, 2 float) 128-thread blocks without a bound
// (-3 ... -10 % time); with more bytes per lane (W = 16, 32, 64) 128-thread blocks and about 96 KiB of loads in flight
// per CU, but at least 8 waves (W = 16: 12 waves, -5 %; W = 32: 8 waves, -4 %; fewer than 8 waves: +15 %).
constexpr uint32_t kDefaultFoldBlock = 1024;
constexpr uint32_t kWideFoldBlock = 128;
constexpr uint32_t kFoldBytesInFlightPerCu = 96 * 1024;
// The fold + optimizer kernel streams W + 3 arrays in and 3 out.  Measured on MI355X (sweeps of block size and of the
// waves a CU holds, three model sizes, W = 1, 8, 16): it runs fastest with small blocks and with about 80 KiB of loads in
// flight per CU, i.e. with FEWER waves the more bytes a lane loads (W = 16: 8 waves, W = 8: 10-12, W = 1: 16-24), but
// never fewer than 8; launches under 2^27 elements prefer 64-thread blocks, longer ones 128-thread blocks.
constexpr uint32_t kFusedBytesInFlightPerCu = 80 * 1024;
constexpr uint64_t kFusedSmallLaunchElems = 1ull << 27;
constexpr uint32_t kDefaultSweepBlock = 256;     // threads per block of the whole-arena optimizer sweep
constexpr uint32_t kDefaultFoldWaves = 32;       // waves a CU may hold: no bound for 1024-thread fold blocks,
constexpr uint32_t kDefaultSweepWaves = 16;      // 4 blocks of 256 threads for the sweep
constexpr uint32_t kDefaultDrainBlocks = 4;      // blocks of the kernel that drains a snapshot to the host
constexpr uint32_t kLdsPerCu = 160 * 1024;
constexpr size_t kMaxSpansPerKind = 65536;

#ifndef SHADOW_BUILD_ID
#define SHADOW_BUILD_ID "unknown"
#endif

bool valid_block(uint32_t b) { return b == 64 || b == 128 || b == 256 || b == 512 || b == 1024; }

// Bytes of LDS a block reserves (and never touches) so that a CU holds at most `waves` waves of it.
uint32_t lds_for_wave_cap(uint32_t block, uint32_t waves)
{
    if (waves >= 32) return 0;
    const uint32_t waves_per_block = block / 64;
    uint32_t blocks_per_cu = waves / waves_per_block;
    if (blocks_per_cu < 1) blocks_per_cu = 1;
    uint32_t lds = (kLdsPerCu / blocks_per_cu) & ~511u;
    return lds > 65536 ? 65536 : lds;             // the most a launch may ask for without a function attribute
}

#define HIP_TRY(expr)                                                                         \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess) {                                                               \
            g_hip_error = std::string(#expr) + ": " + hipGetErrorString(e_);                  \
            return SHADOW_EHIP;                                                               \
        }                                                                                     \
    } while (0)

constexpr uint64_t kAlignElems = 64;   // 256 bytes of float

struct Seg {
    uint32_t tensor;
    uint64_t offset;   // inside the bucket
    uint64_t numel;
    uint8_t wd;
};

struct BucketL {
    uint64_t arena_off = 0;
    uint64_t numel = 0;
    std::vector<Seg> segs;
};

}  // namespace

struct shadow_layout {
    std::vector<shadow_tensor_desc> tensors;
    std::vector<uint32_t> bucket_of;
    std::vector<uint64_t> off_in_bucket;
    std::vector<BucketL> buckets;
    uint64_t num_params = 0;
    uint64_t arena_numel = 0;
    uint32_t grad_elem_bytes = 0;
};

struct shadow_ctx {
    shadow_layout lay;
    shadow_hparams hp;
    float *p = nullptr, *m = nullptr, *v = nullptr, *r = nullptr;
    bool clip = false;
    bool refold = false;                  // clipping on without a scratch arena: views are folded twice
    std::vector<const void*> step_views;  // refold: the iteration's view pointers, bucket-major
    std::vector<hipStream_t> streams;
    bool own_streams = false;
    // device tables owned by the library
    uint8_t* d_tile_mode = nullptr;
    uint64_t* d_run_start = nullptr;
    uint8_t* d_run_flag = nullptr;
    uint32_t num_runs = 0;
    double* d_partial = nullptr;
    double* d_stage1 = nullptr;
    uint32_t nstage1 = 0;
    uint32_t fold_block = kDefaultFoldBlock, adamw_block = kDefaultSweepBlock;
    uint32_t fold_lds = 0, adamw_lds = 0;
    uint32_t fused_block_given = 0;       // 0: chosen per launch by its size
    uint32_t fused_waves = 0;             // waves a CU may hold of the fold + optimizer kernel
    uint32_t drain_blocks = kDefaultDrainBlocks;
    uint64_t max_launch_threads = kMaxThreadsPerLaunch;
    float* d_coef = nullptr;
    double* d_sumsq = nullptr;
    std::vector<uint32_t> slot_base, slot_count;
    uint32_t nslots = 0;
    // iteration state
    uint64_t completed = 0;
    std::vector<uint8_t> arrived;
    uint32_t arrived_count = 0;
    StepScalars sc{};
    uint64_t sc_step = 0;
    std::vector<hipEvent_t> join_ev;      // one per stream
    hipEvent_t boundary_ev = nullptr;     // after the last kernel of an iteration that ends on stream 0
    bool boundary_pending = false;        // streams must wait on boundary_ev before new work
    // snapshots: copies run on a stream of their own, behind the iteration they belong to
    hipStream_t snap_stream = nullptr;
    hipEvent_t state_ev = nullptr;        // replica complete at a boundary (recorded on stream 0 after a join)
    hipEvent_t snap_ev = nullptr;         // last copy out of the replica has run
    std::vector<uint8_t> snap_wait;       // per stream: wait for snap_ev before the next kernel that writes the replica
    float *stage_p = nullptr, *stage_m = nullptr, *stage_v = nullptr;   // lent staging set
    bool armed = false, snap_active = false;   // armed: the next iteration also writes the staging set; active: this one does
    float* armed_host[3] = {nullptr, nullptr, nullptr};
    hipEvent_t drain_ev = nullptr;        // staging set has been drained (or simply completed) for the last armed snapshot
    bool drain_recorded = false;          // drain_ev ends a drain to host arrays that may still be running
    bool have_snapshot = false;           // some snapshot was requested; last_snap_ev tells which event ends it
    hipEvent_t last_snap_ev = nullptr;
    uint64_t last_snap_step = 0;
    std::vector<uint8_t> stream_dirty;    // stream has work since the last join
    bool poisoned = false;
    // buckets accepted but not yet launched, per stream (see hp.batch_bytes)
    struct Pending { uint32_t bucket; const void* ptr[kMaxWorkers]; };
    std::vector<std::vector<Pending>> pending;
    std::vector<uint64_t> pending_bytes;
    // ingest from host memory: device ring of slots, each holding the W views of one bucket
    char* ring = nullptr;
    uint64_t slot_bytes = 0, view_stride = 0;
    uint32_t ring_slots = 0, ring_next = 0;
    hipStream_t copy_stream = nullptr;
    std::vector<hipEvent_t> copied_ev, consumed_ev;
    std::vector<uint8_t> consumed_valid;
    // profiling
    bool profile = false;
    uint32_t profile_kinds = ~0u;         // bit k: launches of kind k are bracketed while profiling is on
    struct Span { hipEvent_t a, b; };
    std::vector<Span> spans[SHADOW_K_COUNT];
    std::vector<hipEvent_t> ev_pool;
};

namespace {

bool plan(shadow_layout& L, const uint32_t* fixed, uint64_t cap)
{
    const uint32_t T = uint32_t(L.tensors.size());
    L.bucket_of.assign(T, 0);
    uint32_t nb = 0;
    if (fixed) {
        uint32_t mx = 0;
        for (uint32_t t = 0; t < T; ++t) {
            if (fixed[t] >= T) return false;      // dense ids 0..B-1 with B <= T
            L.bucket_of[t] = fixed[t];
            if (fixed[t] > mx) mx = fixed[t];
        }
        nb = T ? mx + 1 : 0;
        std::vector<uint8_t> used(nb, 0);
        for (uint32_t t = 0; t < T; ++t) used[fixed[t]] = 1;
        for (uint32_t b = 0; b < nb; ++b) if (!used[b]) return false;
    } else {
        bool open = false;
        uint32_t cur = 0;
        uint64_t cur_bytes = 0;
        for (uint32_t i = T; i-- > 0;) {
            const uint64_t size = L.tensors[i].numel * L.grad_elem_bytes;
            if (size > cap) {                 // too big for any shared bucket: alone, and it closes the open one
                L.bucket_of[i] = nb++;
                open = false;
                continue;
            }
            if (!open || cur_bytes + size > cap) {
                cur = nb++;
                cur_bytes = 0;
                open = true;
            }
            L.bucket_of[i] = cur;
            cur_bytes += size;
        }
    }
    L.buckets.assign(nb, BucketL{});
    L.off_in_bucket.assign(T, 0);
    for (uint32_t i = T; i-- > 0;) {          // members lie in the order they were added: last tensor first
        BucketL& b = L.buckets[L.bucket_of[i]];
        L.off_in_bucket[i] = b.numel;
        b.segs.push_back(Seg{i, b.numel, L.tensors[i].numel, uint8_t(L.tensors[i].weight_decay ? 1 : 0)});
        b.numel += L.tensors[i].numel;
    }
    uint64_t off = 0, total = 0;
    for (BucketL& b : L.buckets) {
        b.arena_off = off;
        total += b.numel;
        off += (b.numel + kAlignElems - 1) / kAlignElems * kAlignElems;
    }
    L.num_params = total;
    L.arena_numel = off;
    return true;
}

void compute_scalars(const shadow_hparams& hp, uint64_t t, StepScalars& s)
{
    const double b1 = hp.beta1, b2 = hp.beta2, lr = hp.lr, wd = hp.weight_decay;
    const double bc1 = 1.0 - std::pow(b1, double(t));
    const double bc2 = 1.0 - std::pow(b2, double(t));
    s.beta1 = hp.beta1;
    s.beta2 = hp.beta2;
    s.omb1 = float(1.0 - b1);
    s.omb2 = float(1.0 - b2);
    s.decay = float(1.0 - lr * wd);
    s.step_size = float(lr / bc1);
    s.isq = float(1.0 / std::sqrt(bc2));
    s.eps = hp.eps;
    s.inv_w = float(1.0 / double(hp.num_workers));
    s.mean = hp.reduce_op == SHADOW_REDUCE_MEAN ? 1u : 0u;
    s.lr = hp.lr;
    s.wd = hp.weight_decay;
}

// threads needed by a per-bucket kernel: one per 4 elements plus one for a ragged tail
uint64_t bucket_threads(uint64_t numel) { return (numel >> 2) + ((numel & 3) ? 1 : 0); }

uint32_t blocks_for(uint64_t threads, uint32_t block)
{
    uint64_t blocks = (threads + block - 1) / block;
    return uint32_t(blocks ? blocks : 1);
}

// groups of 4 elements one lane of the fold + sum-of-squares kernel owns (mirrors fold_vpl in the kernels)
uint32_t sumsq_vpl(const shadow_hparams& hp)
{
    const bool bf16 = hp.grad_dtype == SHADOW_GRAD_BF16;
    switch (hp.num_workers) {
        case 1: return bf16 ? fold_vpl<true, 1>() : fold_vpl<false, 1>();
        case 2: return bf16 ? fold_vpl<true, 2>() : fold_vpl<false, 2>();
        case 4: return bf16 ? fold_vpl<true, 4>() : fold_vpl<false, 4>();
        case 8: return bf16 ? fold_vpl<true, 8>() : fold_vpl<false, 8>();
        case 16: return bf16 ? fold_vpl<true, 16>() : fold_vpl<false, 16>();
        case 32: return bf16 ? fold_vpl<true, 32>() : fold_vpl<false, 32>();
        case 64: return bf16 ? fold_vpl<true, 64>() : fold_vpl<false, 64>();
        default: return 1;      // run-time worker count
    }
}

// Worker counts the kernels are instantiated for: all loads of a lane are then issued before the first add.  Any
// other count takes the run-time loop, 8 views at a time; its registers do not grow with W, so it runs unbounded.
bool unrolled_workers(uint32_t w) { return w == 1 || w == 2 || w == 4 || w == 8 || w == 16 || w == 32 || w == 64; }
constexpr uint32_t kLoopBlock = 128;     // measured on W = 3, 6, 24: 128-thread blocks, 32 waves, both per-bucket kernels

// blocks of a bucket in the fold + sum-of-squares kernel
uint32_t bucket_blocks(const shadow_ctx* c, uint64_t numel)
{
    return blocks_for(bucket_threads(numel), c->fold_block * sumsq_vpl(c->hp));
}

// Launch shape of the fold + optimizer kernel for a launch list of total_elems elements.
void fused_shape(const shadow_ctx* c, uint64_t total_elems, uint32_t* block, uint32_t* lds)
{
    const bool unrolled = unrolled_workers(c->hp.num_workers);
    *block = c->fused_block_given ? c->fused_block_given : (!unrolled ? kLoopBlock : total_elems < kFusedSmallLaunchElems ? 64u : 128u);
    uint32_t waves = c->fused_waves;
    if (!waves && !unrolled) waves = 32;
    if (!waves) {
        const uint32_t state_bytes = c->hp.optimizer == SHADOW_OPT_SGD ? 32u : 48u;
        const uint32_t lane_bytes = kVec * c->lay.grad_elem_bytes * c->hp.num_workers + state_bytes;
        const uint32_t wpb = *block / 64;
        const double want = double(kFusedBytesInFlightPerCu) / (64.0 * lane_bytes);
        waves = uint32_t(want / wpb + 0.5) * wpb;         // nearest whole number of blocks
        if (waves < 8) waves = 8;
        if (waves < wpb) waves = wpb;
    }
    *lds = lds_for_wave_cap(*block, waves);
}

int32_t get_event(shadow_ctx* c, hipEvent_t* out)
{
    if (!c->ev_pool.empty()) { *out = c->ev_pool.back(); c->ev_pool.pop_back(); return SHADOW_OK; }
    HIP_TRY(hipEventCreate(out));
    return SHADOW_OK;
}

struct ProfScope {
    shadow_ctx* c; uint32_t kind; hipStream_t st; hipEvent_t a = nullptr, b = nullptr; int32_t rc = SHADOW_OK; bool on = true;
    ProfScope(shadow_ctx* c_, uint32_t k, hipStream_t s) : c(c_), kind(k), st(s)
    {
        if (!c->profile || !((c->profile_kinds >> k) & 1u) || c->spans[k].size() >= kMaxSpansPerKind) { on = false; return; }
        rc = get_event(c, &a);
        if (rc == SHADOW_OK) rc = get_event(c, &b);
        if (rc == SHADOW_OK && hipEventRecord(a, st) != hipSuccess) rc = SHADOW_EHIP;
    }
    int32_t end()
    {
        if (!on || rc != SHADOW_OK) return rc;
        if (hipEventRecord(b, st) != hipSuccess) return SHADOW_EHIP;
        c->spans[kind].push_back({a, b});
        return SHADOW_OK;
    }
};

// The staging set while the running iteration is armed for a snapshot, else nothing.
SnapSet snap_set(const shadow_ctx* c)
{
    return c->snap_active ? SnapSet{c->stage_p, c->stage_m, c->stage_v} : SnapSet{nullptr, nullptr, nullptr};
}

// update == false: the fold of an arriving bucket (with clipping: sum of squares, reduced gradient stored unless
// re-fold mode).  update == true: fold + optimizer (clipping off: the only pass; re-fold mode: the second pass,
// scaled by the clip coefficient).
template <bool BF16, int W>
void launch_fold(shadow_ctx* c, const FoldBatch& fb, uint32_t grid, hipStream_t st, const WdMap& map, bool update, uint32_t fused_block,
                 uint32_t fused_lds)
{
    const float* coef = c->clip ? c->d_coef : nullptr;
    const SnapSet sn = snap_set(c);
    if (!update)
        k_fold_sumsq<BF16, W><<<grid, c->fold_block, c->fold_lds, st>>>(fb, c->r, c->d_partial, c->sc);
    else if (c->hp.optimizer == SHADOW_OPT_ADAMW)
        k_fold_adamw<BF16, W, kAdamW><<<grid, fused_block, fused_lds, st>>>(fb, c->p, c->m, c->v, coef, map, c->sc, sn);
    else if (c->hp.optimizer == SHADOW_OPT_ADAM)
        k_fold_adamw<BF16, W, kAdam><<<grid, fused_block, fused_lds, st>>>(fb, c->p, c->m, c->v, coef, map, c->sc, sn);
    else
        k_fold_adamw<BF16, W, kSgd><<<grid, fused_block, fused_lds, st>>>(fb, c->p, c->m, c->v, coef, map, c->sc, sn);
}

template <bool BF16>
void dispatch_fold(shadow_ctx* c, const FoldBatch& fb, uint32_t grid, hipStream_t st, const WdMap& map, bool update, uint32_t fblock,
                   uint32_t flds)
{
    switch (c->hp.num_workers) {
        case 1: launch_fold<BF16, 1>(c, fb, grid, st, map, update, fblock, flds); break;
        case 2: launch_fold<BF16, 2>(c, fb, grid, st, map, update, fblock, flds); break;
        case 4: launch_fold<BF16, 4>(c, fb, grid, st, map, update, fblock, flds); break;
        case 8: launch_fold<BF16, 8>(c, fb, grid, st, map, update, fblock, flds); break;
        case 16: launch_fold<BF16, 16>(c, fb, grid, st, map, update, fblock, flds); break;
        case 32: launch_fold<BF16, 32>(c, fb, grid, st, map, update, fblock, flds); break;
        case 64: launch_fold<BF16, 64>(c, fb, grid, st, map, update, fblock, flds); break;
        default: launch_fold<BF16, 0>(c, fb, grid, st, map, update, fblock, flds);
    }
}

WdMap wd_map(const shadow_ctx* c) { return WdMap{c->d_tile_mode, c->d_run_start, c->d_run_flag, c->num_runs}; }

// stream 0 waits for everything enqueued on the other streams
int32_t join_to_stream0(shadow_ctx* c)
{
    for (size_t s = 1; s < c->streams.size(); ++s) {
        if (!c->stream_dirty[s]) continue;
        HIP_TRY(hipEventRecord(c->join_ev[s], c->streams[s]));
        HIP_TRY(hipStreamWaitEvent(c->streams[0], c->join_ev[s], 0));
        c->stream_dirty[s] = 0;
    }
    return SHADOW_OK;
}

int32_t mark_boundary(shadow_ctx* c)
{
    HIP_TRY(hipEventRecord(c->boundary_ev, c->streams[0]));
    c->boundary_pending = true;
    return SHADOW_OK;
}

// A kernel that writes the replica is about to be enqueued on stream sid: copies of an earlier
// snapshot that still read the replica must have run first.
int32_t wait_for_snapshot_copies(shadow_ctx* c, uint32_t sid)
{
    if (!c->snap_wait[sid]) return SHADOW_OK;
    HIP_TRY(hipStreamWaitEvent(c->streams[sid], c->snap_ev, 0));
    c->snap_wait[sid] = 0;
    return SHADOW_OK;
}

// Fold the given buckets on stream st in as few launches as the descriptor allows.
// ptrs(i) yields the W view pointers of the i-th bucket of the list.
template <typename PtrFn>
int32_t launch_buckets(shadow_ctx* c, const uint32_t* ids, size_t count, PtrFn ptrs, uint32_t sid, bool update)
{
    const uint32_t W = c->hp.num_workers;
    const WdMap map = wd_map(c);
    hipStream_t st = c->streams[sid];
    if (update && count) {
        const int32_t rc = wait_for_snapshot_copies(c, sid);
        if (rc != SHADOW_OK) return rc;
    }
    uint32_t fblock = 0, flds = 0;
    if (update) {
        uint64_t total = 0;
        for (size_t j = 0; j < count; ++j) total += c->lay.buckets[ids[j]].numel;
        fused_shape(c, total, &fblock, &flds);
    }
    const uint32_t block = update ? fblock : c->fold_block;
    size_t i = 0;
    while (i < count) {
        FoldBatch fb{};
        fb.w = W;
        uint64_t blocks = 0;
        uint32_t k = 0;
        while (i < count && k < kMaxBatch && (k + 1) * W <= kMaxBatchPtrs) {
            const BucketL& b = c->lay.buckets[ids[i]];
            const uint64_t nb = update ? blocks_for(bucket_threads(b.numel), block) : bucket_blocks(c, b.numel);
            if (k > 0 && (blocks + nb) * block > c->max_launch_threads) break;
            fb.first_block[k] = uint32_t(blocks);
            fb.numel[k] = b.numel;
            fb.arena_off[k] = b.arena_off;
            fb.slot_base[k] = (c->clip && !update) ? c->slot_base[ids[i]] : 0u;
            const void* const* vp = ptrs(i);
            for (uint32_t w = 0; w < W; ++w) fb.ptr[k * W + w] = vp[w];
            blocks += nb;
            ++k;
            ++i;
        }
        fb.count = k;
        const uint32_t grid = uint32_t(blocks);
        for (uint32_t j = k; j <= kMaxBatch; ++j) fb.first_block[j] = kNoBucket;   // "no bucket starts here"
        ProfScope ps(c, update ? SHADOW_K_FOLD_ADAMW : SHADOW_K_FOLD_SUMSQ, st);
        if (ps.rc != SHADOW_OK) return ps.rc;
        if (c->hp.grad_dtype == SHADOW_GRAD_BF16) dispatch_fold<true>(c, fb, grid, st, map, update, fblock, flds);
        else dispatch_fold<false>(c, fb, grid, st, map, update, fblock, flds);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) {
            g_hip_error = std::string("fold kernel launch: ") + hipGetErrorString(e);
            return SHADOW_EHIP;
        }
        if (ps.end() != SHADOW_OK) return SHADOW_EHIP;
    }
    return SHADOW_OK;
}

// Launch everything buffered for stream sid.
int32_t flush_stream(shadow_ctx* c, uint32_t sid)
{
    std::vector<shadow_ctx::Pending>& q = c->pending[sid];
    if (q.empty()) return SHADOW_OK;
    std::vector<uint32_t> ids(q.size());
    for (size_t i = 0; i < q.size(); ++i) ids[i] = q[i].bucket;
    const int32_t rc = launch_buckets(c, ids.data(), ids.size(), [&](size_t i) { return q[i].ptr; }, sid,
                                      /*update=*/!c->clip);
    if (rc != SHADOW_OK) return rc;
    q.clear();
    c->pending_bytes[sid] = 0;
    c->stream_dirty[sid] = 1;
    return SHADOW_OK;
}

int32_t flush_all(shadow_ctx* c)
{
    for (uint32_t s = 0; s < c->streams.size(); ++s) {
        const int32_t rc = flush_stream(c, s);
        if (rc != SHADOW_OK) { c->poisoned = true; return rc; }
    }
    return SHADOW_OK;
}

void free_ctx(shadow_ctx* c)
{
    if (!c) return;
    for (auto& vec : c->spans) for (auto& sp : vec) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); }
    for (hipEvent_t e : c->ev_pool) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->join_ev) if (e) (void)hipEventDestroy(e);
    if (c->boundary_ev) (void)hipEventDestroy(c->boundary_ev);
    if (c->state_ev) (void)hipEventDestroy(c->state_ev);
    if (c->snap_ev) (void)hipEventDestroy(c->snap_ev);
    if (c->drain_ev) (void)hipEventDestroy(c->drain_ev);
    if (c->snap_stream) (void)hipStreamDestroy(c->snap_stream);
    for (hipEvent_t e : c->copied_ev) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->consumed_ev) if (e) (void)hipEventDestroy(e);
    if (c->copy_stream) (void)hipStreamDestroy(c->copy_stream);
    if (c->own_streams) for (hipStream_t s : c->streams) if (s) (void)hipStreamDestroy(s);
    (void)hipFree(c->d_tile_mode);
    (void)hipFree(c->d_run_start);
    (void)hipFree(c->d_run_flag);
    (void)hipFree(c->d_partial);
    (void)hipFree(c->d_stage1);
    (void)hipFree(c->d_coef);
    (void)hipFree(c->d_sumsq);
    delete c;
}

// Runs of equal weight-decay flag over the arena; an alignment gap is a run of its own kind.
void make_runs(const shadow_layout& L, std::vector<uint64_t>& start, std::vector<uint8_t>& flag)
{
    auto push = [&](uint64_t s, uint8_t f) {
        if (!flag.empty() && flag.back() == f) return;
        start.push_back(s);
        flag.push_back(f);
    };
    for (const BucketL& b : L.buckets) {
        for (const Seg& sg : b.segs) push(b.arena_off + sg.offset, sg.wd);
        const uint64_t end = b.arena_off + b.numel;
        const uint64_t padded = (end + kAlignElems - 1) / kAlignElems * kAlignElems;
        if (padded != end) push(end, kRunGap);
    }
    if (start.empty()) { start.push_back(0); flag.push_back(0); }
}

// Norm-partial slots: one per wave of each bucket's fold launch.  false: more than 2^31 - 1 slots.
bool assign_slots(shadow_ctx* c)
{
    const shadow_layout& L = c->lay;
    c->slot_base.resize(L.buckets.size());
    c->slot_count.resize(L.buckets.size());
    uint64_t total = 0;
    for (size_t b = 0; b < L.buckets.size(); ++b) {
        c->slot_base[b] = uint32_t(total);
        c->slot_count[b] = bucket_blocks(c, L.buckets[b].numel) * (c->fold_block / 64);
        total += c->slot_count[b];
        if (total > 0x7FFFFFFFull) return false;
    }
    c->nslots = uint32_t(total);
    c->nstage1 = uint32_t((total + kNormChunk - 1) / kNormChunk);
    if (c->nstage1 == 0) c->nstage1 = 1;
    return true;
}

int32_t build_tables(shadow_ctx* c)
{
    const shadow_layout& L = c->lay;
    std::vector<uint64_t> start;
    std::vector<uint8_t> flag;
    make_runs(L, start, flag);
    c->num_runs = uint32_t(start.size());
    const uint64_t ntiles = (L.arena_numel + (1ull << kWdTileShift) - 1) >> kWdTileShift;
    std::vector<uint8_t> mode(ntiles ? ntiles : 1, 0);
    for (size_t k = 0; k < start.size(); ++k) {
        const uint64_t s = start[k], e = (k + 1 < start.size()) ? start[k + 1] : L.arena_numel;
        if (e <= s) continue;
        for (uint64_t t = s >> kWdTileShift; t <= ((e - 1) >> kWdTileShift); ++t) mode[t] = flag[k];
    }
    for (size_t k = 1; k < start.size(); ++k)
        if (start[k] & ((1ull << kWdTileShift) - 1)) mode[start[k] >> kWdTileShift] = 2;
    HIP_TRY(hipMalloc(&c->d_tile_mode, mode.size()));
    HIP_TRY(hipMalloc(&c->d_run_start, start.size() * sizeof(uint64_t)));
    HIP_TRY(hipMalloc(&c->d_run_flag, flag.size()));
    HIP_TRY(hipMemcpy(c->d_tile_mode, mode.data(), mode.size(), hipMemcpyHostToDevice));
    HIP_TRY(hipMemcpy(c->d_run_start, start.data(), start.size() * sizeof(uint64_t), hipMemcpyHostToDevice));
    HIP_TRY(hipMemcpy(c->d_run_flag, flag.data(), flag.size(), hipMemcpyHostToDevice));
    // alignment gaps are kept at zero in every arena so that whole-arena sweeps may pass over them
    for (const BucketL& b : L.buckets) {
        const uint64_t end = b.arena_off + b.numel;
        const uint64_t padded = (end + kAlignElems - 1) / kAlignElems * kAlignElems;
        if (padded == end) continue;
        const size_t bytes = (padded - end) * sizeof(float);
        HIP_TRY(hipMemset(c->p + end, 0, bytes));
        HIP_TRY(hipMemset(c->m + end, 0, bytes));
        if (c->v) HIP_TRY(hipMemset(c->v + end, 0, bytes));
        if (c->r) HIP_TRY(hipMemset(c->r + end, 0, bytes));
    }
    if (c->clip) {
        if (!assign_slots(c)) return SHADOW_EINVAL;
        const uint64_t total = c->nslots;
        HIP_TRY(hipMalloc(&c->d_partial, (total ? total : 1) * sizeof(double)));
        HIP_TRY(hipMalloc(&c->d_stage1, c->nstage1 * sizeof(double)));
        HIP_TRY(hipMalloc(&c->d_coef, sizeof(float)));
        HIP_TRY(hipMalloc(&c->d_sumsq, sizeof(double)));
        HIP_TRY(hipMemset(c->d_partial, 0, (total ? total : 1) * sizeof(double)));
        HIP_TRY(hipMemset(c->d_coef, 0, sizeof(float)));
        HIP_TRY(hipMemset(c->d_sumsq, 0, sizeof(double)));
    }
    HIP_TRY(hipDeviceSynchronize());
    return SHADOW_OK;
}

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

}  // namespace

extern "C" {

int32_t shadow_layout_create(shadow_layout** out, const shadow_tensor_desc* tensors, uint32_t num_tensors,
                             const uint32_t* bucket_of_tensor, uint32_t grad_elem_bytes, uint64_t bucket_cap_bytes)
{
    if (!out) return SHADOW_EINVAL;
    *out = nullptr;
    if (!tensors || num_tensors == 0) return SHADOW_EINVAL;
    if (grad_elem_bytes != 2 && grad_elem_bytes != 4) return SHADOW_EINVAL;
    if (!bucket_of_tensor && bucket_cap_bytes == 0) return SHADOW_EINVAL;
    uint64_t total = 0;
    for (uint32_t t = 0; t < num_tensors; ++t) {
        if (tensors[t].numel == 0 || tensors[t].weight_decay > 1 || tensors[t].reserved != 0) return SHADOW_EINVAL;
        if (tensors[t].numel > (1ull << 48)) return SHADOW_EINVAL;
        total += tensors[t].numel;
        if (total > (1ull << 48)) return SHADOW_EINVAL;
    }
    shadow_layout* L = new (std::nothrow) shadow_layout();
    if (!L) return SHADOW_ENOMEM;
    try {
        L->tensors.assign(tensors, tensors + num_tensors);
        L->grad_elem_bytes = grad_elem_bytes;
        if (!plan(*L, bucket_of_tensor, bucket_cap_bytes)) { delete L; return SHADOW_EINVAL; }
    } catch (const std::bad_alloc&) {
        delete L;
        return SHADOW_ENOMEM;
    }
    *out = L;
    return SHADOW_OK;
}

int32_t shadow_layout_destroy(shadow_layout* layout)
{
    delete layout;
    return SHADOW_OK;
}

int32_t shadow_layout_num_buckets(const shadow_layout* L, uint32_t* out)
{
    if (!L || !out) return SHADOW_EINVAL;
    *out = uint32_t(L->buckets.size());
    return SHADOW_OK;
}

int32_t shadow_layout_num_params(const shadow_layout* L, uint64_t* out)
{
    if (!L || !out) return SHADOW_EINVAL;
    *out = L->num_params;
    return SHADOW_OK;
}

int32_t shadow_layout_arena_numel(const shadow_layout* L, uint64_t* out)
{
    if (!L || !out) return SHADOW_EINVAL;
    *out = L->arena_numel;
    return SHADOW_OK;
}

int32_t shadow_layout_bucket(const shadow_layout* L, uint32_t bucket, uint64_t* arena_offset, uint64_t* numel,
                             uint32_t* num_tensors)
{
    if (!L) return SHADOW_EINVAL;
    if (bucket >= L->buckets.size()) return SHADOW_EBUCKET;
    if (arena_offset) *arena_offset = L->buckets[bucket].arena_off;
    if (numel) *numel = L->buckets[bucket].numel;
    if (num_tensors) *num_tensors = uint32_t(L->buckets[bucket].segs.size());
    return SHADOW_OK;
}

int32_t shadow_layout_tensor(const shadow_layout* L, uint32_t tensor, uint32_t* bucket, uint64_t* offset_in_bucket,
                             uint64_t* arena_offset)
{
    if (!L || tensor >= L->tensors.size()) return SHADOW_EINVAL;
    const uint32_t b = L->bucket_of[tensor];
    if (bucket) *bucket = b;
    if (offset_in_bucket) *offset_in_bucket = L->off_in_bucket[tensor];
    if (arena_offset) *arena_offset = L->buckets[b].arena_off + L->off_in_bucket[tensor];
    return SHADOW_OK;
}

int32_t shadow_layout_device_plan(const shadow_layout* L, int32_t with_scratch, int32_t with_snapshot_set, uint64_t staging_bytes,
                                  shadow_device_plan* plan)
{
    if (!L || !plan) return SHADOW_EINVAL;
    constexpr uint64_t kGiB = 1ull << 30, kRegion = 96 * kGiB, kBlock = 256 * kGiB;
    const uint64_t arena = L->arena_numel * sizeof(float);
    const uint64_t a = (arena + kGiB - 1) / kGiB * kGiB + kGiB;       // arena rounded up, plus a margin
    if (2 * a > kRegion) return SHADOW_ENOMEM;
    shadow_device_plan out{};
    out.block_bytes = kBlock;
    out.m_offset = kRegion - a;                 // param and m end the first region
    out.param_offset = out.m_offset - a;
    out.v_offset = kRegion + kGiB;              // v starts the second
    uint64_t tail = out.v_offset + a;
    if (with_scratch) {
        if (3 * a <= kRegion) {
            out.scratch_offset = out.param_offset - a;   // written by the fold: away from the views
        } else {
            out.scratch_offset = tail;
            tail += a;
        }
    }
    if (with_snapshot_set) {
        out.snap_param_offset = tail;
        out.snap_m_offset = tail + a;
        out.snap_v_offset = tail + 2 * a;
        tail += 3 * a;
    }
    if (staging_bytes) {
        if (staging_bytes > kBlock) return SHADOW_ENOMEM;
        out.staging_offset = tail;
        tail += staging_bytes;
    }
    if (tail > kBlock) return SHADOW_ENOMEM;
    *plan = out;
    return SHADOW_OK;
}

int32_t shadow_layout_arena_stride(const shadow_layout* L, uint64_t* stride_bytes)
{
    if (!L || !stride_bytes) return SHADOW_EINVAL;
    uint64_t s = 2ull << 20;
    while (s < L->arena_numel * sizeof(float)) s <<= 1;
    *stride_bytes = s;
    return SHADOW_OK;
}

namespace {
constexpr uint64_t kStagingSkew = 4096;
uint64_t staging_view_stride(const shadow_layout* L, uint32_t bucket)
{
    const uint64_t bytes = L->buckets[bucket].numel * L->grad_elem_bytes;
    if (bytes < (2ull << 20)) return (bytes + 255) / 256 * 256;
    // One page more than a multiple of 2 MiB: the fold reads the same offset of all W views at
    // the same time, and views a multiple of 2 MiB apart would send those reads to the same
    // DRAM channel and bank.
    return (bytes + (2ull << 20) - 1) / (2ull << 20) * (2ull << 20) + kStagingSkew;
}
uint64_t staging_bucket_start(const shadow_layout* L, uint32_t num_workers, uint32_t bucket)
{
    uint64_t off = 0;
    for (uint32_t b = 0; b < bucket; ++b) {
        off += staging_view_stride(L, b) * num_workers;
        off = (off + (2ull << 20) - 1) & ~((2ull << 20) - 1);
    }
    return off;
}
}  // namespace

int32_t shadow_layout_staging_bytes(const shadow_layout* L, uint32_t num_workers, uint64_t* bytes)
{
    if (!L || !bytes || num_workers < 1 || num_workers > SHADOW_MAX_WORKERS) return SHADOW_EINVAL;
    *bytes = staging_bucket_start(L, num_workers, uint32_t(L->buckets.size()));
    return SHADOW_OK;
}

int32_t shadow_layout_staging_view(const shadow_layout* L, uint32_t num_workers, uint32_t bucket, uint32_t worker,
                                   uint64_t* byte_offset)
{
    if (!L || !byte_offset || num_workers < 1 || num_workers > SHADOW_MAX_WORKERS || worker >= num_workers) return SHADOW_EINVAL;
    if (bucket >= L->buckets.size()) return SHADOW_EBUCKET;
    *byte_offset = staging_bucket_start(L, num_workers, bucket) + staging_view_stride(L, bucket) * worker;
    return SHADOW_OK;
}

}  // extern "C"

namespace {

// What every way of creating or running a replica checks before it touches the GPU.
int32_t check_replica_args(const shadow_layout* layout, const shadow_hparams* hp, const float* d_param, const float* d_m,
                           const float* d_v, const float* d_reduced)
{
    if (!layout || !hp || !d_param || !d_m) return SHADOW_EINVAL;
    if (hp->optimizer != SHADOW_OPT_ADAMW && hp->optimizer != SHADOW_OPT_ADAM && hp->optimizer != SHADOW_OPT_SGD) return SHADOW_EINVAL;
    const bool sgd = hp->optimizer == SHADOW_OPT_SGD;
    if (sgd ? d_v != nullptr : d_v == nullptr) return SHADOW_EINVAL;       // SGD keeps one state array only
    if (!(hp->lr >= 0.f) || !(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->weight_decay >= 0.f) || std::isnan(hp->max_grad_norm))
        return SHADOW_EINVAL;
    if (!sgd && (!(hp->beta2 >= 0.f && hp->beta2 < 1.f) || !(hp->eps > 0.f))) return SHADOW_EINVAL;
    if (hp->num_workers < 1 || hp->num_workers > SHADOW_MAX_WORKERS) return SHADOW_EINVAL;
    if (hp->grad_dtype != SHADOW_GRAD_F32 && hp->grad_dtype != SHADOW_GRAD_BF16) return SHADOW_EINVAL;
    if ((hp->grad_dtype == SHADOW_GRAD_BF16 ? 2u : 4u) != layout->grad_elem_bytes) return SHADOW_EINVAL;
    if (hp->reduce_op != SHADOW_REDUCE_MEAN && hp->reduce_op != SHADOW_REDUCE_SUM) return SHADOW_EINVAL;
    if (hp->num_streams < 1 || hp->num_streams > SHADOW_MAX_STREAMS) return SHADOW_EINVAL;
    const shadow_launch_shape& ls = hp->launch;
    if ((ls.fold_block && !valid_block(ls.fold_block)) || (ls.fused_block && !valid_block(ls.fused_block)) ||
        (ls.sweep_block && !valid_block(ls.sweep_block)))
        return SHADOW_EINVAL;
    if (ls.fold_waves_per_cu > 32 || ls.fused_waves_per_cu > 32 || ls.sweep_waves_per_cu > 32 || ls.drain_blocks > 4096 || ls.reserved != 0 ||
        ls.max_launch_threads > kMaxThreadsPerLaunch)
        return SHADOW_EINVAL;
    const bool clip = hp->max_grad_norm > 0.f;
    if (!clip && d_reduced) return SHADOW_EINVAL;
    if (!aligned(d_param, 256) || !aligned(d_m, 256) || !aligned(d_v, 256) || !aligned(d_reduced, 256)) return SHADOW_EINVAL;
    if (d_param == d_m || d_param == d_v || d_m == d_v) return SHADOW_EINVAL;

    for (const BucketL& b : layout->buckets)
        if (bucket_threads(b.numel) > kMaxThreadsPerLaunch) return SHADOW_EINVAL;   // one launch per bucket
    return SHADOW_OK;
}

// Launch shape of a context from the hyper-parameters (zero fields take the defaults).
void set_launch_shape(shadow_ctx* c, const shadow_launch_shape& ls)
{
    const uint32_t fold_lane_bytes = kVec * c->lay.grad_elem_bytes * c->hp.num_workers * sumsq_vpl(c->hp);
    const bool unrolled = unrolled_workers(c->hp.num_workers);
    const bool wide = unrolled && fold_lane_bytes > 64;
    const bool narrow = unrolled && sumsq_vpl(c->hp) > 1;
    c->fold_block = ls.fold_block ? ls.fold_block : (!unrolled ? kLoopBlock : (wide || narrow) ? kWideFoldBlock : kDefaultFoldBlock);
    uint32_t fold_waves = ls.fold_waves_per_cu;
    if (!fold_waves) {
        fold_waves = kDefaultFoldWaves;
        if (wide) {
            const uint32_t wpb = c->fold_block / 64;
            fold_waves = uint32_t(double(kFoldBytesInFlightPerCu) / (64.0 * fold_lane_bytes) / wpb + 0.5) * wpb;
            if (fold_waves < 8) fold_waves = 8;
            if (fold_waves < wpb) fold_waves = wpb;
        }
    }
    c->fused_block_given = ls.fused_block;
    c->fused_waves = ls.fused_waves_per_cu;
    c->drain_blocks = ls.drain_blocks ? ls.drain_blocks : kDefaultDrainBlocks;
    c->adamw_block = ls.sweep_block ? ls.sweep_block : kDefaultSweepBlock;
    c->fold_lds = lds_for_wave_cap(c->fold_block, fold_waves);
    c->adamw_lds = lds_for_wave_cap(c->adamw_block, ls.sweep_waves_per_cu ? ls.sweep_waves_per_cu : kDefaultSweepWaves);
    c->max_launch_threads = ls.max_launch_threads ? ls.max_launch_threads : kMaxThreadsPerLaunch;
}

}  // namespace

extern "C" {

int32_t shadow_init(shadow_ctx** out, const shadow_layout* layout, const shadow_hparams* hp, float* d_param, float* d_m,
                    float* d_v, float* d_reduced, uint64_t start_step, void* const* streams)
{
    if (!out) return SHADOW_EINVAL;
    *out = nullptr;
    const int32_t chk = check_replica_args(layout, hp, d_param, d_m, d_v, d_reduced);
    if (chk != SHADOW_OK) return chk;
    const bool clip = hp->max_grad_norm > 0.f;
    const shadow_launch_shape& ls = hp->launch;

    shadow_ctx* c = new (std::nothrow) shadow_ctx();
    if (!c) return SHADOW_ENOMEM;
    int32_t rc = SHADOW_OK;
    try {
        c->lay = *layout;
        c->hp = *hp;
        c->p = d_param; c->m = d_m; c->v = d_v; c->r = d_reduced;
        c->clip = clip;
        c->refold = clip && !d_reduced;
        if (c->refold) c->step_views.assign(layout->buckets.size() * size_t(hp->num_workers), nullptr);
        c->completed = start_step;
        set_launch_shape(c, ls);
        c->snap_wait.assign(hp->num_streams, 0);
        c->arrived.assign(layout->buckets.size(), 0);
        c->stream_dirty.assign(hp->num_streams, 0);
        c->streams.assign(hp->num_streams, nullptr);
        c->join_ev.assign(hp->num_streams, nullptr);
        c->pending.assign(hp->num_streams, {});
        c->pending_bytes.assign(hp->num_streams, 0);
    } catch (const std::bad_alloc&) {
        delete c;
        return SHADOW_ENOMEM;
    }
    auto fail = [&](int32_t code) { free_ctx(c); return code; };
    if (streams) {
        for (uint32_t s = 0; s < hp->num_streams; ++s) c->streams[s] = static_cast<hipStream_t>(streams[s]);
    } else {
        c->own_streams = true;
        for (uint32_t s = 0; s < hp->num_streams; ++s) {
            if (hipStreamCreateWithFlags(&c->streams[s], hipStreamNonBlocking) != hipSuccess) {
                g_hip_error = "hipStreamCreateWithFlags failed";
                return fail(SHADOW_EHIP);
            }
        }
    }
    for (uint32_t s = 0; s < hp->num_streams; ++s) {
        if (hipEventCreateWithFlags(&c->join_ev[s], hipEventDisableTiming) != hipSuccess) {
            g_hip_error = "hipEventCreate failed";
            return fail(SHADOW_EHIP);
        }
    }
    if (hipEventCreateWithFlags(&c->boundary_ev, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->state_ev, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->snap_ev, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->drain_ev, hipEventDisableTiming) != hipSuccess) {
        g_hip_error = "hipEventCreate failed";
        return fail(SHADOW_EHIP);
    }
    if (hipStreamCreateWithFlags(&c->snap_stream, hipStreamNonBlocking) != hipSuccess) {
        g_hip_error = "hipStreamCreateWithFlags failed";
        return fail(SHADOW_EHIP);
    }
    rc = build_tables(c);
    if (rc != SHADOW_OK) return fail(rc);
    *out = c;
    return SHADOW_OK;
}

}  // extern "C"

namespace {

// the checks every delivery of a bucket must pass before anything is enqueued (section 4.1: exactly once per iteration)
int32_t precheck_bucket(const shadow_ctx* c, uint32_t bucket_id, const void* const* views, uint64_t step)
{
    if (!c || !views) return SHADOW_EINVAL;
    if (c->poisoned) return SHADOW_EHIP;
    if (bucket_id >= c->lay.buckets.size()) return SHADOW_EBUCKET;
    if (step != c->completed + 1) return SHADOW_ESTEP;
    if (c->arrived[bucket_id]) return SHADOW_EDUP;
    return SHADOW_OK;
}

// The plain copy kernel over `bytes` (a multiple of 16) on `stream`, as several launches where one would be too large.
int32_t launch_copy(void* d_dst, const void* d_src, uint64_t bytes, hipStream_t stream, uint64_t max_launch_threads)
{
    const uint64_t n16 = bytes >> 4;
    const uint32_t block = 256;
    uint64_t per_launch = max_launch_threads / block;
    if (per_launch < 1) per_launch = 1;
    const uint64_t blocks = (n16 + block - 1) / block;
    for (uint64_t b0 = 0; b0 < blocks; b0 += per_launch) {
        const uint64_t nb = blocks - b0 < per_launch ? blocks - b0 : per_launch;
        k_copy<<<uint32_t(nb), block, 0, stream>>>(static_cast<const u32x4*>(d_src), static_cast<u32x4*>(d_dst), n16, b0);
    }
    HIP_TRY(hipGetLastError());
    return SHADOW_OK;
}

// One array of the replica (or of the staging set) to a snapshot destination, on the copy stream.  Pinned host
// memory is written by the small drain kernel through its device-side mapping, device memory by the plain copy
// kernel (twice the rate of the runtime's device-to-device copy here), host memory the device cannot address by
// the runtime's copy.
int32_t snapshot_copy(shadow_ctx* c, float* dst, const float* src, size_t bytes)
{
    hipPointerAttribute_t attr{};
    const bool known = hipPointerGetAttributes(&attr, dst) == hipSuccess;
    if (!known) (void)hipGetLastError();          // a pointer the runtime does not know leaves an error behind: not ours
    const bool vec = aligned(dst, 16) && bytes % 16 == 0;
    void* mapped = nullptr;
    if (known && vec && attr.type == hipMemoryTypeHost && hipHostGetDevicePointer(&mapped, dst, 0) == hipSuccess && mapped &&
        aligned(mapped, 16)) {
        k_drain<<<c->drain_blocks, 256, 0, c->snap_stream>>>(reinterpret_cast<const u32x4*>(src), static_cast<u32x4*>(mapped), bytes >> 4);
        HIP_TRY(hipGetLastError());
        return SHADOW_OK;
    }
    if (known && vec && attr.type == hipMemoryTypeDevice) return launch_copy(dst, src, bytes, c->snap_stream, c->max_launch_threads);
    HIP_TRY(hipMemcpyAsync(dst, src, bytes, hipMemcpyDefault, c->snap_stream));
    return SHADOW_OK;
}

// The iteration that just completed was armed: its update kernels wrote the staging set as well.
// Order the copy stream behind them and drain the staging set to the host arrays, if any were given.
int32_t finish_armed_snapshot(shadow_ctx* c, uint64_t step)
{
    int32_t rc = join_to_stream0(c);
    if (rc != SHADOW_OK) return rc;
    HIP_TRY(hipEventRecord(c->state_ev, c->streams[0]));
    HIP_TRY(hipStreamWaitEvent(c->snap_stream, c->state_ev, 0));
    const size_t bytes = c->lay.arena_numel * sizeof(float);
    ProfScope ps(c, SHADOW_K_SNAPSHOT, c->snap_stream);
    if (ps.rc != SHADOW_OK) return ps.rc;
    if (c->armed_host[0] && (rc = snapshot_copy(c, c->armed_host[0], c->stage_p, bytes)) != SHADOW_OK) return rc;
    if (c->armed_host[1] && (rc = snapshot_copy(c, c->armed_host[1], c->stage_m, bytes)) != SHADOW_OK) return rc;
    if (c->armed_host[2] && c->stage_v && (rc = snapshot_copy(c, c->armed_host[2], c->stage_v, bytes)) != SHADOW_OK) return rc;
    if (ps.end() != SHADOW_OK) return SHADOW_EHIP;
    HIP_TRY(hipEventRecord(c->drain_ev, c->snap_stream));
    c->drain_recorded = c->armed_host[0] || c->armed_host[1] || (c->armed_host[2] && c->stage_v);
    c->snap_active = false;
    c->have_snapshot = true;
    c->last_snap_ev = c->drain_ev;
    c->last_snap_step = step;
    return SHADOW_OK;
}

// Every bucket of the iteration has been folded (clipping on): the norm over all of them, the clip
// coefficient, then the update of every bucket, all on stream 0 behind the folds.
int32_t enqueue_norm_and_update(shadow_ctx* c, bool single_stream = false)
{
    const uint32_t W = c->hp.num_workers;
    const WdMap map = wd_map(c);
    int32_t rc = single_stream ? int32_t(SHADOW_OK) : join_to_stream0(c);
    if (rc != SHADOW_OK) return rc;
    hipStream_t s0 = c->streams[0];
    {
        ProfScope ps(c, SHADOW_K_NORM, s0);
        if (ps.rc != SHADOW_OK) return ps.rc;
        k_norm_stage1<<<c->nstage1, kNormBlock, 0, s0>>>(c->d_partial, c->nslots, c->d_stage1);
        k_norm_finalize<<<1, kNormBlock, 0, s0>>>(c->d_stage1, c->nstage1, c->hp.max_grad_norm, c->d_coef, c->d_sumsq);
        HIP_TRY(hipGetLastError());
        if (ps.end() != SHADOW_OK) return SHADOW_EHIP;
    }
    if (c->refold) {
        // the reduced gradient was not stored: fold every bucket again, now scaled by the coefficient
        std::vector<uint32_t> ids(c->lay.buckets.size());
        for (size_t i = 0; i < ids.size(); ++i) ids[i] = uint32_t(i);
        rc = launch_buckets(c, ids.data(), ids.size(), [&](size_t i) { return c->step_views.data() + i * W; }, 0, /*update=*/true);
        if (rc != SHADOW_OK) return rc;
    } else {
        rc = wait_for_snapshot_copies(c, 0);
        if (rc != SHADOW_OK) return rc;
        ProfScope ps(c, SHADOW_K_ADAMW, s0);
        if (ps.rc != SHADOW_OK) return ps.rc;
        const SnapSet sn = snap_set(c);
        const uint64_t nvec = c->lay.arena_numel >> 2;      // the arena is a multiple of 64 elements
        uint64_t per_launch = c->max_launch_threads / c->adamw_block;
        if (per_launch < 1) per_launch = 1;
        const uint64_t blocks = (nvec + c->adamw_block - 1) / c->adamw_block;
        for (uint64_t b0 = 0; b0 < blocks; b0 += per_launch) {
            const uint64_t nb = blocks - b0 < per_launch ? blocks - b0 : per_launch;
            if (c->hp.optimizer == SHADOW_OPT_ADAMW)
                k_adamw<kAdamW><<<uint32_t(nb), c->adamw_block, c->adamw_lds, s0>>>(c->r, c->p, c->m, c->v, nvec, b0, c->d_coef, map, c->sc, sn);
            else if (c->hp.optimizer == SHADOW_OPT_ADAM)
                k_adamw<kAdam><<<uint32_t(nb), c->adamw_block, c->adamw_lds, s0>>>(c->r, c->p, c->m, c->v, nvec, b0, c->d_coef, map, c->sc, sn);
            else
                k_adamw<kSgd><<<uint32_t(nb), c->adamw_block, c->adamw_lds, s0>>>(c->r, c->p, c->m, c->v, nvec, b0, c->d_coef, map, c->sc, sn);
        }
        HIP_TRY(hipGetLastError());
        if (ps.end() != SHADOW_OK) return SHADOW_EHIP;
    }
    c->stream_dirty[0] = 1;
    return single_stream ? int32_t(SHADOW_OK) : mark_boundary(c);      // one stream: order is the stream's, no event
}

int32_t enqueue_norm_and_update_on_one_stream(shadow_ctx* c) { return enqueue_norm_and_update(c, true); }

int32_t apply_bucket_impl(shadow_ctx* c, uint32_t bucket_id, const void* const* d_grad_views, uint64_t step, void* ready_event,
                          bool launch_now)
{
    int32_t pre = precheck_bucket(c, bucket_id, d_grad_views, step);
    if (pre != SHADOW_OK) return pre;
    const uint32_t W = c->hp.num_workers;
    shadow_ctx::Pending pend{};
    pend.bucket = bucket_id;
    for (uint32_t w = 0; w < W; ++w) {
        if (!d_grad_views[w] || !aligned(d_grad_views[w], 16)) return SHADOW_EINVAL;
        pend.ptr[w] = d_grad_views[w];
    }
    const BucketL& b = c->lay.buckets[bucket_id];
    const uint32_t S = uint32_t(c->streams.size());
    const uint32_t sid = bucket_id % S;
    try {
        c->pending[sid].reserve(c->pending[sid].size() + 1);
    } catch (const std::bad_alloc&) {
        return SHADOW_ENOMEM;
    }
    // The producer of the views: the bucket's stream waits for it here, so every later launch on that
    // stream (this bucket's fold may be deferred) is ordered behind it.  A wait enqueued for a call
    // that then fails is harmless.
    if (ready_event) HIP_TRY(hipStreamWaitEvent(c->streams[sid], static_cast<hipEvent_t>(ready_event), 0));
    // ---- nothing above changed the replica or the bookkeeping; from here on work is buffered or enqueued ----
    auto hip_fail = [&](const char* what, hipError_t e) {
        g_hip_error = std::string(what) + ": " + hipGetErrorString(e);
        c->poisoned = true;
        return int32_t(SHADOW_EHIP);
    };
    auto poison = [&](int32_t rc) { c->poisoned = true; return rc; };
    hipError_t e;
    if (c->arrived_count == 0) {
        if (c->sc_step != step) { compute_scalars(c->hp, step, c->sc); c->sc_step = step; }
        c->snap_active = c->armed;            // an armed snapshot belongs to the iteration that starts now
        c->armed = false;
        if (c->boundary_pending) {
            // the whole-arena update of the previous iteration ran on stream 0 and read the reduced-gradient
            // arena; every other stream orders behind it before touching the arenas again
            for (uint32_t s = 1; s < S; ++s)
                if ((e = hipStreamWaitEvent(c->streams[s], c->boundary_ev, 0)) != hipSuccess) return hip_fail("hipStreamWaitEvent", e);
            c->boundary_pending = false;
        }
    }
    c->pending[sid].push_back(pend);          // capacity was reserved above
    if (c->refold)
        for (uint32_t w = 0; w < W; ++w) c->step_views[size_t(bucket_id) * W + w] = pend.ptr[w];
    c->pending_bytes[sid] += b.numel * c->lay.grad_elem_bytes * W;
    const bool last = c->arrived_count + 1 == c->lay.buckets.size();
    if (last) {
        const int32_t rc = flush_all(c);
        if (rc != SHADOW_OK) return rc;
    } else if (launch_now || c->pending_bytes[sid] >= c->hp.batch_bytes) {
        const int32_t rc = flush_stream(c, sid);
        if (rc != SHADOW_OK) return poison(rc);
    }
    c->arrived[bucket_id] = 1;
    c->arrived_count++;
    if (c->arrived_count == c->lay.buckets.size()) {
        if (c->clip) {
            const int32_t rc = enqueue_norm_and_update(c);
            if (rc != SHADOW_OK) return poison(rc);
        }
        if (c->snap_active) {
            const int32_t rc = finish_armed_snapshot(c, step);
            if (rc != SHADOW_OK) return poison(rc);
        }
        std::fill(c->arrived.begin(), c->arrived.end(), uint8_t(0));
        c->arrived_count = 0;
        c->completed = step;
    }
    return SHADOW_OK;
}

}  // namespace

extern "C" {

int32_t shadow_apply_bucket(shadow_ctx* c, uint32_t bucket_id, const void* const* d_grad_views, uint64_t step, void* ready_event)
{
    return apply_bucket_impl(c, bucket_id, d_grad_views, step, ready_event, /*launch_now=*/false);
}

int32_t shadow_num_buckets(const shadow_ctx* c, uint32_t* out)
{
    if (!c || !out) return SHADOW_EINVAL;
    *out = uint32_t(c->lay.buckets.size());
    return SHADOW_OK;
}

int32_t shadow_bucket_info(const shadow_ctx* c, uint32_t bucket_id, uint64_t* arena_offset, uint64_t* numel)
{
    if (!c) return SHADOW_EINVAL;
    if (bucket_id >= c->lay.buckets.size()) return SHADOW_EBUCKET;
    if (arena_offset) *arena_offset = c->lay.buckets[bucket_id].arena_off;
    if (numel) *numel = c->lay.buckets[bucket_id].numel;
    return SHADOW_OK;
}

int32_t shadow_record_consumed(shadow_ctx* c, uint32_t bucket_id, void* event)
{
    if (!c || !event) return SHADOW_EINVAL;
    if (c->poisoned) return SHADOW_EHIP;
    if (bucket_id >= c->lay.buckets.size()) return SHADOW_EBUCKET;
    if (c->refold && c->arrived_count != 0) return SHADOW_EBUSY;   // the open iteration's views are read once more at its end
    const uint32_t sid = bucket_id % uint32_t(c->streams.size());
    const int32_t rc = flush_stream(c, sid);
    if (rc != SHADOW_OK) { c->poisoned = true; return rc; }
    // In re-fold mode the last reader of a finished iteration's views ran on stream 0, which
    // every stream of the next iteration is ordered behind; outside it, on the bucket's stream.
    hipStream_t st = c->refold ? c->streams[0] : c->streams[sid];
    HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(event), st));
    return SHADOW_OK;
}

int32_t shadow_ingest_attach(shadow_ctx* c, void* d_ring, uint64_t ring_bytes)
{
    if (!c || !d_ring || !aligned(d_ring, 256)) return SHADOW_EINVAL;
    if (c->refold) return SHADOW_EINVAL;          // folding twice needs the whole iteration's views to persist
    if (c->arrived_count != 0) return SHADOW_EBUSY;
    if (c->ring) return SHADOW_EINVAL;
    uint64_t max_numel = 0;
    for (const BucketL& b : c->lay.buckets) if (b.numel > max_numel) max_numel = b.numel;
    const uint64_t view_stride = (max_numel * c->lay.grad_elem_bytes + 255) / 256 * 256;
    const uint64_t slot_bytes = view_stride * c->hp.num_workers;
    const uint64_t nslots = ring_bytes / slot_bytes;
    if (nslots < 1) return SHADOW_EINVAL;
    const uint32_t n = uint32_t(nslots > 64 ? 64 : nslots);
    // a call that failed half-way left its stream and events with the context: they are used again, not made twice
    if (!c->copy_stream) HIP_TRY(hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking));
    try {
        if (c->copied_ev.size() < n) c->copied_ev.resize(n, nullptr);
        if (c->consumed_ev.size() < n) c->consumed_ev.resize(n, nullptr);
        c->consumed_valid.assign(n, 0);
    } catch (const std::bad_alloc&) {
        return SHADOW_ENOMEM;
    }
    for (uint32_t i = 0; i < n; ++i) {
        if (!c->copied_ev[i]) HIP_TRY(hipEventCreateWithFlags(&c->copied_ev[i], hipEventDisableTiming));
        if (!c->consumed_ev[i]) HIP_TRY(hipEventCreateWithFlags(&c->consumed_ev[i], hipEventDisableTiming));
    }
    c->ring = static_cast<char*>(d_ring);
    c->view_stride = view_stride;
    c->slot_bytes = slot_bytes;
    c->ring_slots = n;
    c->ring_next = 0;
    return SHADOW_OK;
}

int32_t shadow_ingest_bucket(shadow_ctx* c, uint32_t bucket_id, const void* const* h_grad_views, uint64_t step, void* ready_event)
{
    int32_t pre = precheck_bucket(c, bucket_id, h_grad_views, step);
    if (pre != SHADOW_OK) return pre;
    if (!c->ring) return SHADOW_EINVAL;
    const uint32_t W = c->hp.num_workers;
    for (uint32_t w = 0; w < W; ++w)
        if (!h_grad_views[w]) return SHADOW_EINVAL;
    // ---- nothing above changed any state ----
    const BucketL& b = c->lay.buckets[bucket_id];
    const uint64_t bytes = b.numel * c->lay.grad_elem_bytes;
    const uint32_t slot = c->ring_next;
    char* base = c->ring + uint64_t(slot) * c->slot_bytes;
    hipStream_t st = c->streams[bucket_id % c->streams.size()];
    auto fail = [&](const char* what, hipError_t e) {
        g_hip_error = std::string(what) + ": " + hipGetErrorString(e);
        c->poisoned = true;
        return int32_t(SHADOW_EHIP);
    };
    hipError_t e;
    if (ready_event && (e = hipStreamWaitEvent(c->copy_stream, static_cast<hipEvent_t>(ready_event), 0)) != hipSuccess) {
        g_hip_error = std::string("hipStreamWaitEvent(ready_event): ") + hipGetErrorString(e);
        return SHADOW_EHIP;                    // nothing was enqueued
    }
    // the slot's previous occupant must have been folded before it is overwritten
    if (c->consumed_valid[slot] && (e = hipStreamWaitEvent(c->copy_stream, c->consumed_ev[slot], 0)) != hipSuccess)
        return fail("hipStreamWaitEvent", e);
    const void* dev_views[kMaxWorkers];
    for (uint32_t w = 0; w < W; ++w) {
        char* dst = base + uint64_t(w) * c->view_stride;
        if ((e = hipMemcpyAsync(dst, h_grad_views[w], bytes, hipMemcpyHostToDevice, c->copy_stream)) != hipSuccess)
            return fail("hipMemcpyAsync", e);
        dev_views[w] = dst;
    }
    if ((e = hipEventRecord(c->copied_ev[slot], c->copy_stream)) != hipSuccess) return fail("hipEventRecord", e);
    if ((e = hipStreamWaitEvent(st, c->copied_ev[slot], 0)) != hipSuccess) return fail("hipStreamWaitEvent", e);
    const int32_t rc = apply_bucket_impl(c, bucket_id, dev_views, step, nullptr, /*launch_now=*/true);
    if (rc != SHADOW_OK) { c->poisoned = true; return rc; }      // cannot happen after the precheck except for HIP failures
    if ((e = hipEventRecord(c->consumed_ev[slot], st)) != hipSuccess) return fail("hipEventRecord", e);
    c->consumed_valid[slot] = 1;
    c->ring_next = (slot + 1) % c->ring_slots;
    return SHADOW_OK;
}

int32_t shadow_snapshot(shadow_ctx* c, float* dst_param, float* dst_m, float* dst_v, uint64_t* out_step, void* done_event)
{
    if (!c) return SHADOW_EINVAL;
    if (c->poisoned) return SHADOW_EHIP;
    if (c->arrived_count != 0) return SHADOW_EBUSY;
    auto poison = [&](int32_t rc) { c->poisoned = true; return rc; };
    // everything of the completed iteration is ordered before state_ev ...
    int32_t rc = join_to_stream0(c);
    if (rc != SHADOW_OK) return poison(rc);
    HIP_TRY(hipEventRecord(c->state_ev, c->streams[0]));
    HIP_TRY(hipStreamWaitEvent(c->snap_stream, c->state_ev, 0));
    // ... the copies run on the copy stream, and only kernels that write the replica wait for them
    const size_t bytes = c->lay.arena_numel * sizeof(float);
    ProfScope ps(c, SHADOW_K_SNAPSHOT, c->snap_stream);
    if (ps.rc != SHADOW_OK) return ps.rc;
    int32_t rcopy = SHADOW_OK;
    if (dst_param) rcopy = snapshot_copy(c, dst_param, c->p, bytes);
    if (rcopy == SHADOW_OK && dst_m) rcopy = snapshot_copy(c, dst_m, c->m, bytes);
    if (rcopy == SHADOW_OK && dst_v && c->v) rcopy = snapshot_copy(c, dst_v, c->v, bytes);
    // whatever was enqueued, later writers of the replica must stay behind it
    const hipError_t e2 = hipEventRecord(c->snap_ev, c->snap_stream);
    std::fill(c->snap_wait.begin(), c->snap_wait.end(), uint8_t(1));
    if (rcopy != SHADOW_OK) return poison(rcopy);
    if (e2 != hipSuccess) {
        g_hip_error = std::string("hipEventRecord: ") + hipGetErrorString(e2);
        return poison(SHADOW_EHIP);
    }
    if (ps.end() != SHADOW_OK) return poison(SHADOW_EHIP);
    if (done_event) HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(done_event), c->snap_stream));
    c->have_snapshot = true;
    c->last_snap_ev = c->snap_ev;
    c->last_snap_step = c->completed;
    if (out_step) *out_step = c->completed;
    return SHADOW_OK;
}

int32_t shadow_snapshot_attach(shadow_ctx* c, float* d_stage_param, float* d_stage_m, float* d_stage_v)
{
    if (!c || !d_stage_param || !d_stage_m) return SHADOW_EINVAL;
    const bool sgd = c->hp.optimizer == SHADOW_OPT_SGD;
    if (sgd ? d_stage_v != nullptr : d_stage_v == nullptr) return SHADOW_EINVAL;
    if (!aligned(d_stage_param, 256) || !aligned(d_stage_m, 256) || !aligned(d_stage_v, 256)) return SHADOW_EINVAL;
    float* all[6] = {d_stage_param, d_stage_m, d_stage_v, c->p, c->m, c->v};
    for (int i = 0; i < 3; ++i)
        for (int j = i + 1; j < 6; ++j)
            if (all[i] && all[i] == all[j]) return SHADOW_EINVAL;
    if (c->stage_p) return SHADOW_EINVAL;              // at most once
    if (c->arrived_count != 0) return SHADOW_EBUSY;
    // the per-bucket kernels never touch the alignment gaps: zero them once so that the staging
    // set equals the replica everywhere
    for (const BucketL& b : c->lay.buckets) {
        const uint64_t end = b.arena_off + b.numel;
        const uint64_t padded = (end + kAlignElems - 1) / kAlignElems * kAlignElems;
        if (padded == end) continue;
        const size_t bytes = (padded - end) * sizeof(float);
        HIP_TRY(hipMemset(d_stage_param + end, 0, bytes));
        HIP_TRY(hipMemset(d_stage_m + end, 0, bytes));
        if (d_stage_v) HIP_TRY(hipMemset(d_stage_v + end, 0, bytes));
    }
    HIP_TRY(hipDeviceSynchronize());
    c->stage_p = d_stage_param;
    c->stage_m = d_stage_m;
    c->stage_v = d_stage_v;
    return SHADOW_OK;
}

int32_t shadow_snapshot_arm(shadow_ctx* c, float* h_dst_param, float* h_dst_m, float* h_dst_v)
{
    if (!c || !c->stage_p) return SHADOW_EINVAL;
    if (c->poisoned) return SHADOW_EHIP;
    if (c->arrived_count != 0 || c->armed) return SHADOW_EBUSY;
    if (c->drain_recorded) {
        const hipError_t q = hipEventQuery(c->drain_ev);
        if (q == hipErrorNotReady) return SHADOW_EBUSY;     // the staging set is still being drained
        if (q != hipSuccess) { g_hip_error = std::string("hipEventQuery: ") + hipGetErrorString(q); return SHADOW_EHIP; }
    }
    c->armed = true;
    c->armed_host[0] = h_dst_param;
    c->armed_host[1] = h_dst_m;
    c->armed_host[2] = h_dst_v;
    return SHADOW_OK;
}

int32_t shadow_snapshot_record(shadow_ctx* c, void* event)
{
    if (!c || !event) return SHADOW_EINVAL;
    if (c->poisoned) return SHADOW_EHIP;
    if (c->armed || c->snap_active) return SHADOW_EBUSY;    // the armed iteration has not completed yet
    if (!c->have_snapshot) return SHADOW_EINVAL;
    // both kinds of snapshot end on the copy stream, in request order
    HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(event), c->snap_stream));
    return SHADOW_OK;
}

int32_t shadow_snapshot_wait(shadow_ctx* c, uint64_t* out_step)
{
    if (!c) return SHADOW_EINVAL;
    if (c->armed || c->snap_active) return SHADOW_EBUSY;
    if (!c->have_snapshot) return SHADOW_EINVAL;
    HIP_TRY(hipEventSynchronize(c->last_snap_ev));
    if (out_step) *out_step = c->last_snap_step;
    return SHADOW_OK;
}

}  // extern "C"

// ---- one whole iteration without any allocation -----------------------------------------
// Device memory that the kernels need beyond the caller's arrays (the weight-decay tables, the
// norm partials, the clip coefficient) lies in one file-scope device array of fixed size.  Each
// GPU holds its own copy at its own address: the address is looked up once per device and only
// that pointer, never the array's name, is used in host code.
namespace {

constexpr uint64_t kStaticMaxArena = SHADOW_STATIC_MAX_ARENA_NUMEL;
constexpr uint32_t kStaticMaxBuckets = SHADOW_STATIC_MAX_BUCKETS;
constexpr uint32_t kStaticMaxRuns = 8192;
constexpr uint64_t kStaticMaxSlots = kStaticMaxArena / 256 + 17ull * kStaticMaxBuckets;   // a wave covers >= 256 elements
constexpr uint64_t kOffTileMode = 0;                                                       // 1 byte per 1024 elements
constexpr uint64_t kOffRunStart = kOffTileMode + (kStaticMaxArena >> kWdTileShift);
constexpr uint64_t kOffRunFlag = kOffRunStart + 8ull * kStaticMaxRuns;
constexpr uint64_t kOffPartial = kOffRunFlag + kStaticMaxRuns;
constexpr uint64_t kOffStage1 = kOffPartial + 8ull * kStaticMaxSlots;
constexpr uint64_t kOffCoef = kOffStage1 + (8ull * ((kStaticMaxSlots + kNormChunk - 1) / kNormChunk) + 255) / 256 * 256;
constexpr uint64_t kOffSumsq = kOffCoef + 256;
constexpr uint64_t kStaticScratchBytes = kOffSumsq + 256;
static_assert(kOffRunStart % 256 == 0 && kOffRunFlag % 256 == 0 && kOffPartial % 256 == 0 && kOffStage1 % 256 == 0 &&
              kOffCoef % 256 == 0 && kOffSumsq % 256 == 0, "sections of the static scratch are 256-byte aligned");
static_assert(kStaticScratchBytes < (6ull << 20), "the static scratch stays modest");

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

// Device address of this GPU's copy of the scratch array (looked up on the first call on that device).
int32_t static_scratch(unsigned char** out)
{
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return SHADOW_EINVAL;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        unsigned char* ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch)));
        if (!ptr) { g_hip_error = "hipGetSymbolAddress returned a null address"; return SHADOW_EHIP; }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SHADOW_OK;
}

}  // namespace

extern "C" {

int32_t shadow_apply_iteration_static(const shadow_layout* layout, const shadow_hparams* hp, float* d_param, float* d_m, float* d_v,
                                      float* d_reduced, const void* const* d_grad_views, uint64_t step, void* stream)
{
    const int32_t chk = check_replica_args(layout, hp, d_param, d_m, d_v, d_reduced);
    if (chk != SHADOW_OK) return chk;
    if (!d_grad_views || step == 0) return SHADOW_EINVAL;
    const uint32_t W = hp->num_workers;
    const size_t B = layout->buckets.size();
    for (size_t i = 0; i < B * W; ++i)
        if (!d_grad_views[i] || !aligned(d_grad_views[i], 16)) return SHADOW_EINVAL;
    if (layout->arena_numel > kStaticMaxArena || B > kStaticMaxBuckets) return SHADOW_ETOOBIG;

    // a context on the stack: host bookkeeping only, its device tables point into the static scratch
    shadow_ctx c;
    std::vector<uint64_t> run_start;
    std::vector<uint8_t> run_flag;
    std::vector<uint32_t> ids;
    try {
        c.lay = *layout;
        c.streams.assign(1, static_cast<hipStream_t>(stream));
        c.stream_dirty.assign(1, 0);
        c.snap_wait.assign(1, 0);
        make_runs(c.lay, run_start, run_flag);
        ids.resize(B);
    } catch (const std::bad_alloc&) {
        return SHADOW_ENOMEM;
    }
    c.hp = *hp;
    c.p = d_param; c.m = d_m; c.v = d_v; c.r = d_reduced;
    c.clip = hp->max_grad_norm > 0.f;
    c.refold = c.clip && !d_reduced;
    set_launch_shape(&c, hp->launch);
    if (run_start.size() > kStaticMaxRuns) return SHADOW_ETOOBIG;
    if (c.clip) {
        try {
            if (!assign_slots(&c)) return SHADOW_ETOOBIG;
        } catch (const std::bad_alloc&) {
            return SHADOW_ENOMEM;
        }
        if (c.nslots > kStaticMaxSlots) return SHADOW_ETOOBIG;
    }
    unsigned char* base = nullptr;
    const int32_t rs = static_scratch(&base);
    if (rs != SHADOW_OK) return rs;
    c.d_tile_mode = base + kOffTileMode;
    c.d_run_start = reinterpret_cast<uint64_t*>(base + kOffRunStart);
    c.d_run_flag = base + kOffRunFlag;
    c.num_runs = uint32_t(run_start.size());
    c.d_partial = reinterpret_cast<double*>(base + kOffPartial);
    c.d_stage1 = reinterpret_cast<double*>(base + kOffStage1);
    c.d_coef = reinterpret_cast<float*>(base + kOffCoef);
    c.d_sumsq = reinterpret_cast<double*>(base + kOffSumsq);
    compute_scalars(c.hp, step, c.sc);

    // The scratch keeps the previous call's contents.  Nothing in it has to start at zero: the run table and the
    // tile modes are rewritten below for this layout, every wave of the folds writes its own partial slot, the norm
    // kernels write every stage-1 entry they later read, and the coefficient is written before the update reads it.
    hipStream_t st = c.streams[0];
    for (uint32_t first = 0; first < c.num_runs; first += kRunChunk) {
        RunChunk ch{};
        ch.first = first;
        ch.count = c.num_runs - first < uint32_t(kRunChunk) ? c.num_runs - first : uint32_t(kRunChunk);
        for (uint32_t i = 0; i < ch.count; ++i) { ch.start[i] = run_start[first + i]; ch.flag[i] = run_flag[first + i]; }
        k_put_runs<<<1, kRunChunk, 0, st>>>(ch, c.d_run_start, c.d_run_flag);
    }
    const uint64_t ntiles = (c.lay.arena_numel + (1ull << kWdTileShift) - 1) >> kWdTileShift;
    k_build_tile_mode<<<uint32_t((ntiles + 255) / 256), 256, 0, st>>>(c.d_run_start, c.d_run_flag, c.num_runs, c.lay.arena_numel,
                                                                      c.d_tile_mode, ntiles);
    HIP_TRY(hipGetLastError());
    for (size_t i = 0; i < B; ++i) ids[i] = uint32_t(i);
    auto views_of = [&](size_t i) { return d_grad_views + i * W; };
    int32_t rc = launch_buckets(&c, ids.data(), B, views_of, 0, /*update=*/!c.clip);
    if (rc != SHADOW_OK) return rc;
    if (c.clip) {
        if (c.refold) {
            try {
                c.step_views.assign(d_grad_views, d_grad_views + B * W);
            } catch (const std::bad_alloc&) {
                return SHADOW_ENOMEM;       // the folds already ran; the replica itself is still untouched
            }
        }
        rc = enqueue_norm_and_update_on_one_stream(&c);
        if (rc != SHADOW_OK) return rc;
    }
    return SHADOW_OK;
}

int32_t shadow_sync(shadow_ctx* c)
{
    if (!c) return SHADOW_EINVAL;
    if (!c->poisoned) {
        const int32_t rc = flush_all(c);
        if (rc != SHADOW_OK) return rc;
    }
    for (hipStream_t s : c->streams) HIP_TRY(hipStreamSynchronize(s));
    HIP_TRY(hipStreamSynchronize(c->snap_stream));
    if (c->copy_stream) HIP_TRY(hipStreamSynchronize(c->copy_stream));
    return SHADOW_OK;
}

int32_t shadow_destroy(shadow_ctx* c)
{
    if (!c) return SHADOW_OK;
    if (!c->poisoned) (void)flush_all(c);     // buffered buckets were accepted: their work is owed
    for (hipStream_t s : c->streams) (void)hipStreamSynchronize(s);
    if (c->snap_stream) (void)hipStreamSynchronize(c->snap_stream);
    if (c->copy_stream) (void)hipStreamSynchronize(c->copy_stream);
    free_ctx(c);
    return SHADOW_OK;
}

int32_t shadow_step(const shadow_ctx* c, uint64_t* completed_step, uint32_t* buckets_pending)
{
    if (!c) return SHADOW_EINVAL;
    if (completed_step) *completed_step = c->completed;
    if (buckets_pending) *buckets_pending = c->arrived_count ? uint32_t(c->lay.buckets.size()) - c->arrived_count : 0;
    return SHADOW_OK;
}

int32_t shadow_bucket_stream(const shadow_ctx* c, uint32_t bucket_id, void** out_stream)
{
    if (!c || !out_stream) return SHADOW_EINVAL;
    if (bucket_id >= c->lay.buckets.size()) return SHADOW_EBUCKET;
    *out_stream = c->streams[bucket_id % c->streams.size()];
    return SHADOW_OK;
}

int32_t shadow_clip_state(shadow_ctx* c, float* out_coef, double* out_sumsq)
{
    if (!c || !c->clip) return SHADOW_EINVAL;
    int32_t rc = shadow_sync(c);
    if (rc != SHADOW_OK) return rc;
    if (out_coef) HIP_TRY(hipMemcpy(out_coef, c->d_coef, sizeof(float), hipMemcpyDeviceToHost));
    if (out_sumsq) HIP_TRY(hipMemcpy(out_sumsq, c->d_sumsq, sizeof(double), hipMemcpyDeviceToHost));
    return SHADOW_OK;
}

int32_t shadow_set_lr(shadow_ctx* c, float lr)
{
    if (!c || !(lr >= 0.f)) return SHADOW_EINVAL;
    if (c->arrived_count != 0) return SHADOW_EBUSY;
    c->hp.lr = lr;
    c->sc_step = 0;
    return SHADOW_OK;
}

int32_t shadow_profile_enable(shadow_ctx* c, int32_t on)
{
    if (!c) return SHADOW_EINVAL;
    c->profile = on != 0;
    return SHADOW_OK;
}

int32_t shadow_profile_kinds(shadow_ctx* c, uint32_t kind_mask)
{
    if (!c || (kind_mask >> SHADOW_K_COUNT) != 0) return SHADOW_EINVAL;
    c->profile_kinds = kind_mask;
    return SHADOW_OK;
}

int32_t shadow_profile_read(shadow_ctx* c, uint32_t kind, uint64_t* launches, double* total_ms)
{
    if (!c || kind >= SHADOW_K_COUNT) return SHADOW_EINVAL;
    int32_t rc = shadow_sync(c);
    if (rc != SHADOW_OK) return rc;
    double total = 0.0;
    uint64_t n = 0;
    for (auto& sp : c->spans[kind]) {
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, sp.a, sp.b));
        total += ms;
        ++n;
        c->ev_pool.push_back(sp.a);
        c->ev_pool.push_back(sp.b);
    }
    c->spans[kind].clear();
    if (launches) *launches = n;
    if (total_ms) *total_ms = total;
    return SHADOW_OK;
}

int32_t shadow_copy_probe(void* d_dst, const void* d_src, uint64_t bytes, void* stream, uint64_t max_launch_threads)
{
    if (!d_dst || !d_src || (bytes & 15) || !aligned(d_dst, 16) || !aligned(d_src, 16)) return SHADOW_EINVAL;
    if (max_launch_threads > kMaxThreadsPerLaunch) return SHADOW_EINVAL;
    if (bytes == 0) return SHADOW_OK;
    return launch_copy(d_dst, d_src, bytes, static_cast<hipStream_t>(stream), max_launch_threads ? max_launch_threads : kMaxThreadsPerLaunch);
}

}  // extern "C"

namespace {

template <int R, int D>
void launch_streams(const ProbeSet& ps, u32x4* sink, uint64_t n16, uint32_t block, uint32_t lds, hipStream_t st)
{
    const uint64_t per_launch = kMaxThreadsPerLaunch / block;
    const uint64_t blocks = (n16 + block - 1) / block;
    for (uint64_t b0 = 0; b0 < blocks; b0 += per_launch) {
        const uint64_t nb = blocks - b0 < per_launch ? blocks - b0 : per_launch;
        k_streams<R, D><<<uint32_t(nb), block, lds, st>>>(ps, sink, n16, b0);
    }
}

template <int R>
bool dispatch_streams_dst(uint32_t d, const ProbeSet& ps, u32x4* sink, uint64_t n16, uint32_t block, uint32_t lds, hipStream_t st)
{
    switch (d) {
        case 0: launch_streams<R, 0>(ps, sink, n16, block, lds, st); return true;
        case 1: launch_streams<R, 1>(ps, sink, n16, block, lds, st); return true;
        case 3: launch_streams<R, 3>(ps, sink, n16, block, lds, st); return true;
        default: return false;
    }
}

}  // namespace

extern "C" {

int32_t shadow_stream_probe(void* const* d_dst, uint32_t n_dst, const void* const* d_src, uint32_t n_src, void* d_sink, uint64_t bytes,
                            void* stream, uint32_t block, uint32_t waves_per_cu)
{
    if (n_src > uint32_t(kProbeMaxSrc) || n_dst > uint32_t(kProbeMaxDst) || (n_src == 0 && n_dst == 0) || (bytes & 15)) return SHADOW_EINVAL;
    if ((n_src && !d_src) || (n_dst && !d_dst) || (n_dst == 0 && (!d_sink || !aligned(d_sink, 16)))) return SHADOW_EINVAL;
    if (block == 0) block = 256;
    if (!valid_block(block) || waves_per_cu > 32) return SHADOW_EINVAL;
    ProbeSet ps{};
    for (uint32_t k = 0; k < n_src; ++k) {
        if (!d_src[k] || !aligned(d_src[k], 16)) return SHADOW_EINVAL;
        ps.src[k] = static_cast<const u32x4*>(d_src[k]);
    }
    for (uint32_t k = 0; k < n_dst; ++k) {
        if (!d_dst[k] || !aligned(d_dst[k], 16)) return SHADOW_EINVAL;
        ps.dst[k] = static_cast<u32x4*>(d_dst[k]);
    }
    if (bytes == 0) return SHADOW_OK;
    const uint64_t n16 = bytes >> 4;
    const uint32_t lds = lds_for_wave_cap(block, waves_per_cu ? waves_per_cu : 32);
    hipStream_t st = static_cast<hipStream_t>(stream);
    u32x4* sink = static_cast<u32x4*>(d_sink);
    bool known = false;
    switch (n_src) {
        case 0: known = dispatch_streams_dst<0>(n_dst, ps, sink, n16, block, lds, st); break;
        case 1: known = dispatch_streams_dst<1>(n_dst, ps, sink, n16, block, lds, st); break;
        case 2: known = dispatch_streams_dst<2>(n_dst, ps, sink, n16, block, lds, st); break;
        case 4: known = dispatch_streams_dst<4>(n_dst, ps, sink, n16, block, lds, st); break;
        case 7: known = dispatch_streams_dst<7>(n_dst, ps, sink, n16, block, lds, st); break;
        case 8: known = dispatch_streams_dst<8>(n_dst, ps, sink, n16, block, lds, st); break;
        case 16: known = dispatch_streams_dst<16>(n_dst, ps, sink, n16, block, lds, st); break;
        default: break;
    }
    if (!known) return SHADOW_EINVAL;          // a mix the kernel is not instantiated for
    HIP_TRY(hipGetLastError());
    return SHADOW_OK;
}

const char* shadow_strerror(int32_t status)
{
    switch (status) {
        case SHADOW_OK: return "ok";
        case SHADOW_EINVAL: return "invalid argument";
        case SHADOW_EBUCKET: return "bucket id out of range";
        case SHADOW_EDUP: return "bucket already applied in this iteration";
        case SHADOW_ESTEP: return "step is not the last completed step + 1";
        case SHADOW_EBUSY: return "an iteration is partly applied";
        case SHADOW_EHIP: return "HIP runtime failure";
        case SHADOW_ENOMEM: return "out of memory";
        case SHADOW_ETOOBIG: return "input exceeds the fixed capacity of the library's static scratch";
        default: return "unknown status";
    }
}

const char* shadow_last_hip_error(void) { return g_hip_error.c_str(); }

const char* shadow_build_id(void) { return SHADOW_BUILD_ID; }

}  // extern "C"
