// Device kernels of the shadow update for gfx950 (wave64, HBM-bound streaming).
//
// What is computed (Checkmate, arxiv 2507.13522: section 4 overview step 4 and
// section 4.2.3 -- the shadow runs the trainers' optimizer step on the
// gradients of the iteration; section 2.1 -- gradients of the data-parallel
// workers are reduced by summing or averaging; section 4.2.4 -- the optimizer
// is functional, every element independent):
//
//   fold     r[i] = g_0[i] + g_1[i] + ... + g_{W-1}[i]   (float, left to right;
//            bfloat16 inputs are widened exactly first), then r[i] *= float(1/W)
//            for a mean.
//   clip     S = sum_i r[i]^2 over the whole model (double), c = min(1,
//            max_norm / (sqrt(S) + 1e-6)) rounded to float, g = r*c.
//   AdamW    p *= (1 - lr*wd) on tensors with the flag;
//            m = b1*m + (1-b1)*g;  v = b2*v + ((1-b2)*g)*g;
//            p -= step_size * (m / (sqrt(v)*isq + eps)),
//            step_size = lr/(1-b1^t), isq = 1/sqrt(1-b2^t).
//   Adam     as AdamW without the decay multiply, the L2 penalty joining the
//            gradient first: g = g + wd*p on tensors with the flag.
//   SGD      g = g + wd*p;  b = mu*b + g;  p -= lr*b   (b kept where Adam keeps m).
//
// Every float operation above is a separate IEEE-754 operation (the file is
// compiled with -ffp-contract=off and correctly rounded divide/sqrt, denormals
// kept), so results do not depend on launch shape, bucket order or stream.
//
// Memory plan (from measurement on MI355X): one lane owns 4 consecutive
// elements and makes exactly one trip: one 64-bit load per bfloat16 view (one
// 128-bit load per float view) and one 128-bit load and store for each of p, m,
// v.  Grids are flat (one block per 4*blockDim elements, no grid-stride loop)
// so the hardware keeps refilling CUs with fresh waves whose loads are all
// issued before the first use; every global access carries the non-temporal
// hint, since no line is touched twice within a kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace shadow {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kVec = 4;              // elements per lane
constexpr int kMaxBlock = 1024;
constexpr int kMaxWorkers = 64;
constexpr int kWdTileShift = 10;     // weight-decay map granularity: 1024 elements

// One launch folds a batch of buckets.  The descriptor travels in the kernel
// arguments (no device table to keep coherent with the host): bucket k of the
// batch owns blocks [first_block[k], first_block[k+1]) and its W view pointers
// are ptr[k*w .. k*w+w).
constexpr int kMaxBatch = 32;
constexpr int kMaxBatchPtrs = 320;
struct FoldBatch {
    uint32_t count;
    uint32_t w;
    uint32_t first_block[kMaxBatch + 1];
    uint32_t slot_base[kMaxBatch];      // first norm-partial slot of the bucket (clipping on)
    uint64_t numel[kMaxBatch];
    uint64_t arena_off[kMaxBatch];      // arena index of the bucket's first element
    const void* ptr[kMaxBatchPtrs];
};

// Unused first_block entries hold 0x7FFFFFFF (block indices stay below 2^31), so the bucket
// of a block is the number of entries 1..kMaxBatch-1 that are <= the block index, read off
// the sign bits of (block - entry): two wide scalar loads and a chain of scalar ALU ops, no
// dependent memory round trips before the wave can issue its loads.
constexpr uint32_t kNoBucket = 0x7FFFFFFFu;
__device__ __forceinline__ uint32_t bucket_of_block(const FoldBatch& fb, uint32_t block)
{
    uint32_t above = 0;
#pragma unroll
    for (int j = 1; j < kMaxBatch; ++j) above += (block - fb.first_block[j]) >> 31;
    return uint32_t(kMaxBatch - 1) - above;
}

// Per-iteration scalars, prepared on the host in double and rounded once to float.
struct StepScalars {
    float beta1, beta2, omb1, omb2, decay, step_size, isq, eps, inv_w;
    uint32_t mean;
    float lr, wd;      // as given (SGD step, L2 penalty of Adam and SGD)
};

// Optimizers (section 4.2.4: SGD, Adam and AdamW are functional).
enum : int { kAdamW = 0, kAdam = 1, kSgd = 2 };

// Weight-decay flag of every arena element: a byte per 1024-element tile
// (0 = no decay, 1 = decay, 2 = the tile holds the start of a run, look the
// element up) plus the sorted run table for those rare tiles.  A run is a
// stretch of elements with one flag: 0 = no decay, 1 = decay, 2 = alignment gap
// between two buckets (no parameter lives there; a sweep over the whole arena
// leaves it untouched, so it stays zero even when the clip coefficient is NaN).
constexpr uint8_t kTileMixed = 2;
constexpr uint8_t kRunGap = 2;
struct WdMap {
    const uint8_t* tile_mode;
    const uint64_t* run_start;   // run k covers [run_start[k], run_start[k+1])
    const uint8_t* run_flag;
    uint32_t num_runs;
};

template <typename T>
__device__ __forceinline__ T load_once(const T* p) { return __builtin_nontemporal_load(p); }
template <typename T>
__device__ __forceinline__ void store_once(T* p, T v) { __builtin_nontemporal_store(v, p); }

__device__ __forceinline__ float bits_to_float(uint32_t b) { return __builtin_bit_cast(float, b); }

// One element.  flag: the tensor takes weight decay.  AdamW multiplies a masked element by
// 1.0f (which returns it unchanged) instead of branching; the L2 penalty of Adam and SGD is
// selected, not multiplied by zero, because g + 0*p is not always g (signed zeros, infinities).
template <int OPT>
__device__ __forceinline__ void opt_elem(float& p, float& m, float& v, float g, bool flag, const StepScalars& s)
{
    if constexpr (OPT == kAdamW) {
        p = p * (flag ? s.decay : 1.0f);
    } else {
        const float pen = g + s.wd * p;
        g = flag ? pen : g;
    }
    if constexpr (OPT == kSgd) {
        m = s.beta1 * m + g;
        p = p - s.lr * m;
    } else {
        m = s.beta1 * m + s.omb1 * g;
        v = s.beta2 * v + (s.omb2 * g) * g;
        float denom = sqrtf(v) * s.isq + s.eps;
        p = p - s.step_size * (m / denom);
    }
}

__device__ __forceinline__ uint8_t run_flag_of(const WdMap& map, uint64_t e)
{
    uint32_t lo = 0, hi = map.num_runs;     // largest k with run_start[k] <= e
    while (hi - lo > 1) {
        uint32_t mid = (lo + hi) >> 1;
        if (map.run_start[mid] <= e) lo = mid; else hi = mid;
    }
    return map.run_flag[lo];
}

__device__ __forceinline__ bool decay_flag_of(const WdMap& map, uint64_t e) { return run_flag_of(map, e) == 1; }

// ---- fold of 4 consecutive elements ---------------------------------------------------
// W > 0: compile-time worker count, all loads of a batch issued before the adds (which stay
// strictly in worker order); W == 0: run-time worker count.
__device__ __forceinline__ void widen_first(const u32x2& a, f32x4& r)
{
    r[0] = bits_to_float(a[0] << 16);              // even element: low half-word
    r[1] = bits_to_float(a[0] & 0xFFFF0000u);
    r[2] = bits_to_float(a[1] << 16);
    r[3] = bits_to_float(a[1] & 0xFFFF0000u);
}

__device__ __forceinline__ void widen_add(const u32x2& a, f32x4& r)
{
    r[0] = r[0] + bits_to_float(a[0] << 16);
    r[1] = r[1] + bits_to_float(a[0] & 0xFFFF0000u);
    r[2] = r[2] + bits_to_float(a[1] << 16);
    r[3] = r[3] + bits_to_float(a[1] & 0xFFFF0000u);
}

// The W views' vectors of one group of 4 elements, as loaded: loading and reducing are
// separate so that a lane that owns several groups has all its loads in flight at once.
template <bool BF16>
struct RawVec { typedef f32x4 type; };
template <>
struct RawVec<true> { typedef u32x2 type; };

template <bool BF16, int W>
__device__ __forceinline__ void load_views4(const void* const* vp, uint64_t vec, typename RawVec<BF16>::type (&raw)[W])
{
    typedef typename RawVec<BF16>::type V;
#pragma unroll
    for (int w = 0; w < W; ++w) raw[w] = load_once(reinterpret_cast<const V*>(vp[w]) + vec);
}

template <bool BF16, int W>
__device__ __forceinline__ f32x4 reduce_views4(const typename RawVec<BF16>::type (&raw)[W], const StepScalars& s)
{
    f32x4 r;
    if constexpr (BF16) {
        widen_first(raw[0], r);
#pragma unroll
        for (int w = 1; w < W; ++w) widen_add(raw[w], r);
    } else {
        r = raw[0];
#pragma unroll
        for (int w = 1; w < W; ++w) r = r + raw[w];
    }
    if (s.mean) r = r * s.inv_w;
    return r;
}

// Worker count known only at run time: the views are taken in chunks of kLoopChunk, every load of a chunk issued
// before its adds, the adds still strictly in worker order.
constexpr int kLoopChunk = 8;
template <bool BF16>
__device__ __forceinline__ void accumulate_view(const typename RawVec<BF16>::type& a, bool first, f32x4& r)
{
    if constexpr (BF16) {
        if (first) widen_first(a, r); else widen_add(a, r);
    } else {
        if (first) r = a; else r = r + a;
    }
}

template <bool BF16>
__device__ __forceinline__ f32x4 fold4_loop(const void* const* vp, uint32_t w_rt, uint64_t vec)
{
    typedef typename RawVec<BF16>::type V;
    f32x4 r = f32x4{0.f, 0.f, 0.f, 0.f};
    uint32_t w0 = 0;
    for (; w0 + kLoopChunk <= w_rt; w0 += kLoopChunk) {
        V raw[kLoopChunk];
#pragma unroll
        for (int j = 0; j < kLoopChunk; ++j) raw[j] = load_once(reinterpret_cast<const V*>(vp[w0 + j]) + vec);
#pragma unroll
        for (int j = 0; j < kLoopChunk; ++j) accumulate_view<BF16>(raw[j], j == 0 && w0 == 0, r);
    }
    if (w0 < w_rt) {
        V raw[kLoopChunk];
#pragma unroll
        for (int j = 0; j < kLoopChunk - 1; ++j)
            if (w0 + j < w_rt) raw[j] = load_once(reinterpret_cast<const V*>(vp[w0 + j]) + vec);
#pragma unroll
        for (int j = 0; j < kLoopChunk - 1; ++j)
            if (w0 + j < w_rt) accumulate_view<BF16>(raw[j], j == 0 && w0 == 0, r);
    }
    return r;
}

template <bool BF16, int W>
__device__ __forceinline__ f32x4 fold4(const void* const* vp, uint32_t w_rt, uint64_t vec, const StepScalars& s)
{
    f32x4 r;
    if constexpr (BF16) {
        if constexpr (W > 0) {
            u32x2 raw[W];
            load_views4<true, W>(vp, vec, raw);
            return reduce_views4<true, W>(raw, s);
        } else {
            r = fold4_loop<true>(vp, w_rt, vec);
        }
    } else {
        if constexpr (W > 0) {
            constexpr int kBatch = 16;
#pragma unroll
            for (int w0 = 0; w0 < W; w0 += kBatch) {
                f32x4 raw[kBatch];
#pragma unroll
                for (int j = 0; j < kBatch; ++j)
                    if (w0 + j < W) raw[j] = load_once(reinterpret_cast<const f32x4*>(vp[w0 + j]) + vec);
#pragma unroll
                for (int j = 0; j < kBatch; ++j) {
                    if (w0 + j < W) {
                        if (w0 + j == 0) r = raw[j]; else r = r + raw[j];
                    }
                }
            }
        } else {
            r = fold4_loop<false>(vp, w_rt, vec);
        }
    }
    if (s.mean) r = r * s.inv_w;
    return r;
}

// one element (ragged tail of a bucket)
template <bool BF16>
__device__ __forceinline__ float fold1(const void* const* vp, uint32_t w_rt, uint64_t e, const StepScalars& s)
{
    float acc;
    if constexpr (BF16) {
        acc = bits_to_float(uint32_t(reinterpret_cast<const uint16_t*>(vp[0])[e]) << 16);
        for (uint32_t w = 1; w < w_rt; ++w)
            acc = acc + bits_to_float(uint32_t(reinterpret_cast<const uint16_t*>(vp[w])[e]) << 16);
    } else {
        acc = reinterpret_cast<const float*>(vp[0])[e];
        for (uint32_t w = 1; w < w_rt; ++w) acc = acc + reinterpret_cast<const float*>(vp[w])[e];
    }
    if (s.mean) acc = acc * s.inv_w;
    return acc;
}

// State of 4 consecutive arena elements (vector index vec, first element e0 = 4 * vec) and the
// decay mode of their tile.  Loading, stepping and storing are separate calls so that a kernel
// can issue every load of a lane, state and gradient views alike, before the first use.
// SGD has no second moment: v is never touched (it may be null).
struct State4 {
    f32x4 p, m, v;
    uint8_t mode;
};

template <int OPT>
__device__ __forceinline__ State4 load_state4(const float* p, const float* m, const float* v, uint64_t vec, uint64_t e0,
                                              const WdMap& map)
{
    State4 st;
    st.p = load_once(reinterpret_cast<const f32x4*>(p) + vec);
    st.m = load_once(reinterpret_cast<const f32x4*>(m) + vec);
    st.v = f32x4{0.f, 0.f, 0.f, 0.f};
    if constexpr (OPT != kSgd) st.v = load_once(reinterpret_cast<const f32x4*>(v) + vec);
    st.mode = map.tile_mode[e0 >> kWdTileShift];
    return st;
}

template <int OPT>
__device__ __forceinline__ void step_state4(State4& st, uint64_t e0, const f32x4& g, const WdMap& map, const StepScalars& s)
{
#pragma unroll
    for (int k = 0; k < kVec; ++k) {
        const uint8_t f = (st.mode != kTileMixed) ? st.mode : run_flag_of(map, e0 + k);
        if (f == kRunGap) continue;
        float pk = st.p[k], mk = st.m[k], vk = st.v[k];
        opt_elem<OPT>(pk, mk, vk, g[k], f != 0, s);
        st.p[k] = pk; st.m[k] = mk; st.v[k] = vk;
    }
}

template <int OPT>
__device__ __forceinline__ void store_state4(const State4& st, float* p, float* m, float* v, uint64_t vec)
{
    store_once(reinterpret_cast<f32x4*>(p) + vec, st.p);
    store_once(reinterpret_cast<f32x4*>(m) + vec, st.m);
    if constexpr (OPT != kSgd) store_once(reinterpret_cast<f32x4*>(v) + vec, st.v);
}

// A second set of arenas that receives every new value as well while a snapshot is armed
// (section 4: the checkpoint is kept at per-iteration granularity; this is how a consistent
// copy of one iteration's state is taken without a separate pass over the replica).
// p == nullptr: no snapshot armed (uniform over the launch).
struct SnapSet {
    float* p;
    float* m;
    float* v;
};

// ---- kernel: fold + AdamW in one pass (clipping off) ---------------------------------
// p, m, v are the arenas.  Within its bucket, thread i < n/4 owns elements 4i..4i+3 and
// thread n/4 owns the (n mod 4) tail elements.
// coef == nullptr: clipping off.  Otherwise the reduced gradient is multiplied by *coef first
// (second fold of an iteration whose reduced gradient was not stored).
template <bool BF16, int W, int OPT>
__global__ __launch_bounds__(kMaxBlock) void k_fold_adamw(FoldBatch fb, float* __restrict__ p, float* __restrict__ m,
                                                          float* __restrict__ v, const float* __restrict__ coef, WdMap map,
                                                          StepScalars s, SnapSet snap)
{
    const uint32_t k = bucket_of_block(fb, blockIdx.x);
    const void* const* vp = fb.ptr + k * fb.w;
    const uint64_t n = fb.numel[k], off = fb.arena_off[k];
    const uint64_t nvec = n >> 2;
    const uint64_t vec = uint64_t(blockIdx.x - fb.first_block[k]) * blockDim.x + threadIdx.x;
    if (vec < nvec) {
        float* pb = p + off;
        float* mb = m + off;
        float* vb = OPT == kSgd ? nullptr : v + off;
        const uint64_t e0 = off + (vec << 2);
        State4 st = load_state4<OPT>(pb, mb, vb, vec, e0, map);   // in flight together with the views
        f32x4 r = fold4<BF16, W>(vp, fb.w, vec, s);
        if (coef) r = r * (*coef);
        step_state4<OPT>(st, e0, r, map, s);
        store_state4<OPT>(st, pb, mb, vb, vec);
        if (snap.p) store_state4<OPT>(st, snap.p + off, snap.m + off, OPT == kSgd ? nullptr : snap.v + off, vec);
    } else if (vec == nvec) {
        for (uint64_t e = nvec << 2; e < n; ++e) {
            float g = fold1<BF16>(vp, fb.w, e, s);
            if (coef) g = g * (*coef);
            float pp = p[off + e], mm = m[off + e], vv = 0.f;
            if constexpr (OPT != kSgd) vv = v[off + e];
            opt_elem<OPT>(pp, mm, vv, g, decay_flag_of(map, off + e), s);
            p[off + e] = pp; m[off + e] = mm;
            if constexpr (OPT != kSgd) v[off + e] = vv;
            if (snap.p) {
                snap.p[off + e] = pp; snap.m[off + e] = mm;
                if constexpr (OPT != kSgd) snap.v[off + e] = vv;
            }
        }
    }
}

// ---- kernel: fold + sum of squares, reduced gradient stored (clipping on) -------------
// With few or narrow views a lane that owns only 4 elements moves too few bytes per wave
// launched (W = 1 bf16: 8 bytes), so the lane owns kVpl groups of 4 elements, blockDim apart
// (every load instruction of a wave still covers one contiguous run), chosen so that a lane
// reads at least 64 bytes.
constexpr int kFoldLaneBytes = 64;
template <bool BF16, int W>
constexpr int fold_vpl()
{
    if (W <= 0) return 1;
    const int bytes = 4 * (BF16 ? 2 : 4) * (W > 0 ? W : 1);
    const int v = kFoldLaneBytes / bytes;
    return v < 1 ? 1 : (v > 8 ? 8 : v);
}

// Sum of the squares of 4 reduced gradients, added to acc in element order.
__device__ __forceinline__ void add_squares(const f32x4& g, double& acc)
{
#pragma unroll
    for (int q = 0; q < kVec; ++q) {
        const double d = double(g[q]);
        acc = fma(d, d, acc);        // d*d is exact in double, so this equals acc + d*d
    }
}

// 8 consecutive bf16 elements per view behind one 128-bit load each; adds in worker order.
template <int W>
__device__ __forceinline__ void load_views8_bf16(const void* const* vp, uint64_t vec8, u32x4 (&raw)[W])
{
#pragma unroll
    for (int w = 0; w < W; ++w) raw[w] = load_once(reinterpret_cast<const u32x4*>(vp[w]) + vec8);
}

template <int W>
__device__ __forceinline__ void reduce_views8_bf16(const u32x4 (&raw)[W], const StepScalars& s, f32x4& lo, f32x4& hi)
{
    widen_first(u32x2{raw[0][0], raw[0][1]}, lo);
    widen_first(u32x2{raw[0][2], raw[0][3]}, hi);
#pragma unroll
    for (int w = 1; w < W; ++w) {
        widen_add(u32x2{raw[w][0], raw[w][1]}, lo);
        widen_add(u32x2{raw[w][2], raw[w][3]}, hi);
    }
    if (s.mean) { lo = lo * s.inv_w; hi = hi * s.inv_w; }
}

// r == nullptr: the reduced gradient is not stored (it will be folded again for the update).
// Every wave writes the sum of its lanes' squares to its own slot, partial[slot_base of the
// bucket + wave index within the bucket]: no barrier, fixed order.
template <bool BF16, int W>
__global__ __launch_bounds__(kMaxBlock) void k_fold_sumsq(FoldBatch fb, float* __restrict__ r, double* __restrict__ partial,
                                                          StepScalars s)
{
    constexpr int kVpl = fold_vpl<BF16, W>();
    const uint32_t k = bucket_of_block(fb, blockIdx.x);
    const void* const* vp = fb.ptr + k * fb.w;
    const uint64_t n = fb.numel[k];
    float* r_out = r ? r + fb.arena_off[k] : nullptr;
    const uint64_t nvec = n >> 2;
    const uint32_t local_block = blockIdx.x - fb.first_block[k];
    const uint64_t slot = fb.slot_base[k] + uint64_t(local_block) * (blockDim.x >> 6) + (threadIdx.x >> 6);
    // Few bf16 views and nothing to store (a pure read pass): the lane's groups of 4 elements
    // are taken in pairs, as 8 consecutive elements behind one 128-bit load per view; the
    // block covers the same elements, so grid and slots are those of the general path.
    if constexpr (BF16 && W > 0 && kVpl % 2 == 0) {
        if (!r_out) {
            constexpr int kVpl8 = kVpl / 2;
            const uint64_t nvec8 = n >> 3;
            const uint64_t base8 = uint64_t(local_block) * blockDim.x * kVpl8 + threadIdx.x;
            u32x4 raw[kVpl8][W];
#pragma unroll
            for (int j = 0; j < kVpl8; ++j) {
                const uint64_t vec8 = base8 + uint64_t(j) * blockDim.x;
                if (vec8 < nvec8) load_views8_bf16<W>(vp, vec8, raw[j]);
            }
            double acc = 0.0;
#pragma unroll
            for (int j = 0; j < kVpl8; ++j) {
                const uint64_t vec8 = base8 + uint64_t(j) * blockDim.x;
                if (vec8 < nvec8) {
                    f32x4 lo, hi;
                    reduce_views8_bf16<W>(raw[j], s, lo, hi);
                    add_squares(lo, acc);
                    add_squares(hi, acc);
                } else if (vec8 == nvec8) {
                    for (uint64_t e = nvec8 << 3; e < n; ++e) {
                        const double d = double(fold1<BF16>(vp, fb.w, e, s));
                        acc = fma(d, d, acc);
                    }
                }
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) acc += __shfl_down(acc, o, 64);
            if ((threadIdx.x & 63) == 0) partial[slot] = acc;
            return;
        }
    }
    const uint64_t base = uint64_t(local_block) * blockDim.x * kVpl + threadIdx.x;
    // several groups per lane: every group's loads are issued before the first one is reduced
    constexpr bool kSplit = kVpl > 1;
    typename RawVec<BF16>::type raw[kSplit ? kVpl : 1][kSplit ? W : 1];
    if constexpr (kSplit) {
#pragma unroll
        for (int j = 0; j < kVpl; ++j) {
            const uint64_t vec = base + uint64_t(j) * blockDim.x;
            if (vec < nvec) load_views4<BF16, W>(vp, vec, raw[j]);
        }
    }
    double acc = 0.0;
#pragma unroll
    for (int j = 0; j < kVpl; ++j) {
        const uint64_t vec = base + uint64_t(j) * blockDim.x;
        if (vec < nvec) {
            f32x4 rr;
            if constexpr (kSplit) rr = reduce_views4<BF16, W>(raw[j], s);
            else rr = fold4<BF16, W>(vp, fb.w, vec, s);
            if (r_out) store_once(reinterpret_cast<f32x4*>(r_out) + vec, rr);
            add_squares(rr, acc);
        } else if (vec == nvec) {
            for (uint64_t e = nvec << 2; e < n; ++e) {
                const float g = fold1<BF16>(vp, fb.w, e, s);
                if (r_out) r_out[e] = g;
                const double d = double(g);
                acc = fma(d, d, acc);
            }
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_down(acc, o, 64);
    if ((threadIdx.x & 63) == 0) partial[slot] = acc;
}

// ---- block-wide sum of doubles in a fixed order ----------------------------------------
__device__ __forceinline__ double block_sum(double x, double* lds)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_down(x, off, 64);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (lane == 0) lds[wave] = x;
    __syncthreads();
    double t = 0.0;
    if (threadIdx.x == 0) {
        const int nw = blockDim.x >> 6;
        for (int w = 0; w < nw; ++w) t += lds[w];
    }
    return t;   // valid in thread 0
}

// ---- kernels: norm and clip coefficient, two stages with fixed summation order ---------
// stage 1: block b sums slots [b*chunk, (b+1)*chunk), lane t taking every blockDim-th slot
constexpr int kNormBlock = 1024;
constexpr uint32_t kNormChunk = kNormBlock * 4;
__global__ __launch_bounds__(kNormBlock) void k_norm_stage1(const double* __restrict__ partial, uint32_t nslots,
                                                            double* __restrict__ stage1)
{
    __shared__ double lds[kNormBlock / 64];
    const uint64_t lo = uint64_t(blockIdx.x) * kNormChunk;
    const uint64_t hi = (lo + kNormChunk < nslots) ? lo + kNormChunk : nslots;
    double acc = 0.0;
    for (uint64_t i = lo + threadIdx.x; i < hi; i += kNormBlock) acc += load_once(partial + i);
    const double t = block_sum(acc, lds);
    if (threadIdx.x == 0) stage1[blockIdx.x] = t;
}

__global__ __launch_bounds__(kNormBlock) void k_norm_finalize(const double* __restrict__ stage1, uint32_t n1, float max_norm,
                                                              float* __restrict__ coef_out, double* __restrict__ sumsq_out)
{
    __shared__ double lds[kNormBlock / 64];
    double acc = 0.0;
    for (uint32_t i = threadIdx.x; i < n1; i += kNormBlock) acc += stage1[i];
    const double S = block_sum(acc, lds);
    if (threadIdx.x == 0) {
        const double norm = sqrt(S);
        double c = double(max_norm) / (norm + 1e-6);
        if (c > 1.0) c = 1.0;
        *coef_out = float(c);
        *sumsq_out = S;
    }
}

// ---- kernel: AdamW over the whole arena from the stored reduced gradient ---------------
// block_base lets one logical sweep be issued as several launches (grid size limit).
template <int OPT>
__global__ __launch_bounds__(kMaxBlock) void k_adamw(const float* __restrict__ r, float* __restrict__ p, float* __restrict__ m,
                                                     float* __restrict__ v, uint64_t nvec, uint64_t block_base,
                                                     const float* __restrict__ coef, WdMap map, StepScalars s, SnapSet snap)
{
    const uint64_t vec = (block_base + blockIdx.x) * blockDim.x + threadIdx.x;
    if (vec >= nvec) return;
    const float c = *coef;
    f32x4 g = load_once(reinterpret_cast<const f32x4*>(r) + vec);
    State4 st = load_state4<OPT>(p, m, v, vec, vec << 2, map);
    g = g * c;
    step_state4<OPT>(st, vec << 2, g, map, s);
    store_state4<OPT>(st, p, m, v, vec);
    if (snap.p) store_state4<OPT>(st, snap.p, snap.m, snap.v, vec);
}

// ---- kernel: plain copy (bandwidth yardstick) ------------------------------------------
__global__ __launch_bounds__(kMaxBlock) void k_copy(const u32x4* __restrict__ src, u32x4* __restrict__ dst, uint64_t n16,
                                                    uint64_t block_base)
{
    const uint64_t i = (block_base + blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n16) store_once(dst + i, load_once(src + i));
}

// ---- kernel: R arrays in, D arrays out (bandwidth yardstick for a mix of streams) ----------
// Vector i of every destination d receives the XOR of vector i of all sources, with d added to
// its first word (R == 0: the vector {i, 0, 0, d}).  All loads of a lane are issued before the
// first use, as in the update kernels.  D == 0 measures reads alone: the XOR is stored to
// sink[0] only by a lane whose four words all equal kProbeNever.
constexpr int kProbeMaxSrc = 16, kProbeMaxDst = 4;
constexpr uint32_t kProbeNever = 0x9E3779B9u;
struct ProbeSet {
    const u32x4* src[kProbeMaxSrc];
    u32x4* dst[kProbeMaxDst];
};

template <int R, int D>
__global__ __launch_bounds__(kMaxBlock) void k_streams(ProbeSet ps, u32x4* __restrict__ sink, uint64_t n16, uint64_t block_base)
{
    const uint64_t i = (block_base + blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= n16) return;
    u32x4 acc = u32x4{uint32_t(i), 0u, 0u, 0u};
    if constexpr (R > 0) {
        u32x4 raw[R];
#pragma unroll
        for (int k = 0; k < R; ++k) raw[k] = load_once(ps.src[k] + i);
        acc = raw[0];
#pragma unroll
        for (int k = 1; k < R; ++k) acc = acc ^ raw[k];
    }
    if constexpr (D > 0) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            u32x4 out = acc;
            out[0] += uint32_t(d);
            store_once(ps.dst[d] + i, out);
        }
    } else {
        if (acc[0] == kProbeNever && acc[1] == kProbeNever && acc[2] == kProbeNever && acc[3] == kProbeNever) sink[0] = acc;
    }
}

// ---- kernel: drain a snapshot to host memory at a bounded rate --------------------------
// dst is pinned host memory mapped into the device's address space.  The grid is a handful of
// blocks on purpose.  Measured on MI355X: while stores to the host saturate the link (this
// kernel with 8 blocks or more, and equally the runtime's own device-to-host copy kernel), every
// kernel that runs beside them takes 1.5 to 2 times as long, although the link carries under
// 1 % of the HBM rate; with 1 to 4 blocks (10-34 GB/s to the host) the others lose 3-7 %.
// Every lane walks the array with the grid's stride, four vectors in flight, until it is past
// the end.
__global__ __launch_bounds__(256) void k_drain(const u32x4* __restrict__ src, u32x4* __restrict__ dst, uint64_t n16)
{
    const uint64_t stride = uint64_t(gridDim.x) * blockDim.x;
    uint64_t i = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4 a = load_once(src + i), b = load_once(src + i + stride), c = load_once(src + i + 2 * stride),
                    d = load_once(src + i + 3 * stride);
        dst[i] = a;
        dst[i + stride] = b;
        dst[i + 2 * stride] = c;
        dst[i + 3 * stride] = d;
    }
    for (; i < n16; i += stride) dst[i] = load_once(src + i);
}

// ---- kernels: weight-decay tables written on the device (no host-to-device copy) ---------
// A chunk of the run table travels in the kernel arguments and is written to its place.
constexpr int kRunChunk = 256;
struct RunChunk {
    uint32_t first;     // index of the chunk's first run
    uint32_t count;
    uint64_t start[kRunChunk];
    uint8_t flag[kRunChunk];
};

__global__ __launch_bounds__(kRunChunk) void k_put_runs(RunChunk c, uint64_t* __restrict__ run_start, uint8_t* __restrict__ run_flag)
{
    const uint32_t i = threadIdx.x;
    if (i < c.count) {
        run_start[c.first + i] = c.start[i];
        run_flag[c.first + i] = c.flag[i];
    }
}

// Tile t takes the flag of the run that covers its first element, or kTileMixed when another run
// starts inside it.
__global__ __launch_bounds__(256) void k_build_tile_mode(const uint64_t* __restrict__ run_start, const uint8_t* __restrict__ run_flag,
                                                         uint32_t num_runs, uint64_t arena_numel, uint8_t* __restrict__ tile_mode,
                                                         uint64_t ntiles)
{
    const uint64_t t = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (t >= ntiles) return;
    const uint64_t first = t << kWdTileShift;
    uint64_t end = first + (1ull << kWdTileShift);
    if (end > arena_numel) end = arena_numel;
    uint32_t lo = 0, hi = num_runs;             // largest k with run_start[k] <= first
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (run_start[mid] <= first) lo = mid; else hi = mid;
    }
    uint8_t mode = run_flag[lo];
    if (lo + 1 < num_runs && run_start[lo + 1] < end) mode = kTileMixed;
    tile_mode[t] = mode;
}

}  // namespace shadow
