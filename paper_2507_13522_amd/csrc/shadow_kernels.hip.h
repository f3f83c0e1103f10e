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
//
// Every float operation above is a separate IEEE-754 operation (the file is
// compiled with -ffp-contract=off and correctly rounded divide/sqrt, denormals
// kept), so results do not depend on launch shape, bucket order or stream.
//
// Memory plan: each lane owns 8 consecutive elements per trip: one 128-bit load
// per bfloat16 view (two per float view), two 128-bit loads and stores for each
// of p, m, v.  A wave therefore touches 1 KiB (bf16) / 2 KiB (fp32) contiguous
// per stream per instruction, and all W loads of a trip are issued before the
// first add so that W+3 independent requests per lane are in flight.  Gradient
// and reduced-gradient reads are single-use and marked non-temporal.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace shadow {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBlock = 256;          // 4 waves
constexpr int kVec = 8;              // elements per lane per trip
constexpr int kMaxWorkers = 64;
constexpr int kWdTileShift = 10;     // weight-decay map granularity: 1024 elements

struct GradViews {
    const void* ptr[kMaxWorkers];
};

// Per-iteration scalars, prepared on the host in double and rounded once to float.
struct StepScalars {
    float beta1, beta2, omb1, omb2, decay, step_size, isq, eps, inv_w;
    uint32_t mean;
};

// Weight-decay flag of every arena element: a byte per 1024-element tile
// (0 = no decay, 1 = decay, 2 = the tile straddles tensors with different
// flags) plus the sorted run table for the rare straddling tiles.
struct WdMap {
    const uint8_t* tile_mode;
    const uint64_t* run_start;   // run k covers [run_start[k], run_start[k+1])
    const uint8_t* run_flag;
    uint32_t num_runs;
};

#ifndef SHADOW_NT_LOADS
#define SHADOW_NT_LOADS 1
#endif

template <typename T>
__device__ __forceinline__ T load_once(const T* p)
{
#if SHADOW_NT_LOADS
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}

__device__ __forceinline__ float bits_to_float(uint32_t b) { return __builtin_bit_cast(float, b); }

__device__ __forceinline__ float decay_factor_of(const WdMap& map, uint64_t e, float decay)
{
    uint32_t lo = 0, hi = map.num_runs;     // largest k with run_start[k] <= e
    while (hi - lo > 1) {
        uint32_t mid = (lo + hi) >> 1;
        if (map.run_start[mid] <= e) lo = mid; else hi = mid;
    }
    return map.run_flag[lo] ? decay : 1.0f;
}

// x * 1.0f returns x unchanged, so a masked element is multiplied by one
// instead of branching around the multiply.
__device__ __forceinline__ void adamw_elem(float& p, float& m, float& v, float g, float dfac, const StepScalars& s)
{
    p = p * dfac;
    m = s.beta1 * m + s.omb1 * g;
    v = s.beta2 * v + (s.omb2 * g) * g;
    float denom = sqrtf(v) * s.isq + s.eps;
    p = p - s.step_size * (m / denom);
}

// ---- fold of 8 consecutive elements --------------------------------------------------
// W > 0: compile-time worker count, loads issued in batches of up to kBatch views before the
// adds (which stay strictly in worker order); W == 0: run-time worker count.
__device__ __forceinline__ void widen_first(const u32x4& a, float (&r)[kVec])
{
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        r[2 * k] = bits_to_float(a[k] << 16);          // even element: low half-word
        r[2 * k + 1] = bits_to_float(a[k] & 0xFFFF0000u);
    }
}

__device__ __forceinline__ void widen_add(const u32x4& a, float (&r)[kVec])
{
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        r[2 * k] = r[2 * k] + bits_to_float(a[k] << 16);
        r[2 * k + 1] = r[2 * k + 1] + bits_to_float(a[k] & 0xFFFF0000u);
    }
}

template <int W>
__device__ __forceinline__ void fold8_bf16(const GradViews& gv, uint32_t w_rt, uint64_t vec, float (&r)[kVec])
{
    if constexpr (W > 0) {
        constexpr int kBatch = 16;
#pragma unroll
        for (int w0 = 0; w0 < W; w0 += kBatch) {
            u32x4 raw[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; ++j)
                if (w0 + j < W) raw[j] = load_once(reinterpret_cast<const u32x4*>(gv.ptr[w0 + j]) + vec);
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                if (w0 + j < W) {
                    if (w0 + j == 0) widen_first(raw[j], r); else widen_add(raw[j], r);
                }
            }
        }
    } else {
        widen_first(load_once(reinterpret_cast<const u32x4*>(gv.ptr[0]) + vec), r);
        for (uint32_t w = 1; w < w_rt; ++w) widen_add(load_once(reinterpret_cast<const u32x4*>(gv.ptr[w]) + vec), r);
    }
}

template <int W>
__device__ __forceinline__ void fold8_f32(const GradViews& gv, uint32_t w_rt, uint64_t vec, float (&r)[kVec])
{
    if constexpr (W > 0) {
        constexpr int kBatch = 8;
#pragma unroll
        for (int w0 = 0; w0 < W; w0 += kBatch) {
            f32x4 lo[kBatch], hi[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                if (w0 + j < W) {
                    lo[j] = load_once(reinterpret_cast<const f32x4*>(gv.ptr[w0 + j]) + 2 * vec);
                    hi[j] = load_once(reinterpret_cast<const f32x4*>(gv.ptr[w0 + j]) + 2 * vec + 1);
                }
            }
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                if (w0 + j < W) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        if (w0 + j == 0) { r[k] = lo[j][k]; r[4 + k] = hi[j][k]; }
                        else { r[k] = r[k] + lo[j][k]; r[4 + k] = r[4 + k] + hi[j][k]; }
                    }
                }
            }
        }
    } else {
        f32x4 a = load_once(reinterpret_cast<const f32x4*>(gv.ptr[0]) + 2 * vec);
        f32x4 b = load_once(reinterpret_cast<const f32x4*>(gv.ptr[0]) + 2 * vec + 1);
#pragma unroll
        for (int k = 0; k < 4; ++k) { r[k] = a[k]; r[4 + k] = b[k]; }
        for (uint32_t w = 1; w < w_rt; ++w) {
            a = load_once(reinterpret_cast<const f32x4*>(gv.ptr[w]) + 2 * vec);
            b = load_once(reinterpret_cast<const f32x4*>(gv.ptr[w]) + 2 * vec + 1);
#pragma unroll
            for (int k = 0; k < 4; ++k) { r[k] = r[k] + a[k]; r[4 + k] = r[4 + k] + b[k]; }
        }
    }
}

template <bool BF16, int W>
__device__ __forceinline__ void fold8(const GradViews& gv, uint32_t w_rt, uint64_t vec, float (&r)[kVec], const StepScalars& s)
{
    if constexpr (BF16) fold8_bf16<W>(gv, w_rt, vec, r); else fold8_f32<W>(gv, w_rt, vec, r);
    if (s.mean) {
#pragma unroll
        for (int k = 0; k < kVec; ++k) r[k] = r[k] * s.inv_w;
    }
}

// one element (ragged tail of a bucket)
template <bool BF16>
__device__ __forceinline__ float fold1(const GradViews& gv, uint32_t w_rt, uint64_t e, const StepScalars& s)
{
    float acc;
    if constexpr (BF16) {
        acc = bits_to_float(uint32_t(reinterpret_cast<const uint16_t*>(gv.ptr[0])[e]) << 16);
        for (uint32_t w = 1; w < w_rt; ++w)
            acc = acc + bits_to_float(uint32_t(reinterpret_cast<const uint16_t*>(gv.ptr[w])[e]) << 16);
    } else {
        acc = reinterpret_cast<const float*>(gv.ptr[0])[e];
        for (uint32_t w = 1; w < w_rt; ++w) acc = acc + reinterpret_cast<const float*>(gv.ptr[w])[e];
    }
    if (s.mean) acc = acc * s.inv_w;
    return acc;
}

__device__ __forceinline__ void load8(const float* base, uint64_t vec, float (&x)[kVec])
{
    f32x4 a = reinterpret_cast<const f32x4*>(base)[2 * vec];
    f32x4 b = reinterpret_cast<const f32x4*>(base)[2 * vec + 1];
#pragma unroll
    for (int k = 0; k < 4; ++k) { x[k] = a[k]; x[4 + k] = b[k]; }
}

__device__ __forceinline__ void load8_once(const float* base, uint64_t vec, float (&x)[kVec])
{
    f32x4 a = load_once(reinterpret_cast<const f32x4*>(base) + 2 * vec);
    f32x4 b = load_once(reinterpret_cast<const f32x4*>(base) + 2 * vec + 1);
#pragma unroll
    for (int k = 0; k < 4; ++k) { x[k] = a[k]; x[4 + k] = b[k]; }
}

__device__ __forceinline__ void store8(float* base, uint64_t vec, const float (&x)[kVec])
{
    f32x4 a, b;
#pragma unroll
    for (int k = 0; k < 4; ++k) { a[k] = x[k]; b[k] = x[4 + k]; }
    reinterpret_cast<f32x4*>(base)[2 * vec] = a;
    reinterpret_cast<f32x4*>(base)[2 * vec + 1] = b;
}

// AdamW on 8 consecutive arena elements starting at arena element e0 (multiple of 8).
__device__ __forceinline__ void adamw8(float* p, float* m, float* v, uint64_t vec, uint64_t e0, const float (&g)[kVec],
                                       const WdMap& map, const StepScalars& s)
{
    float pp[kVec], mm[kVec], vv[kVec];
    load8(p, vec, pp);
    load8(m, vec, mm);
    load8(v, vec, vv);
    const uint8_t mode = map.tile_mode[e0 >> kWdTileShift];
    if (mode != 2) {
        const float dfac = mode ? s.decay : 1.0f;
#pragma unroll
        for (int k = 0; k < kVec; ++k) adamw_elem(pp[k], mm[k], vv[k], g[k], dfac, s);
    } else {
#pragma unroll
        for (int k = 0; k < kVec; ++k) adamw_elem(pp[k], mm[k], vv[k], g[k], decay_factor_of(map, e0 + k, s.decay), s);
    }
    store8(p, vec, pp);
    store8(m, vec, mm);
    store8(v, vec, vv);
}

// ---- kernel: fold + AdamW in one pass (clipping off) ---------------------------------
// p, m, v point at the bucket's first element; arena_off is that element's arena index.
template <bool BF16, int W>
__global__ __launch_bounds__(kBlock) void k_fold_adamw(GradViews gv, uint32_t w_rt, float* __restrict__ p,
                                                       float* __restrict__ m, float* __restrict__ v, uint64_t n,
                                                       uint64_t arena_off, WdMap map, StepScalars s)
{
    const uint64_t nvec = n >> 3;
    const uint64_t stride = uint64_t(gridDim.x) * kBlock;
    for (uint64_t vec = uint64_t(blockIdx.x) * kBlock + threadIdx.x; vec < nvec; vec += stride) {
        float r[kVec];
        fold8<BF16, W>(gv, w_rt, vec, r, s);
        adamw8(p, m, v, vec, arena_off + (vec << 3), r, map, s);
    }
    const uint32_t tail = uint32_t(n & 7);
    if (blockIdx.x == 0 && threadIdx.x < tail) {
        const uint64_t e = (nvec << 3) + threadIdx.x;
        float g = fold1<BF16>(gv, w_rt, e, s);
        float pp = p[e], mm = m[e], vv = v[e];
        adamw_elem(pp, mm, vv, g, decay_factor_of(map, arena_off + e, s.decay), s);
        p[e] = pp; m[e] = mm; v[e] = vv;
    }
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

// ---- kernel: fold + sum of squares, reduced gradient stored (clipping on) -------------
// r_out points at the bucket's first scratch element; partial has gridDim.x slots.
template <bool BF16, int W>
__global__ __launch_bounds__(kBlock) void k_fold_sumsq(GradViews gv, uint32_t w_rt, float* __restrict__ r_out, uint64_t n,
                                                       double* __restrict__ partial, StepScalars s)
{
    __shared__ double lds[kBlock / 64];
    const uint64_t nvec = n >> 3;
    const uint64_t stride = uint64_t(gridDim.x) * kBlock;
    double acc = 0.0;
    for (uint64_t vec = uint64_t(blockIdx.x) * kBlock + threadIdx.x; vec < nvec; vec += stride) {
        float r[kVec];
        fold8<BF16, W>(gv, w_rt, vec, r, s);
        store8(r_out, vec, r);
#pragma unroll
        for (int k = 0; k < kVec; ++k) {
            const double d = double(r[k]);
            acc = fma(d, d, acc);        // d*d is exact in double, so this equals acc + d*d
        }
    }
    const uint32_t tail = uint32_t(n & 7);
    if (blockIdx.x == 0 && threadIdx.x < tail) {
        const uint64_t e = (nvec << 3) + threadIdx.x;
        const float g = fold1<BF16>(gv, w_rt, e, s);
        r_out[e] = g;
        const double d = double(g);
        acc = fma(d, d, acc);
    }
    const double t = block_sum(acc, lds);
    if (threadIdx.x == 0) partial[blockIdx.x] = t;
}

// ---- kernel: norm and clip coefficient (one block, fixed summation order) --------------
__global__ __launch_bounds__(1024) void k_norm_finalize(const double* __restrict__ partial, uint32_t nslots, float max_norm,
                                                        float* __restrict__ coef_out, double* __restrict__ sumsq_out)
{
    __shared__ double lds[1024 / 64];
    double acc = 0.0;
    for (uint32_t i = threadIdx.x; i < nslots; i += blockDim.x) acc += partial[i];
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
__global__ __launch_bounds__(kBlock) void k_adamw(const float* __restrict__ r, float* __restrict__ p, float* __restrict__ m,
                                                  float* __restrict__ v, uint64_t nvec, const float* __restrict__ coef,
                                                  WdMap map, StepScalars s)
{
    const float c = *coef;
    const uint64_t stride = uint64_t(gridDim.x) * kBlock;
    for (uint64_t vec = uint64_t(blockIdx.x) * kBlock + threadIdx.x; vec < nvec; vec += stride) {
        float g[kVec];
        load8_once(r, vec, g);
#pragma unroll
        for (int k = 0; k < kVec; ++k) g[k] = g[k] * c;
        adamw8(p, m, v, vec, vec << 3, g, map, s);
    }
}

// ---- kernel: plain copy (bandwidth yardstick) ------------------------------------------
__global__ __launch_bounds__(kBlock) void k_copy(const u32x4* __restrict__ src, u32x4* __restrict__ dst, uint64_t n16)
{
    const uint64_t stride = uint64_t(gridDim.x) * kBlock;
    for (uint64_t i = uint64_t(blockIdx.x) * kBlock + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace shadow
