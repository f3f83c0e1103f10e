/*
 * The C ABI used from plain C, without Python or PyTorch: build a layout, allocate the arenas with the
 * HIP runtime, apply one iteration of two buckets (W = 2, float gradients, no clipping) and check the
 * result against the closed form of the first AdamW step:
 *     m = (1-b1) g,  v = (1-b2) g^2,  p = p0 (1 - lr wd) - lr g / (|g| + eps)      (g = mean gradient)
 * evaluated in double.  Exit status 0 = pass.
 *
 * gcc -std=c11 -D__HIP_PLATFORM_AMD__ -I/opt/rocm/include -Iinclude abi_smoke.c -L<libdir> -lshadow -L/opt/rocm/lib -lamdhip64 -lm
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include "shadow.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define CHECK_SH(x) do { int32_t s_ = (x); if (s_ != SHADOW_OK) { printf("shadow error %s (%d) at line %d: %s\n", shadow_strerror(s_), s_, __LINE__, shadow_last_hip_error()); return 3; } } while (0)

int main(void)
{
    const shadow_tensor_desc tensors[3] = {{1000, 1, 0}, {37, 0, 0}, {5003, 1, 0}};
    shadow_layout* lay = NULL;
    CHECK_SH(shadow_layout_create(&lay, tensors, 3, NULL, 4, 6000 * 4));
    uint32_t nb = 0;
    uint64_t arena = 0, params = 0;
    CHECK_SH(shadow_layout_num_buckets(lay, &nb));
    CHECK_SH(shadow_layout_arena_numel(lay, &arena));
    CHECK_SH(shadow_layout_num_params(lay, &params));
    if (nb != 2 || params != 6040) { printf("unexpected layout: %u buckets, %llu params\n", nb, (unsigned long long)params); return 1; }

    shadow_hparams hp = {0};
    hp.lr = 1e-3f; hp.beta1 = 0.9f; hp.beta2 = 0.999f; hp.eps = 1e-8f; hp.weight_decay = 0.01f; hp.max_grad_norm = 0.f;
    hp.num_workers = 2; hp.grad_dtype = SHADOW_GRAD_F32; hp.reduce_op = SHADOW_REDUCE_MEAN; hp.num_streams = 2;
    hp.optimizer = SHADOW_OPT_ADAMW; hp.batch_bytes = 0;

    float *h_p = calloc(arena, sizeof(float)), *h_out = calloc(arena, sizeof(float));
    float *d_p, *d_m, *d_v;
    CHECK_HIP(hipMalloc((void**)&d_p, arena * sizeof(float)));
    CHECK_HIP(hipMalloc((void**)&d_m, arena * sizeof(float)));
    CHECK_HIP(hipMalloc((void**)&d_v, arena * sizeof(float)));
    for (uint64_t i = 0; i < arena; ++i) h_p[i] = 0.02f * (float)((int)(i * 7919u % 2001u) - 1000) / 1000.0f;
    CHECK_HIP(hipMemcpy(d_p, h_p, arena * sizeof(float), hipMemcpyHostToDevice));
    CHECK_HIP(hipMemset(d_m, 0, arena * sizeof(float)));
    CHECK_HIP(hipMemset(d_v, 0, arena * sizeof(float)));

    shadow_ctx* ctx = NULL;
    CHECK_SH(shadow_init(&ctx, lay, &hp, d_p, d_m, d_v, NULL, 0, NULL));

    int bad = 0;
    float* d_g[2][2];
    float* h_g[2][2];
    uint64_t off[2], n[2];
    for (uint32_t b = 0; b < nb; ++b) {
        uint32_t nt;
        CHECK_SH(shadow_layout_bucket(lay, b, &off[b], &n[b], &nt));
        for (int w = 0; w < 2; ++w) {
            h_g[b][w] = malloc(n[b] * sizeof(float));
            for (uint64_t i = 0; i < n[b]; ++i)
                h_g[b][w][i] = 1e-3f * (float)((int)((i * 31u + (unsigned)w * 17u + b * 5u) % 201u) - 100) / 100.0f;
            CHECK_HIP(hipMalloc((void**)&d_g[b][w], n[b] * sizeof(float)));
            CHECK_HIP(hipMemcpy(d_g[b][w], h_g[b][w], n[b] * sizeof(float), hipMemcpyHostToDevice));
        }
    }
    /* the replica knows its bucket map */
    uint32_t nb_ctx = 0;
    CHECK_SH(shadow_num_buckets(ctx, &nb_ctx));
    for (uint32_t b = 0; b < nb; ++b) {
        uint64_t o2 = 0, n2 = 0;
        CHECK_SH(shadow_bucket_info(ctx, b, &o2, &n2));
        if (nb_ctx != nb || o2 != off[b] || n2 != n[b]) { printf("bucket map of the context differs from the layout's\n"); bad = 1; }
    }
    /* deliver bucket 1 first: arrival order is free; a duplicate is refused.  Bucket 0's views are
       produced by copies on a stream of the caller's: the event recorded behind them orders the fold. */
    const void* v1[2] = {d_g[1][0], d_g[1][1]};
    const void* v0[2] = {d_g[0][0], d_g[0][1]};
    hipStream_t producer;
    hipEvent_t ready, consumed, snapped;
    CHECK_HIP(hipStreamCreateWithFlags(&producer, hipStreamNonBlocking));
    CHECK_HIP(hipEventCreateWithFlags(&ready, hipEventDisableTiming));
    CHECK_HIP(hipEventCreateWithFlags(&consumed, hipEventDisableTiming));
    CHECK_HIP(hipEventCreateWithFlags(&snapped, hipEventDisableTiming));
    CHECK_SH(shadow_apply_bucket(ctx, 1, v1, 1, NULL));
    if (shadow_apply_bucket(ctx, 1, v1, 1, NULL) != SHADOW_EDUP) { printf("duplicate bucket was not refused\n"); bad = 1; }
    if (shadow_snapshot(ctx, h_out, NULL, NULL, NULL, NULL) != SHADOW_EBUSY) { printf("snapshot inside an iteration was not refused\n"); bad = 1; }
    CHECK_HIP(hipEventRecord(ready, producer));
    CHECK_SH(shadow_apply_bucket(ctx, 0, v0, 1, ready));
    CHECK_SH(shadow_record_consumed(ctx, 0, consumed));
    uint64_t step = 0;
    float* d_snap;
    CHECK_HIP(hipMalloc((void**)&d_snap, arena * sizeof(float)));
    CHECK_SH(shadow_snapshot(ctx, d_snap, NULL, NULL, &step, snapped));
    CHECK_HIP(hipEventSynchronize(consumed));
    CHECK_HIP(hipEventSynchronize(snapped));       /* the copy is complete without a shadow_sync */
    CHECK_HIP(hipMemcpy(h_out, d_snap, arena * sizeof(float), hipMemcpyDeviceToHost));
    uint64_t waited = 0;
    CHECK_SH(shadow_snapshot_wait(ctx, &waited));
    if (waited != 1) { printf("snapshot_wait step %llu\n", (unsigned long long)waited); bad = 1; }
    CHECK_SH(shadow_sync(ctx));
    if (step != 1) { printf("snapshot step %llu\n", (unsigned long long)step); bad = 1; }

    /* closed form, per tensor (tensor t -> bucket, offset) */
    double worst = 0.0;
    for (uint32_t t = 0; t < 3; ++t) {
        uint32_t b;
        uint64_t ob, oa;
        CHECK_SH(shadow_layout_tensor(lay, t, &b, &ob, &oa));
        for (uint64_t i = 0; i < tensors[t].numel; ++i) {
            const double g = ((double)h_g[b][0][ob + i] + (double)h_g[b][1][ob + i]) / 2.0;
            const double p0 = h_p[oa + i];
            const double decay = tensors[t].weight_decay ? 1.0 - (double)hp.lr * (double)hp.weight_decay : 1.0;
            const double want = p0 * decay - (double)hp.lr * g / (fabs(g) + (double)hp.eps);
            /* relative to the size of the terms: p0 and the step may cancel */
            const double err = fabs((double)h_out[oa + i] - want) / fmax(fmax(fabs(want), fabs(p0)), (double)hp.lr);
            if (err > worst) worst = err;
        }
    }
    printf("abi smoke: %u buckets, arena %llu floats, worst error vs closed form relative to the terms %.3g\n", nb, (unsigned long long)arena, worst);
    if (worst > 1e-6) bad = 1;     /* a few float roundings */
    CHECK_SH(shadow_destroy(ctx));
    CHECK_SH(shadow_layout_destroy(lay));
    return bad;
}
