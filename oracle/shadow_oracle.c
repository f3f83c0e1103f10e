/*
 * CPU oracle for the shadow update (TEST INFRASTRUCTURE ONLY).
 *
 * A plain, slow, direct transcription of what the shadow node of the paper
 * computes once per iteration (section 4, step 4 of the overview; section
 * 4.2.3 "Updating the Checkpoint"): take the gradients of an iteration,
 * reduce them over the data-parallel workers (section 2.1: the reduce of
 * AllReduce sums or averages), and run the same optimizer step the trainers
 * run -- AdamW (section 6, Loshchilov & Hutter) -- on the checkpoint
 * replica's parameters and optimizer state.  Section 4.2.4 requires the
 * optimizer to be "functional" (every element is updated independently), so
 * every loop here is a loop over independent elements.
 *
 * Only tests, the smoke check and the CPU-baseline leg of the benchmark may
 * call this file.  It shares no code with the GPU library.
 *
 * Two variants:
 *   *_f32  the canonical single-precision evaluation order (the precision the
 *          replica is kept in); the GPU path is compared against this one.
 *   *_f64  the textbook formulas in double precision from the same inputs; it
 *          bounds the rounding error of the f32 variant and is the brute-force
 *          check on small vectors.
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -fPIC -shared (no fast-math, no
 * -march flags: every +,*,/,sqrt below is one IEEE-754 operation, denormals kept).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- threads (elements are independent: section 4.2.4) ------------------ */
void oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int oracle_get_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* bfloat16 -> float: the 16 bits are the top half of the float's pattern. */
static inline float widen_bf16(uint16_t h)
{
    uint32_t b = (uint32_t)h << 16;
    float f;
    memcpy(&f, &b, sizeof f);
    return f;
}

void oracle_widen_bf16(const uint16_t *h, uint64_t n, float *out)
{
    for (uint64_t i = 0; i < n; ++i) out[i] = widen_bf16(h[i]);
}

/* ---- reduce over the W workers (section 2.1, "summing or averaging") -----
 * r[i] = g_0[i] + g_1[i] + ... + g_{W-1}[i], left to right in float, then
 * (mean) one multiply by float(1/W).  Gradients given in bfloat16 are widened
 * exactly first; nothing is ever added in bfloat16. */
void oracle_fold_f32(const float *const *g, uint32_t W, uint64_t n, int mean, float *r)
{
    const float invW = (float)(1.0 / (double)W);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i) {
        float acc = g[0][i];
        for (uint32_t w = 1; w < W; ++w) acc = acc + g[w][i];
        if (mean) acc = acc * invW;
        r[i] = acc;
    }
}

void oracle_fold_bf16(const uint16_t *const *g, uint32_t W, uint64_t n, int mean, float *r)
{
    const float invW = (float)(1.0 / (double)W);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i) {
        float acc = widen_bf16(g[0][i]);
        for (uint32_t w = 1; w < W; ++w) acc = acc + widen_bf16(g[w][i]);
        if (mean) acc = acc * invW;
        r[i] = acc;
    }
}

/* double-precision reduce: exact sum of the inputs' values (as far as double
 * allows), divided by W. */
void oracle_fold_f32_f64(const float *const *g, uint32_t W, uint64_t n, int mean, double *r)
{
    for (uint64_t i = 0; i < n; ++i) {
        double acc = 0.0;
        for (uint32_t w = 0; w < W; ++w) acc += (double)g[w][i];
        r[i] = mean ? acc / (double)W : acc;
    }
}

void oracle_fold_bf16_f64(const uint16_t *const *g, uint32_t W, uint64_t n, int mean, double *r)
{
    for (uint64_t i = 0; i < n; ++i) {
        double acc = 0.0;
        for (uint32_t w = 0; w < W; ++w) acc += (double)widen_bf16(g[w][i]);
        r[i] = mean ? acc / (double)W : acc;
    }
}

/* ---- global-norm clipping ------------------------------------------------
 * Not part of the paper's text; it is the usual gradient-norm clipping that
 * precedes an optimizer step: with S the sum of squares of the WHOLE reduced
 * gradient, c = min(1, max_norm / (sqrt(S) + 1e-6)).  S is accumulated in
 * extended precision so that it is the mathematical sum to well below one
 * float ulp of c; c is rounded once to float. */
void oracle_sumsq_accumulate(const float *r, uint64_t n, long double *acc)
{
    long double s = *acc;
    for (uint64_t i = 0; i < n; ++i) s += (long double)r[i] * (long double)r[i];
    *acc = s;
}

void oracle_sumsq_accumulate_f64(const double *r, uint64_t n, long double *acc)
{
    long double s = *acc;
    for (uint64_t i = 0; i < n; ++i) s += (long double)r[i] * (long double)r[i];
    *acc = s;
}

/* weighted form for inputs that repeat a tile: adds count * r^2 */
void oracle_sumsq_accumulate_weighted(const float *r, const uint64_t *count, uint64_t n, long double *acc)
{
    long double s = *acc;
    for (uint64_t i = 0; i < n; ++i)
        s += (long double)count[i] * ((long double)r[i] * (long double)r[i]);
    *acc = s;
}

double oracle_sumsq_value(const long double *acc) { return (double)*acc; }

double oracle_clip_coef_f64(const long double *sumsq, float max_norm)
{
    long double norm = sqrtl(*sumsq);
    long double c = (long double)max_norm / (norm + (long double)1e-6);
    if (c > 1.0L) c = 1.0L;
    return (double)c;
}

float oracle_clip_coef_f32(const long double *sumsq, float max_norm)
{
    long double norm = sqrtl(*sumsq);
    long double c = (long double)max_norm / (norm + (long double)1e-6);
    if (c > 1.0L) c = 1.0L;
    return (float)c;
}

/* ---- AdamW, canonical float evaluation ----------------------------------
 * Per-step scalars are formed in double from the float hyper-parameters and
 * rounded once to float:
 *   decay = 1 - lr*wd, omb1 = 1 - beta1, omb2 = 1 - beta2,
 *   step_size = lr / (1 - beta1^t), isq = 1 / sqrt(1 - beta2^t).
 * out[5] = {decay, omb1, omb2, step_size, isq}; t counts from 1. */
void oracle_step_scalars(float lr, float beta1, float beta2, float wd, uint64_t t, float out[5])
{
    double bc1 = 1.0 - pow((double)beta1, (double)t);
    double bc2 = 1.0 - pow((double)beta2, (double)t);
    out[0] = (float)(1.0 - (double)lr * (double)wd);
    out[1] = (float)(1.0 - (double)beta1);
    out[2] = (float)(1.0 - (double)beta2);
    out[3] = (float)((double)lr / bc1);
    out[4] = (float)(1.0 / sqrt(bc2));
}

/* One tensor (or any run of elements with one weight-decay flag).
 *   r: reduced gradient (unclipped).  clip != 0: r is first multiplied by c.
 *   wd_flag != 0: decoupled weight decay p *= (1 - lr*wd) before the Adam step;
 *   wd_flag == 0: the multiply is skipped (bias / norm tensors).
 * Adam step with bias correction folded into step_size and isq:
 *   m = b1*m + (1-b1)*g ; v = b2*v + ((1-b2)*g)*g ;
 *   p = p - step_size * ( m / (sqrt(v)*isq + eps) ).                        */
void oracle_adamw_f32(float *p, float *m, float *v, const float *r, uint64_t n, int wd_flag,
                      float lr, float beta1, float beta2, float eps, float wd, uint64_t t,
                      int clip, float c)
{
    float s[5];
    oracle_step_scalars(lr, beta1, beta2, wd, t, s);
    const float decay = s[0], omb1 = s[1], omb2 = s[2], step_size = s[3], isq = s[4];
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i) {
        float g = r[i];
        if (clip) g = g * c;
        float pi = p[i];
        if (wd_flag) pi = pi * decay;
        float mi = beta1 * m[i] + omb1 * g;
        float vi = beta2 * v[i] + (omb2 * g) * g;
        float denom = sqrtf(vi) * isq + eps;
        pi = pi - step_size * (mi / denom);
        p[i] = pi;
        m[i] = mi;
        v[i] = vi;
    }
}

/* ---- AdamW, textbook formulas in double -----------------------------------
 *   g' = c*g ; p = p*(1 - lr*wd) ;
 *   m = b1*m + (1-b1)*g' ; v = b2*v + (1-b2)*g'^2 ;
 *   mhat = m/(1-b1^t) ; vhat = v/(1-b2^t) ;
 *   p = p - lr*mhat/(sqrt(vhat) + eps).                                     */
void oracle_adamw_f64(double *p, double *m, double *v, const double *r, uint64_t n, int wd_flag,
                      double lr, double beta1, double beta2, double eps, double wd, uint64_t t,
                      int clip, double c)
{
    const double bc1 = 1.0 - pow(beta1, (double)t);
    const double bc2 = 1.0 - pow(beta2, (double)t);
    for (uint64_t i = 0; i < n; ++i) {
        double g = clip ? r[i] * c : r[i];
        double pi = p[i];
        if (wd_flag) pi = pi * (1.0 - lr * wd);
        double mi = beta1 * m[i] + (1.0 - beta1) * g;
        double vi = beta2 * v[i] + (1.0 - beta2) * g * g;
        double mhat = mi / bc1;
        double vhat = vi / bc2;
        pi = pi - lr * mhat / (sqrt(vhat) + eps);
        p[i] = pi;
        m[i] = mi;
        v[i] = vi;
    }
}

/* ---- other functional optimizers (section 4.2.4 names SGD, Adam and AdamW) --
 * Adam (Kingma & Ba) with the classic L2 penalty: the decay term joins the
 * gradient, g' = g + wd*p (on tensors with the flag), and then the moments and
 * the bias-corrected step are those of AdamW without its decay multiply.      */
void oracle_adam_f32(float *p, float *m, float *v, const float *r, uint64_t n, int wd_flag,
                     float lr, float beta1, float beta2, float eps, float wd, uint64_t t,
                     int clip, float c)
{
    float s[5];
    oracle_step_scalars(lr, beta1, beta2, wd, t, s);
    const float omb1 = s[1], omb2 = s[2], step_size = s[3], isq = s[4];
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i) {
        float g = r[i];
        if (clip) g = g * c;
        float pi = p[i];
        if (wd_flag) g = g + wd * pi;
        float mi = beta1 * m[i] + omb1 * g;
        float vi = beta2 * v[i] + (omb2 * g) * g;
        float denom = sqrtf(vi) * isq + eps;
        pi = pi - step_size * (mi / denom);
        p[i] = pi;
        m[i] = mi;
        v[i] = vi;
    }
}

void oracle_adam_f64(double *p, double *m, double *v, const double *r, uint64_t n, int wd_flag,
                     double lr, double beta1, double beta2, double eps, double wd, uint64_t t,
                     int clip, double c)
{
    const double bc1 = 1.0 - pow(beta1, (double)t);
    const double bc2 = 1.0 - pow(beta2, (double)t);
    for (uint64_t i = 0; i < n; ++i) {
        double g = clip ? r[i] * c : r[i];
        double pi = p[i];
        if (wd_flag) g = g + wd * pi;
        double mi = beta1 * m[i] + (1.0 - beta1) * g;
        double vi = beta2 * v[i] + (1.0 - beta2) * g * g;
        pi = pi - lr * (mi / bc1) / (sqrt(vi / bc2) + eps);
        p[i] = pi;
        m[i] = mi;
        v[i] = vi;
    }
}

/* SGD with momentum mu (no dampening, no Nesterov), L2 penalty in the gradient:
 *   g' = g + wd*p ; b = mu*b + g' ; p = p - lr*b.   b starts at zero, so the
 *   first step is b = g'.  mu = 0 is plain SGD.                               */
void oracle_sgd_f32(float *p, float *b, const float *r, uint64_t n, int wd_flag,
                    float lr, float mu, float wd, int clip, float c)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i) {
        float g = r[i];
        if (clip) g = g * c;
        float pi = p[i];
        if (wd_flag) g = g + wd * pi;
        float bi = mu * b[i] + g;
        pi = pi - lr * bi;
        p[i] = pi;
        b[i] = bi;
    }
}

void oracle_sgd_f64(double *p, double *b, const double *r, uint64_t n, int wd_flag,
                    double lr, double mu, double wd, int clip, double c)
{
    for (uint64_t i = 0; i < n; ++i) {
        double g = clip ? r[i] * c : r[i];
        double pi = p[i];
        if (wd_flag) g = g + wd * pi;
        double bi = mu * b[i] + g;
        pi = pi - lr * bi;
        p[i] = pi;
        b[i] = bi;
    }
}
