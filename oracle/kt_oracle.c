/*
 * CPU checker for the per-device gradient reduction stage of a load-adaptive
 * data-parallel step (KAITIAN, Sec. III: gradient synchronisation under DDP;
 * Sec. III-C: batch shares b_i proportional to device score, sum b_i = B).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, single-threaded C that writes out the
 * definitions; it shares nothing with the GPU library and must never be used
 * by it.  Build with -ffp-contract=off (no fused contraction of a*b+c).
 *
 * What is combined: device k computes the mean gradient over its b_k samples;
 * the mean over the whole global batch of B samples is sum_k (b_k/B) * g_k,
 * so the K peer copies of a bucket are combined with weights w_k = b_k/B
 * (consequence of the unequal shares of Sec. III-C, display equation).
 *
 * Two arithmetic modes for every floating-point step:
 *   D ("definition"): products and sums in double, ascending k, ONE rounding
 *      to the storage type at the end.  This is the graded reference.
 *   S ("strict"): the stated device arithmetic step by step -- fp32 product
 *      for k = 0, then fp32 fused multiply-add for k = 1..K-1 in ascending k,
 *      then (bf16 only) round-to-nearest-even to bf16.
 *
 * bf16 = the upper 16 bits of an IEEE binary32 (1 sign, 8 exponent, 7 fraction).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* ---- bf16 helpers ------------------------------------------------------ */

/* bf16 -> binary32, exact: the bits become the upper half of the word. */
float kto_bf16_widen(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* double -> bf16 with a single round-to-nearest-even.
 * Values are scaled by a power of two (exact) so that one unit equals the
 * bf16 spacing at that magnitude, then rounded with nearbyint (RNE in the
 * default rounding mode).  Spacing: 2^(e-7) for 2^e <= |d| < 2^(e+1), with e
 * clamped below at -126 (subnormals share the spacing 2^-133).  Anything that
 * rounds to 2^128 or more becomes infinity.  NaN stays a quiet NaN. */
uint16_t kto_bf16_round(double d)
{
    uint16_t sign = (uint16_t)(signbit(d) ? 0x8000u : 0u);
    if (isnan(d)) return (uint16_t)(sign | 0x7FC0u);
    double a = fabs(d);
    if (isinf(a)) return (uint16_t)(sign | 0x7F80u);
    if (a == 0.0) return sign;
    int ex;
    (void)frexp(a, &ex);            /* a = m * 2^ex, m in [0.5, 1) */
    int e = ex - 1;                 /* 2^e <= a < 2^(e+1) */
    if (e < -126) e = -126;
    double q = ldexp(1.0, e - 7);   /* spacing */
    double m = nearbyint(a / q);    /* a/q exact: power-of-two scaling */
    double r = m * q;               /* representable in bf16, or 2^128 */
    if (r >= ldexp(1.0, 128)) return (uint16_t)(sign | 0x7F80u);
    float f = (float)r;             /* exact: bf16 values are binary32 values */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return (uint16_t)(sign | (uint16_t)(u >> 16));
}

/* ---- K-way weighted combine: out[i] = sum_k w[k] * x[k][i] -------------- */

void kto_reduce_f32_D(const float *const *x, const float *w, int K, int64_t n,
                      float *out)
{
    for (int64_t i = 0; i < n; ++i) {
        double acc = 0.0;
        for (int k = 0; k < K; ++k) acc += (double)w[k] * (double)x[k][i];
        out[i] = (float)acc;
    }
}

void kto_reduce_f32_S(const float *const *x, const float *w, int K, int64_t n,
                      float *out)
{
    for (int64_t i = 0; i < n; ++i) {
        float acc = w[0] * x[0][i];
        for (int k = 1; k < K; ++k) acc = fmaf(w[k], x[k][i], acc);
        out[i] = acc;
    }
}

void kto_reduce_bf16_D(const uint16_t *const *x, const float *w, int K,
                       int64_t n, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i) {
        double acc = 0.0;
        for (int k = 0; k < K; ++k)
            acc += (double)w[k] * (double)kto_bf16_widen(x[k][i]);
        out[i] = kto_bf16_round(acc);
    }
}

void kto_reduce_bf16_S(const uint16_t *const *x, const float *w, int K,
                       int64_t n, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i) {
        float acc = w[0] * kto_bf16_widen(x[0][i]);
        for (int k = 1; k < K; ++k)
            acc = fmaf(w[k], kto_bf16_widen(x[k][i]), acc);
        out[i] = kto_bf16_round((double)acc);
    }
}

/* ---- scale step of unpack: out[i] = scale * in[i] ----------------------- */

/* fp32: a binary32 product is exact in double, so D and S coincide. */
void kto_scale_f32(const float *in, int64_t n, float scale, float *out)
{
    for (int64_t i = 0; i < n; ++i)
        out[i] = (float)((double)scale * (double)in[i]);
}

void kto_scale_bf16_D(const uint16_t *in, int64_t n, float scale,
                      uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i)
        out[i] = kto_bf16_round((double)scale * (double)kto_bf16_widen(in[i]));
}

void kto_scale_bf16_S(const uint16_t *in, int64_t n, float scale,
                      uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i) {
        float p = scale * kto_bf16_widen(in[i]);   /* rounded to binary32 */
        out[i] = kto_bf16_round((double)p);
    }
}

/* ---- SGD with momentum and weight decay applied while unpacking ----------
 * The optimizer of the paper's training runs (Sec. IV-B: SGD, momentum 0.9,
 * weight decay 5e-4), in the usual form: with gradient g = scale * bucket value,
 *     g' = g + wd * p;   v' = g'  (first step)  or  mu * v + g';   p' = p - lr * v'.
 * Parameters p and momentum v are binary32 and updated in place.
 * D: each stored result (v', p') is the exact expression of the stored inputs,
 *    evaluated in double, rounded once; p' uses the stored (rounded) v'.
 * S: binary32 steps: g = scale*x (rounded), g' = fma(wd, p, g),
 *    v' = fma(mu, v, g'), p' = fma(-lr, v', p).                              */

void kto_sgd_f32_D(const float *x, int64_t n, float scale, float *p, float *v,
                   float lr, float mu, float wd, int first)
{
    for (int64_t i = 0; i < n; ++i) {
        double g = (double)scale * (double)x[i] + (double)wd * (double)p[i];
        double vv = first ? g : (double)mu * (double)v[i] + g;
        float vn = (float)vv;
        p[i] = (float)((double)p[i] - (double)lr * (double)vn);
        v[i] = vn;
    }
}

void kto_sgd_f32_S(const float *x, int64_t n, float scale, float *p, float *v,
                   float lr, float mu, float wd, int first)
{
    for (int64_t i = 0; i < n; ++i) {
        float g = scale * x[i];
        float g2 = fmaf(wd, p[i], g);
        float vn = first ? g2 : fmaf(mu, v[i], g2);
        p[i] = fmaf(-lr, vn, p[i]);
        v[i] = vn;
    }
}

void kto_sgd_bf16_D(const uint16_t *x, int64_t n, float scale, float *p, float *v,
                    float lr, float mu, float wd, int first)
{
    for (int64_t i = 0; i < n; ++i) {
        double g = (double)scale * (double)kto_bf16_widen(x[i]) + (double)wd * (double)p[i];
        double vv = first ? g : (double)mu * (double)v[i] + g;
        float vn = (float)vv;
        p[i] = (float)((double)p[i] - (double)lr * (double)vn);
        v[i] = vn;
    }
}

void kto_sgd_bf16_S(const uint16_t *x, int64_t n, float scale, float *p, float *v,
                    float lr, float mu, float wd, int first)
{
    for (int64_t i = 0; i < n; ++i) {
        float g = scale * kto_bf16_widen(x[i]);
        float g2 = fmaf(wd, p[i], g);
        float vn = first ? g2 : fmaf(mu, v[i], g2);
        p[i] = fmaf(-lr, vn, p[i]);
        v[i] = vn;
    }
}

/* ---- mixed precision: the bf16 model copy of binary32 master parameters ----
 * model[i] = p[i] rounded to nearest-even to bf16 (one rounding; NaN quiet). */
void kto_f32_to_bf16(const float *p, int64_t n, uint16_t *model)
{
    for (int64_t i = 0; i < n; ++i) model[i] = kto_bf16_round((double)p[i]);
}

