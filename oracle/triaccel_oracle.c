/*
 * CPU oracle for the Tri-Accel per-layer optimizer step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the yardstick the HIP library is
 * checked against; it is deliberately plain and slow and shares no code,
 * table or helper with the HIP path.  Nothing in the product may call it.
 *
 * Each function states the passage of the paper (arXiv 2508.16905) it follows.
 * Where the paper leaves a quantity undefined, the reading taken is stated in
 * the function's comment.
 *
 * Arithmetic conventions
 *   - Reductions (mean, variance): two passes, accumulated in double.
 *   - Element-wise state recurrences: IEEE binary32, one rounding per written
 *     operation, fused multiply-add only where fmaf() is written.  Build with
 *     -ffp-contract=off and without -ffast-math.
 *   - Precision codes: 0 = FP16, 1 = BF16, 2 = FP32 (the order of the cases in
 *     the precision rule of Sec. 3.1).
 */

#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_FP16 = 0, ORC_BF16 = 1, ORC_FP32 = 2 };

static uint32_t bits_of(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float float_of(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* ------------------------------------------------------------------------ */
/* Number formats.  IEEE 754 binary16 and bfloat16 (binary32 with the low 16
 * significand bits removed), written from the formats' definitions: a value is
 * rounded to the nearest representable one, ties to the one with an even last
 * significand digit; magnitudes at or beyond the overflow threshold become
 * infinity; NaN stays NaN (quiet).                                          */
/* ------------------------------------------------------------------------ */

float oracle_f16_to_f32(uint16_t h)
{
    int sign = h >> 15, e = (h >> 10) & 31, m = h & 0x3ff;
    float v;
    if (e == 31) {
        if (m) return float_of(((uint32_t)sign << 31) | 0x7fc00000u | ((uint32_t)m << 13));
        v = INFINITY;
    } else if (e == 0) {
        v = ldexpf((float)m, -24);            /* subnormal: m * 2^-24 */
    } else {
        v = ldexpf((float)(1024 + m), e - 25); /* (1 + m/1024) * 2^(e-15) */
    }
    return sign ? -v : v;
}

float oracle_bf16_to_f32(uint16_t b) { return float_of((uint32_t)b << 16); }

uint16_t oracle_f32_to_f16(float x)
{
    uint16_t sign = (uint16_t)((bits_of(x) >> 31) << 15);
    if (isnan(x)) return (uint16_t)(sign | 0x7e00);
    double a = fabs((double)x);
    if (a >= 65520.0) return (uint16_t)(sign | 0x7c00); /* 65504 + half an ulp and beyond */
    if (a == 0.0) return sign;
    int e;
    frexp(a, &e);               /* a = f * 2^e, f in [0.5, 1)  =>  a in [2^(e-1), 2^e) */
    int ex = e - 1;             /* floor(log2 a) */
    if (ex < -14) ex = -14;     /* subnormal range shares the smallest normal exponent */
    double quantum = ldexp(1.0, ex - 10);
    double q = nearbyint(a / quantum); /* default rounding mode: to nearest, ties to even */
    /* q in [0, 2048]; 2048 means the value rounded up into the next binade */
    if (q >= 2048.0) { q = 1024.0; ex += 1; }
    if (q < 1024.0) return (uint16_t)(sign | (uint16_t)q);             /* subnormal or zero */
    return (uint16_t)(sign | (uint16_t)((ex + 15) << 10) | (uint16_t)(q - 1024.0));
}

uint16_t oracle_f32_to_bf16(float x)
{
    uint16_t sign = (uint16_t)((bits_of(x) >> 31) << 15);
    if (isnan(x)) return (uint16_t)(sign | 0x7fc0);
    double a = fabs((double)x);
    if (isinf(a)) return (uint16_t)(sign | 0x7f80);
    if (a == 0.0) return sign;
    int e;
    frexp(a, &e);
    int ex = e - 1;
    if (ex < -126) ex = -126;
    double quantum = ldexp(1.0, ex - 7);   /* 8 significant bits */
    double r = nearbyint(a / quantum) * quantum;
    float rf = (float)r;                   /* exact, or +inf when r reaches 2^128 */
    return (uint16_t)(sign | (uint16_t)(bits_of(rf) >> 16));
}

void oracle_f32_to_f16_array(const float *x, uint16_t *out, int64_t n)
{ for (int64_t i = 0; i < n; ++i) out[i] = oracle_f32_to_f16(x[i]); }
void oracle_f32_to_bf16_array(const float *x, uint16_t *out, int64_t n)
{ for (int64_t i = 0; i < n; ++i) out[i] = oracle_f32_to_bf16(x[i]); }
void oracle_f16_to_f32_array(const uint16_t *x, float *out, int64_t n)
{ for (int64_t i = 0; i < n; ++i) out[i] = oracle_f16_to_f32(x[i]); }

static float widen(const void *buf, int dtype, int64_t i)
{
    if (dtype == ORC_FP32) return ((const float *)buf)[i];
    if (dtype == ORC_BF16) return oracle_bf16_to_f32(((const uint16_t *)buf)[i]);
    return oracle_f16_to_f32(((const uint16_t *)buf)[i]);
}

/* ------------------------------------------------------------------------ */
/* Overflow detection.  Dynamic loss scaling is the prior art the paper cites
 * in Sec. 2 (mixed-precision paragraph); the reading taken here: a step is
 * skipped when any stored gradient element of any tensor is +-inf or NaN.   */
/* ------------------------------------------------------------------------ */
int oracle_found_nonfinite(const void *g, int dtype, int64_t n)
{
    for (int64_t i = 0; i < n; ++i)
        if (!isfinite(widen(g, dtype, i))) return 1;
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Var[grad_l(t)] of Sec. 3.1 (the quantity smoothed by the variance EMA).
 * Reading: the population variance (divide by n) over the n elements of the
 * tensor at this step, of the unscaled gradient x_i = fp32(g_i) * inv_scale
 * (one fp32 multiply), two passes in double.                                */
/* ------------------------------------------------------------------------ */
void oracle_grad_stats(const void *g, int dtype, int64_t n, float inv_scale,
                       double *mean_out, double *var_out)
{
    double s = 0.0;
    for (int64_t i = 0; i < n; ++i) s += (double)(widen(g, dtype, i) * inv_scale);
    double mean = s / (double)n;
    double q = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double d = (double)(widen(g, dtype, i) * inv_scale) - mean;
        q += d * d;
    }
    *mean_out = mean;
    *var_out = q / (double)n;
}

/* v_l(t) = beta v_l(t-1) + (1 - beta) Var[grad_l(t)]   (Sec. 3.1, first equation).
 * Reading: v_l at the first applied step is that step's variance, so the
 * weights sum to one at every t.  Computed in double from the fp32-stored
 * previous value, stored as fp32.                                            */
float oracle_var_ema(float v_prev, double var, float beta, int first)
{
    if (first) return (float)var;
    return (float)((double)beta * (double)v_prev + (1.0 - (double)beta) * var);
}

/* ------------------------------------------------------------------------ */
/* Diagonal curvature signal ("sparse second-order signals", Sec. 3.2; the
 * abstract's "Hessian/Fisher sparsity patterns").  Reading: one Hutchinson
 * sample per element, u_i = z_i (Hz)_i / S for a Rademacher probe z, smoothed
 * by an EMA with factor beta_h; the first probe initialises h.  A non-finite
 * sample leaves h_i unchanged and raises the tensor's diagnostic flag.
 * fp32 throughout: two separately rounded multiplies, then
 * h = fma(beta_h, h, fp32((1 - beta_h) * u)).                                */
/* ------------------------------------------------------------------------ */
void oracle_curv_ema(const float *z, const float *hz, float *h, int64_t n,
                     float inv_scale, float beta_h, int first, uint32_t *nonfinite)
{
    const float omb = 1.0f - beta_h;
    for (int64_t i = 0; i < n; ++i) {
        float u = z[i] * hz[i];
        u = u * inv_scale;
        if (!isfinite(u)) { *nonfinite = 1; continue; }
        if (first) { h[i] = u; continue; }
        float p = omb * u;
        h[i] = fmaf(beta_h, h[i], p);
    }
}

/* Empirical-Fisher variant of the same signal ("Hessian or Fisher", Sec. 1 and
 * 3.2): the sample is the squared unscaled gradient, u_i = (g_i / S)^2, no
 * probe.  Same EMA, same non-finite rule (the square can overflow).
 * fp32: x = fp32(g_i) * inv_scale, u = x * x, h = fma(beta_h, h, fp32((1 - beta_h) * u)). */
void oracle_fisher_ema(const void *g, int g_dtype, float *h, int64_t n, float inv_scale,
                       float beta_h, int first, uint32_t *nonfinite)
{
    const float omb = 1.0f - beta_h;
    for (int64_t i = 0; i < n; ++i) {
        float x = widen(g, g_dtype, i) * inv_scale;
        float u = x * x;
        if (!isfinite(u)) { *nonfinite = 1; continue; }
        if (first) { h[i] = u; continue; }
        float p = omb * u;
        h[i] = fmaf(beta_h, h[i], p);
    }
}

/* ------------------------------------------------------------------------ */
/* Sparsification of the curvature ("top-k Hessian or Fisher entries", Sec. 1
 * and 3.2).  Plain definition by sorting:
 *   k = n - floor(n * s_ppm / 1e6), clamped to [1, n];
 *   theta = k-th largest of |h_i|;
 *   mask_i = (|h_i| >= theta) and (|h_i| > 0)   (ties kept, zeros never);
 *   nnz = popcount(mask);  lambda = largest masked |h_i| (0 if none).
 * Magnitudes are compared through their 31-bit patterns, which order finite
 * non-negative floats exactly.  Mask bit i%32 of word i/32.                  */
/* ------------------------------------------------------------------------ */
static int cmp_desc_u32(const void *a, const void *b)
{
    uint32_t x = *(const uint32_t *)a, y = *(const uint32_t *)b;
    return (x < y) - (x > y);
}

int64_t oracle_topk_count(int64_t n, uint32_t s_ppm)
{
    int64_t k = n - (int64_t)(((__int128)n * (int64_t)s_ppm) / 1000000);
    if (k < 1) k = 1;
    if (k > n) k = n;
    return k;
}

/* The same with the number of kept entries given directly (the paper's "top-k" with a fixed k,
 * Sec. 4.1: k = 5), clamped to [1, n]. */
void oracle_threshold_mask_k(const float *h, int64_t n, int64_t k, uint32_t *mask,
                             float *theta_out, uint32_t *nnz_out, float *lambda_out);

void oracle_threshold_mask(const float *h, int64_t n, uint32_t s_ppm, uint32_t *mask,
                           float *theta_out, uint32_t *nnz_out, float *lambda_out)
{
    oracle_threshold_mask_k(h, n, oracle_topk_count(n, s_ppm), mask, theta_out, nnz_out, lambda_out);
}

void oracle_threshold_mask_k(const float *h, int64_t n, int64_t k, uint32_t *mask,
                             float *theta_out, uint32_t *nnz_out, float *lambda_out)
{
    uint32_t *a = (uint32_t *)malloc((size_t)n * sizeof(uint32_t));
    for (int64_t i = 0; i < n; ++i) a[i] = bits_of(h[i]) & 0x7fffffffu;
    if (k < 1) k = 1;
    if (k > n) k = n;
    uint32_t *sorted = (uint32_t *)malloc((size_t)n * sizeof(uint32_t));
    memcpy(sorted, a, (size_t)n * sizeof(uint32_t));
    qsort(sorted, (size_t)n, sizeof(uint32_t), cmp_desc_u32);
    uint32_t theta = sorted[k - 1];
    free(sorted);
    int64_t words = (n + 31) / 32;
    memset(mask, 0, (size_t)words * sizeof(uint32_t));
    uint32_t nnz = 0, lam = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (a[i] >= theta && a[i] > 0) {
            mask[i >> 5] |= 1u << (i & 31);
            ++nnz;
            if (a[i] > lam) lam = a[i];
        }
    }
    free(a);
    *theta_out = float_of(theta);
    *nnz_out = nnz;
    *lambda_out = float_of(lam);
}

/* ------------------------------------------------------------------------ */
/* Precision rule of Sec. 3.1 (second equation):
 *   FP16 if v < tau_low;  BF16 if tau_low <= v < tau_high;  FP32 if v >= tau_high,
 * followed by the promotion of Sec. 3.2 ("Precision promotion"): a layer whose
 * curvature exceeds tau_curv moves one level up, FP16 -> BF16 -> FP32,
 * saturating at FP32.  Curvature is the magnitude lambda_l >= 0.               */
/* ------------------------------------------------------------------------ */
int oracle_precision_code(float v, float lambda, float tau_low, float tau_high, float tau_curv)
{
    int base = (v < tau_low) ? ORC_FP16 : (v < tau_high) ? ORC_BF16 : ORC_FP32;
    if (lambda > tau_curv && base < ORC_FP32) base += 1;
    return base;
}

/* eta_l = eta_0 / (1 + alpha * max_i lambda_i(H_l))   (Sec. 3.2, "Step size scaling").
 * fp32: one fma for the denominator, one correctly rounded division.          */
float oracle_eta(float lr, float alpha, float lambda)
{
    float den = fmaf(alpha, lambda, 1.0f);
    return lr / den;
}

/* ------------------------------------------------------------------------ */
/* Parameter update.  The paper states the base optimizer only for its FP32
 * baseline (Sec. 4.1: SGD with momentum 0.9, tuned weight decay); reading:
 * heavy-ball SGD with coupled L2 decay, the per-layer step size of Sec. 3.2
 * multiplying the momentum buffer.  Per element in fp32:
 *   theta = widen(stored parameter);  gt = fp32(g) * inv_scale;
 *   d = fma(wd, theta, gt);  m = fma(mu, m, d)  (m = d when no buffer);
 *   theta' = fma(-eta, m, theta);  store theta' in the layer's new precision,
 *   round to nearest even.
 * `param` holds n elements of the old dtype on entry and of the new dtype on
 * return (capacity 4n bytes).                                                */
/* ------------------------------------------------------------------------ */
void oracle_update(void *param, int prev_code, int new_code, const void *g, int grad_dtype,
                   float *m, int64_t n, float inv_scale, float wd, float mu, float eta)
{
    float *next = (float *)malloc((size_t)n * sizeof(float));
    const float neg_eta = -eta;
    for (int64_t i = 0; i < n; ++i) {
        float th = widen(param, prev_code, i);
        float gt = widen(g, grad_dtype, i) * inv_scale;
        float d = fmaf(wd, th, gt);
        float mm;
        if (m) { m[i] = fmaf(mu, m[i], d); mm = m[i]; } else { mm = d; }
        next[i] = fmaf(neg_eta, mm, th);
    }
    if (new_code == ORC_FP32) {
        memcpy(param, next, (size_t)n * sizeof(float));
    } else if (new_code == ORC_BF16) {
        uint16_t *p = (uint16_t *)param;
        for (int64_t i = 0; i < n; ++i) p[i] = oracle_f32_to_bf16(next[i]);
    } else {
        uint16_t *p = (uint16_t *)param;
        for (int64_t i = 0; i < n; ++i) p[i] = oracle_f32_to_f16(next[i]);
    }
    free(next);
}

/* ------------------------------------------------------------------------ */
/* Element-wise form of the step-size scaling (Sec. 3.2, fourth equation, applied
 * per entry of the sparsified curvature instead of once per layer):
 *   eta_i = eta_0 / (1 + alpha * a_i),   a_i = |h_i| if mask_i else 0,
 * so that the mask acts on the update; with h constant over a fully masked layer it
 * is the per-layer rule.  Everything else as in oracle_update.  fp32 per element:
 *   den = fma(alpha, a_i, 1);  eta_i = lr / den;  theta' = fma(-eta_i, m, theta).   */
/* ------------------------------------------------------------------------ */
void oracle_update_elementwise(void *param, int prev_code, int new_code, const void *g, int grad_dtype,
                               float *m, const float *h, const uint32_t *mask, int64_t n,
                               float inv_scale, float wd, float mu, float lr, float alpha)
{
    float *next = (float *)malloc((size_t)n * sizeof(float));
    for (int64_t i = 0; i < n; ++i) {
        float th = widen(param, prev_code, i);
        float gt = widen(g, grad_dtype, i) * inv_scale;
        float d = fmaf(wd, th, gt);
        float mm;
        if (m) { m[i] = fmaf(mu, m[i], d); mm = m[i]; } else { mm = d; }
        float a = ((mask[i >> 5] >> (i & 31)) & 1u) ? fabsf(h[i]) : 0.0f;
        float den = fmaf(alpha, a, 1.0f);
        float eta = lr / den;
        next[i] = fmaf(-eta, mm, th);
    }
    if (new_code == ORC_FP32) {
        memcpy(param, next, (size_t)n * sizeof(float));
    } else if (new_code == ORC_BF16) {
        uint16_t *p = (uint16_t *)param;
        for (int64_t i = 0; i < n; ++i) p[i] = oracle_f32_to_bf16(next[i]);
    } else {
        uint16_t *p = (uint16_t *)param;
        for (int64_t i = 0; i < n; ++i) p[i] = oracle_f32_to_f16(next[i]);
    }
    free(next);
}

/* ------------------------------------------------------------------------ */
/* Dynamic loss scaling (prior art cited in Sec. 2): after a skipped step the
 * scale is multiplied by `backoff` and the count of good steps restarts; after
 * `growth_interval` consecutive good steps it is multiplied by `growth`.      */
/* ------------------------------------------------------------------------ */
float oracle_loss_scale_next(float scale, int skipped, int32_t *good_steps,
                             float backoff, float growth, int32_t growth_interval)
{
    if (skipped) { *good_steps = 0; return scale * backoff; }
    *good_steps += 1;
    if (*good_steps >= growth_interval) { *good_steps = 0; return scale * growth; }
    return scale;
}

/* ------------------------------------------------------------------------ */
/* Memory-elastic batch rule (Sec. 3.3):
 *   B + delta_up   if MemUsage <  rho_low  * MemMax
 *   B - delta_down if MemUsage >  rho_high * MemMax
 *   B              otherwise,
 * strict inequalities as printed; result clamped to [b_min, b_max].          */
/* ------------------------------------------------------------------------ */
int32_t oracle_batch_next(int32_t batch, uint64_t mem_used, uint64_t mem_total,
                          double rho_low, double rho_high, int32_t delta_up,
                          int32_t delta_down, int32_t b_min, int32_t b_max)
{
    double used = (double)mem_used, total = (double)mem_total;
    int64_t b = batch;
    if (used < rho_low * total) b += delta_up;
    else if (used > rho_high * total) b -= delta_down;
    if (b < b_min) b = b_min;
    if (b > b_max) b = b_max;
    return (int32_t)b;
}

/* ------------------------------------------------------------------------ */
/* Power iteration of Sec. 3.2 (third equation) for the top-k eigenvalues, one
 * iteration on k supplied pairs (u_j, H u_j), j = 0..k-1, vector j stored at
 * offset j*n:
 *   rayleigh_j = u_j^T (H u_j) / u_j^T u_j                      (the printed quotient)
 *   resid_j    = || H u_j - rayleigh_j u_j || / || u_j ||        (convergence measure)
 *   hnorm_j    = || H u_j ||
 *   v_j = H u_j - sum_{i<j} (q_i^T v_j) q_i     in order i = 0..j-1 (modified Gram-Schmidt)
 *   q_j = v_j / || v_j ||,   u_j <- q_j
 * For k = 1 this is the printed iteration u <- H u / ||H u|| literally; for k > 1 the earlier
 * directions are projected out before normalising, which is what makes vector j converge to
 * the j-th eigenvector (the paper asks for the top k but prints the single-vector form only).
 * A vector whose remainder is numerically nothing, ||v_j||^2 <= 1e-12 ||H u_j||^2, has no
 * direction left: q_j = 0 and bit j of *deficient is set.  A zero iterate (u_j^T u_j = 0) has
 * no quotient: rayleigh_j = resid_j = 0.
 * Everything in double; the new vectors are rounded to fp32 once.            */
/* ------------------------------------------------------------------------ */
void oracle_power_step(const float *u, const float *hu, float *u_next, int64_t n, int32_t k,
                       double *rayleigh, double *resid, double *hnorm, uint32_t *deficient)
{
    double *q = (double *)malloc((size_t)k * (size_t)n * sizeof(double));
    uint32_t def = 0;
    for (int32_t j = 0; j < k; ++j) {
        const float *uj = u + (int64_t)j * n, *wj = hu + (int64_t)j * n;
        double uw = 0.0, uu = 0.0, ww = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            uw += (double)uj[i] * (double)wj[i];
            uu += (double)uj[i] * (double)uj[i];
            ww += (double)wj[i] * (double)wj[i];
        }
        double lam = 0.0, rr = 0.0;
        if (uu > 0.0) {
            lam = uw / uu;
            for (int64_t i = 0; i < n; ++i) {
                double d = (double)wj[i] - lam * (double)uj[i];
                rr += d * d;
            }
            rr = sqrt(rr) / sqrt(uu);
        }
        rayleigh[j] = lam;
        resid[j] = rr;
        hnorm[j] = sqrt(ww);
        double *v = q + (int64_t)j * n;
        for (int64_t i = 0; i < n; ++i) v[i] = (double)wj[i];
        for (int32_t p = 0; p < j; ++p) {
            const double *qp = q + (int64_t)p * n;
            double dot = 0.0;
            for (int64_t i = 0; i < n; ++i) dot += qp[i] * v[i];
            for (int64_t i = 0; i < n; ++i) v[i] -= dot * qp[i];
        }
        double vv = 0.0;
        for (int64_t i = 0; i < n; ++i) vv += v[i] * v[i];
        if (vv <= 1e-12 * ww) {
            def |= 1u << j;
            for (int64_t i = 0; i < n; ++i) v[i] = 0.0;
        } else {
            double nv = sqrt(vv);
            for (int64_t i = 0; i < n; ++i) v[i] = v[i] / nv;
        }
        for (int64_t i = 0; i < n; ++i) u_next[(int64_t)j * n + i] = (float)v[i];
    }
    *deficient = def;
    free(q);
}
