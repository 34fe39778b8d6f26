/*
 * CPU oracle for stacks of non-convolution CNN layers -- TEST INFRASTRUCTURE.
 *
 * This file is the slow, plain, layer-by-layer ("breadth-first", Section 3.1
 * and Figure 2 of the BrainSlug paper) definition of every layer the fused GPU
 * path supports.  It exists to check that path; it is never part of it.  Only
 * the tests, the smoke check and the benchmark's CPU-baseline leg may load it.
 * It shares no code with the HIP library.
 *
 * Each function computes one whole layer over one whole NCHW float32 tensor
 * with scalar loops over (n, c, oh, ow).  Nothing is tiled, fused or reordered.
 *
 * Precision.  The paper computes in 32-bit float (Section 5.1) and promises
 * that the depth-first order gives the same numerical results (Sections 1, 3
 * and 6).  The layers are therefore evaluated in float32 with one fixed
 * operation order each, stated at the function; the float64 "textbook"
 * BatchNorm is kept beside it as a cross-check of the folded form.
 *
 * The one parallel construct is an OpenMP "parallel for" over the N*C planes
 * (the axis the paper's own CPU path parallelises over, Section 5.2); planes
 * are independent in every layer, so the result does not depend on it.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

#define BSO_API __attribute__((visibility("default")))

/* ------------------------------------------------------------------ */
/* bfloat16 rounding: round-to-nearest-even of a float32 to the 8-bit  */
/* mantissa format, returned as float32.  NaN stays NaN.               */
/* ------------------------------------------------------------------ */
static float round_to_bf16(float v)
{
    uint32_t u;
    memcpy(&u, &v, 4);
    if ((u & 0x7f800000u) == 0x7f800000u) { /* inf or nan: truncate, keep nan a nan */
        if (u & 0x007fffffu) u |= 0x00400000u;
        u &= 0xffff0000u;
    } else {
        uint32_t lsb = (u >> 16) & 1u;
        u += 0x7fffu + lsb;
        u &= 0xffff0000u;
    }
    memcpy(&v, &u, 4);
    return v;
}

BSO_API void bso_round_bf16(float *x, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) x[i] = round_to_bf16(x[i]);
}

/* ------------------------------------------------------------------ */
/* IEEE binary16 rounding: round-to-nearest-even of a float32 to the   */
/* half-precision format (5 exponent bits, 10 mantissa bits, gradual   */
/* underflow, overflow to infinity), returned as float32.              */
/* The grid of representable values around v has spacing               */
/* 2^(e-10) for |v| in [2^e, 2^(e+1)), e >= -14, and 2^-24 below 2^-14;*/
/* scaling by that spacing makes the rounding an integer rounding.     */
/* ------------------------------------------------------------------ */
static float round_to_f16(float v)
{
    if (v != v || v == INFINITY || v == -INFINITY || v == 0.0f) return v;
    int e;
    (void)frexpf(v, &e); /* |v| = m * 2^e, m in [0.5, 1) : |v| in [2^(e-1), 2^e) */
    int ulp_exp = (e - 1) - 10;
    if (ulp_exp < -24) ulp_exp = -24;           /* subnormal range: fixed spacing */
    const float scaled = ldexpf(v, -ulp_exp);   /* exact: a power-of-two scaling */
    const float r = nearbyintf(scaled);         /* ties to even in the default rounding mode */
    const float y = ldexpf(r, ulp_exp);
    if (y > 65504.0f) return INFINITY;          /* beyond the largest half value */
    if (y < -65504.0f) return -INFINITY;
    return y;
}

BSO_API void bso_round_f16(float *x, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) x[i] = round_to_f16(x[i]);
}

/* ------------------------------------------------------------------ */
/* BatchNorm, inference mode (the "normalization" element-wise layer   */
/* of Section 2).  Folded form: per channel                            */
/*     scale = gamma / sqrt(var + eps)                                 */
/*     shift = beta - mean * scale                                     */
/* both evaluated in float64 and rounded once to float32; then         */
/*     y = fma(x, scale, shift)   (one float32 fused multiply-add).    */
/* ------------------------------------------------------------------ */
BSO_API void bso_bn_fold(const float *gamma, const float *beta, const float *mean,
                         const float *var, double eps, int64_t C, float *scale, float *shift)
{
    for (int64_t c = 0; c < C; ++c) {
        double inv_std = 1.0 / sqrt((double)var[c] + eps);
        double s = (double)gamma[c] * inv_std;
        scale[c] = (float)s;
        shift[c] = (float)((double)beta[c] - (double)mean[c] * s);
    }
}

BSO_API void bso_batchnorm(const float *x, float *y, int64_t N, int64_t C, int64_t H, int64_t W,
                           const float *scale, const float *shift)
{
    const int64_t hw = H * W;
#pragma omp parallel for schedule(static)
    for (int64_t plane = 0; plane < N * C; ++plane) {
        const int64_t c = plane % C;
        const float *xp = x + plane * hw;
        float *yp = y + plane * hw;
        for (int64_t i = 0; i < hw; ++i) yp[i] = fmaf(xp[i], scale[c], shift[c]);
    }
}

/* Textbook BatchNorm in float64, unfolded: (x - mean) / sqrt(var + eps) * gamma + beta. */
BSO_API void bso_batchnorm_textbook_f64(const float *x, double *y, int64_t N, int64_t C, int64_t H,
                                        int64_t W, const float *gamma, const float *beta,
                                        const float *mean, const float *var, double eps)
{
    const int64_t hw = H * W;
    for (int64_t plane = 0; plane < N * C; ++plane) {
        const int64_t c = plane % C;
        for (int64_t i = 0; i < hw; ++i) {
            double v = (double)x[plane * hw + i];
            y[plane * hw + i] =
                (v - (double)mean[c]) / sqrt((double)var[c] + eps) * (double)gamma[c] + (double)beta[c];
        }
    }
}

/* ReLU, f(x) = max(0, x) (Section 2): positive values pass, everything else
 * (negative, -0, NaN) becomes +0. */
BSO_API void bso_relu(const float *x, float *y, int64_t n)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) y[i] = (x[i] > 0.0f) ? x[i] : 0.0f;
}

/* Leaky ReLU (one of the further element-wise activations Section 2 alludes to with
 * "BatchNorm, ReLU, ..."): positive values pass, everything else is multiplied by the
 * slope (one float32 rounding). */
BSO_API void bso_leaky_relu(const float *x, float *y, int64_t n, float slope)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) y[i] = (x[i] > 0.0f) ? x[i] : x[i] * slope;
}

/* Clamp to [lo, hi] (ReLU6 = clamp to [0, 6]; "hard tanh"): first raised to lo -- anything
 * not above lo, NaN included, becomes lo -- then lowered to hi. */
BSO_API void bso_clamp(const float *x, float *y, int64_t n, float lo, float hi)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        const float t = (x[i] > lo) ? x[i] : lo;
        y[i] = (t < hi) ? t : hi;
    }
}

/* Residual add: y = a + r, one float32 rounding. */
BSO_API void bso_add(const float *a, const float *r, float *y, int64_t n)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) y[i] = a[i] + r[i];
}

/* Pooling output size.  Floor mode: the windows that fit the padded input.  Ceil mode (the
 * rule of the framework the paper's front-end targets; the paper itself is silent): one more
 * window if the last fitting one leaves cells uncovered, unless that window would start
 * beyond the input and its leading padding. */
BSO_API int64_t bso_pool_out(int64_t in, int64_t k, int64_t s, int64_t p, int ceil_mode)
{
    if (!ceil_mode) return (in + 2 * p - k) / s + 1;
    int64_t o = (in + 2 * p - k + s - 1) / s + 1;
    if ((o - 1) * s >= in + p) --o;
    return o;
}

/* ------------------------------------------------------------------ */
/* Max pooling over fixed windows (Section 2, Figure 1b).  Padding     */
/* cells are outside the tensor and never candidates.  The window is   */
/* scanned row-major; the first maximum wins (strict '>').  idx (may   */
/* be NULL) receives ih*W+iw of the winner in the layer's input plane. */
/* ------------------------------------------------------------------ */
BSO_API void bso_maxpool(const float *x, float *y, int32_t *idx, int64_t N, int64_t C, int64_t H,
                         int64_t W, int64_t kh, int64_t kw, int64_t sh, int64_t sw, int64_t ph,
                         int64_t pw, int ceil_mode)
{
    const int64_t Ho = bso_pool_out(H, kh, sh, ph, ceil_mode), Wo = bso_pool_out(W, kw, sw, pw, ceil_mode);
#pragma omp parallel for schedule(static)
    for (int64_t plane = 0; plane < N * C; ++plane) {
        const float *xp = x + plane * H * W;
        for (int64_t oh = 0; oh < Ho; ++oh) {
            for (int64_t ow = 0; ow < Wo; ++ow) {
                float best = -INFINITY;
                int64_t best_i = -1;
                for (int64_t dh = 0; dh < kh; ++dh) {
                    const int64_t ih = oh * sh - ph + dh;
                    if (ih < 0 || ih >= H) continue;
                    for (int64_t dw = 0; dw < kw; ++dw) {
                        const int64_t iw = ow * sw - pw + dw;
                        if (iw < 0 || iw >= W) continue;
                        const float v = xp[ih * W + iw];
                        if (best_i < 0) best_i = ih * W + iw; /* first in-range cell */
                        if (v > best) { best = v; best_i = ih * W + iw; }
                    }
                }
                y[(plane * Ho + oh) * Wo + ow] = best;
                if (idx) idx[(plane * Ho + oh) * Wo + ow] = (int32_t)best_i;
            }
        }
    }
}

/* ------------------------------------------------------------------ */
/* Average pooling = window sum ("AvgPooling") followed by the         */
/* element-wise "AvgNormalization" (Listing 2).  The sum runs over the */
/* in-range cells in row-major order starting from +0; padding cells   */
/* add nothing.  The normalisation multiplies by the float32           */
/* reciprocal of the divisor: with count_include_pad the number of     */
/* window cells inside the padded input (kh*kw for every floor-mode    */
/* window; fewer for a ceil-mode window that overhangs the padding),   */
/* else the number of in-range cells.                                  */
/* ------------------------------------------------------------------ */
BSO_API void bso_avgpool(const float *x, float *y, int64_t N, int64_t C, int64_t H, int64_t W,
                         int64_t kh, int64_t kw, int64_t sh, int64_t sw, int64_t ph, int64_t pw,
                         int count_include_pad, int ceil_mode)
{
    const int64_t Ho = bso_pool_out(H, kh, sh, ph, ceil_mode), Wo = bso_pool_out(W, kw, sw, pw, ceil_mode);
#pragma omp parallel for schedule(static)
    for (int64_t plane = 0; plane < N * C; ++plane) {
        const float *xp = x + plane * H * W;
        for (int64_t oh = 0; oh < Ho; ++oh) {
            for (int64_t ow = 0; ow < Wo; ++ow) {
                float sum = 0.0f;
                int64_t cells = 0;
                for (int64_t dh = 0; dh < kh; ++dh) {
                    const int64_t ih = oh * sh - ph + dh;
                    if (ih < 0 || ih >= H) continue;
                    for (int64_t dw = 0; dw < kw; ++dw) {
                        const int64_t iw = ow * sw - pw + dw;
                        if (iw < 0 || iw >= W) continue;
                        sum = sum + xp[ih * W + iw];
                        ++cells;
                    }
                }
                const int64_t h0 = oh * sh - ph, w0 = ow * sw - pw;
                const int64_t hp = (h0 + kh < H + ph ? h0 + kh : H + ph) - h0;  /* rows inside the padded input */
                const int64_t wp = (w0 + kw < W + pw ? w0 + kw : W + pw) - w0;
                const float inv = 1.0f / (float)(count_include_pad ? hp * wp : cells);
                y[(plane * Ho + oh) * Wo + ow] = sum * inv;
            }
        }
    }
}
