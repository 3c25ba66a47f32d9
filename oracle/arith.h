/*
 * TEST INFRASTRUCTURE ONLY -- CPU oracle for the MixA-Q Two-Branch Swin Block.
 * Nothing on the product path may include, link or call this file.
 *
 * Scalar arithmetic primitives shared by the oracle's translation units.  The
 * paper (Sec. 3.2, "Two-Branch Swin Block") fixes the block's structure only:
 * duplicated LayerNorms, shared weights, per-branch step sizes and zero points.
 * It is silent on the integer-inference arithmetic, so every float operation
 * that decides an integer code is pinned here as an explicit IEEE-754 binary32
 * sequence (compile with -ffp-contract=off; fused multiply-adds appear only
 * where fmaf() is written).  Reductions that feed a code are accumulated in
 * binary64 and rounded once.
 */
#ifndef MIXAQ_ORACLE_ARITH_H
#define MIXAQ_ORACLE_ARITH_H
#include <math.h>
#include <stdint.h>

/* Uniform affine quantizer, x_hat = scale*(q - zero_point)  (Sec. 3.2 keeps one
 * step size and zero point per branch).  q = clamp(round(v*inv_s + z)), rounding
 * half-to-even, evaluated exactly: the product of two binary32 numbers fits
 * binary64, and the integer zero point is added to its integer part so that no
 * bit is lost before the rounding decision. */
static inline int32_t orc_q(float v, float inv_s, int32_t z, int bits)
{
    const double lo = -(double)(1 << (bits - 1)), hi = (double)((1 << (bits - 1)) - 1);
    double p = (double)v * (double)inv_s;
    if (!(fabs(p) < 1e9)) return p > 0 ? (int32_t)hi : (int32_t)lo;
    double fl = floor(p), fr = p - fl;              /* exact, 0 <= fr < 1 */
    double n = fl + (double)z;                      /* exact integer */
    if (fr > 0.5 || (fr == 0.5 && fmod(n, 2.0) != 0.0)) n += 1.0;
    if (n < lo) n = lo;
    if (n > hi) n = hi;
    return (int32_t)n;
}

/* 2^y for y <= 0: clamp at -100, split into integer and fraction in [-1/2,1/2],
 * degree-5 polynomial for the fraction, exact scaling by the power of two. */
static inline float orc_exp2_pinned(float y)
{
    y = fmaxf(y, -100.0f);
    float n = rintf(y);
    float r = y - n;
    float p = 0x1.5f48c8p-10f;
    p = fmaf(p, r, 0x1.3d107cp-7f);
    p = fmaf(p, r, 0x1.c6aeccp-5f);
    p = fmaf(p, r, 0x1.ebf906p-3f);
    p = fmaf(p, r, 0x1.62e430p-1f);
    p = fmaf(p, r, 0x1.000002p+0f);
    return ldexpf(p, (int)n);
}

/* GELU in the erf form, GELU(x) = x*Phi(x) = max(x,0) - H(|x|) with the even
 * remainder H(a) = a*Phi(-a) = (a/2)*erfc(a/sqrt 2).  H is pinned as a piecewise
 * cubic: [0,6) is cut into 96 intervals of width 1/16; on interval i the cubic in
 * d = 16a - i interpolates H at the four points a = (3i+j)/48, j = 0..3 (both
 * ends and the thirds), its coefficients computed in binary64 and rounded to
 * binary32; beyond a = 6 the argument is held at the end of the last interval
 * (H(6) < 1e-8).  The table is filled when the library is loaded. */
#define ORC_GELU_INTERVALS 96
static float orc_gelu_tab[ORC_GELU_INTERVALS][4];
static inline double orc_gelu_remainder(double a) { return (0.5 * a) * erfc(a * 0.70710678118654752440); }
__attribute__((constructor)) static void orc_gelu_fill_table(void)
{
    for (int i = 0; i < ORC_GELU_INTERVALS; ++i) {
        double y[4];
        for (int j = 0; j < 4; ++j) y[j] = orc_gelu_remainder((double)(3 * i + j) / 48.0);
        orc_gelu_tab[i][0] = (float)y[0];
        orc_gelu_tab[i][1] = (float)((-11.0 * y[0] + 18.0 * y[1] - 9.0 * y[2] + 2.0 * y[3]) * 0.5);
        orc_gelu_tab[i][2] = (float)((18.0 * y[0] - 45.0 * y[1] + 36.0 * y[2] - 9.0 * y[3]) * 0.5);
        orc_gelu_tab[i][3] = (float)((-9.0 * y[0] + 27.0 * y[1] - 27.0 * y[2] + 9.0 * y[3]) * 0.5);
    }
}
static inline float orc_gelu_pinned(float x)
{
    float u = fminf(fabsf(x) * 16.0f, 0x1.7ffffep+6f);  /* largest binary32 below 96 */
    float fl = floorf(u);
    float d = u - fl;                                   /* exact */
    const float *c = orc_gelu_tab[(int)fl];
    float h = fmaf(c[3], d, c[2]);
    h = fmaf(h, d, c[1]);
    h = fmaf(h, d, c[0]);
    return fmaxf(x, 0.0f) - h;
}

/* LayerNorm of one token (Sec. 3.2: one LayerNorm per branch).  Mean and
 * population variance are accumulated in binary64 and rounded once. */
static inline void orc_layernorm(const float *x, int C, const float *gamma, const float *beta,
                                 float eps, float *y)
{
    double s = 0.0;
    for (int c = 0; c < C; ++c) s += (double)x[c];
    float mean = (float)(s / (double)C);
    double v = 0.0;
    for (int c = 0; c < C; ++c) { double dlt = (double)x[c] - (double)mean; v += dlt * dlt; }
    float var = (float)(v / (double)C);
    float rstd = 1.0f / sqrtf(var + eps);
    for (int c = 0; c < C; ++c) y[c] = fmaf((x[c] - mean) * rstd, gamma[c], beta[c]);
}
#endif
