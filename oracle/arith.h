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

/* GELU(x) = x*Phi(x) = max(x,0) - a*Phi(-a), a = |x|.  The even remainder
 * a*Phi(-a) is a degree-14 polynomial in t = 2a/5.5 - 1 on a in [0,5.5] and is
 * held at its (1e-7) end value beyond. */
static inline float orc_gelu_pinned(float x)
{
    static const float c[15] = {
        0x1.0c8760p-7f, -0x1.f0423cp-5f, 0x1.8794f2p-3f, -0x1.3c122ap-2f, 0x1.711f2ap-3f,
        0x1.0a7892p-2f, -0x1.46f9bap-1f, 0x1.d7ab76p-2f, 0x1.88e9f6p-3f, -0x1.18547cp-1f,
        0x1.7cae60p-3f, 0x1.e1f934p-3f, -0x1.3d2fc0p-3f, -0x1.42e9b8p-5f, 0x1.280820p-5f };
    float a = fminf(fabsf(x), 5.5f);
    float t = fmaf(a, 0x1.745d18p-2f, -1.0f);
    float h = c[14];
    for (int k = 13; k >= 0; --k) h = fmaf(h, t, c[k]);
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
