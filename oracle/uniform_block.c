/*
 * TEST INFRASTRUCTURE ONLY -- a uniform-precision quantized Swin block written
 * separately from the two-branch oracle, as its special-case pin: with every
 * window in one branch the Two-Branch Swin Block must be this block (paper
 * Sec. 3.1: the computation flow is unchanged and the worst case is bounded by
 * the low-precision branch).  No scoring, no gather list, natural window order.
 * It materialises each step of the classic shifted-window pipeline instead of
 * indexing through it: pad -> roll -> partition -> attention with a mask built
 * from region labels -> reverse -> roll back -> crop.
 * Only the scalar primitives of arith.h are common with the oracle.
 */
#include <stdlib.h>
#include <string.h>
#include "arith.h"

typedef struct { float scale; int32_t zero_point; } ub_qparam;
typedef struct {
    int32_t B, H, W, C, window, shift, heads, mlp_ratio, bits;
    float ln_eps;
    const float *ln1_gamma, *ln1_beta, *ln2_gamma, *ln2_beta, *b_qkv, *b_proj, *b_fc1, *b_fc2;
    ub_qparam a_qkv_in, a_q, a_k, a_v, a_p, a_proj_in, a_fc1_in, a_fc2_in;
    const int8_t *w_qkv, *w_proj, *w_fc1, *w_fc2;
    const float *s_qkv, *s_proj, *s_fc1, *s_fc2, *rel_pos_bias;
} ub_params;

/* out[t,n] = sum_k (a[t,k]-z) * W[n,k], weights-outer loop order */
static void lin(const int32_t *a, int T, int K, const int8_t *W, int N, int z, int32_t *out)
{
    memset(out, 0, sizeof(int32_t) * T * N);
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k) {
            int wv = W[(size_t)n * K + k];
            for (int t = 0; t < T; ++t) out[t * N + n] += (a[t * K + k] - z) * wv;
        }
}

static int region(int p, int n, int ws, int s)      /* label of a rolled-frame coordinate */
{
    if (p < n - ws) return 0;
    if (p < n - s) return 1;
    return 2;
}

int ub_forward(const ub_params *P, const float *x, float *y)
{
    const int ws = P->window, s = P->shift, C = P->C, T = ws * ws, nh = P->heads, hd = C / nh, F = C * P->mlp_ratio;
    const int Hp = (P->H + ws - 1) / ws * ws, Wp = (P->W + ws - 1) / ws * ws, bits = P->bits;
    float *pad = (float *)malloc(sizeof(float) * Hp * Wp * C), *rol = (float *)malloc(sizeof(float) * Hp * Wp * C);
    float *outr = (float *)malloc(sizeof(float) * Hp * Wp * C);
    unsigned char *okp = (unsigned char *)malloc((size_t)Hp * Wp), *okr = (unsigned char *)malloc((size_t)Hp * Wp);
    int32_t *a = (int32_t *)malloc(sizeof(int32_t) * T * C), *acc = (int32_t *)malloc(sizeof(int32_t) * T * F);
    int32_t *qkv = (int32_t *)malloc(sizeof(int32_t) * T * 3 * C), *ao = (int32_t *)malloc(sizeof(int32_t) * T * C);
    int32_t *g = (int32_t *)malloc(sizeof(int32_t) * T * F);
    float *sc = (float *)malloc(sizeof(float) * T * C), *hr = (float *)malloc(sizeof(float) * T * C), *ln = (float *)malloc(sizeof(float) * C);
    float *lg = (float *)malloc(sizeof(float) * T), *ev = (float *)malloc(sizeof(float) * T);
    int32_t *pc = (int32_t *)malloc(sizeof(int32_t) * T);
    for (int b = 0; b < P->B; ++b) {
        /* pad */
        memset(pad, 0, sizeof(float) * Hp * Wp * C); memset(okp, 0, (size_t)Hp * Wp);
        for (int r = 0; r < P->H; ++r)
            for (int c = 0; c < P->W; ++c) {
                memcpy(pad + ((size_t)r * Wp + c) * C, x + (((size_t)b * P->H + r) * P->W + c) * C, sizeof(float) * C);
                okp[r * Wp + c] = 1;
            }
        /* roll by -s: element at (r,c) moves to (r-s, c-s) */
        for (int r = 0; r < Hp; ++r)
            for (int c = 0; c < Wp; ++c) {
                int rr = ((r - s) % Hp + Hp) % Hp, cc = ((c - s) % Wp + Wp) % Wp;
                memcpy(rol + ((size_t)rr * Wp + cc) * C, pad + ((size_t)r * Wp + c) * C, sizeof(float) * C);
                okr[rr * Wp + cc] = okp[r * Wp + c];
            }
        for (int wr = 0; wr < Hp / ws; ++wr)
            for (int wc = 0; wc < Wp / ws; ++wc) {
                /* partition + LN1 + quantize */
                for (int t = 0; t < T; ++t) {
                    int r = wr * ws + t / ws, c = wc * ws + t % ws;
                    const float *px = rol + ((size_t)r * Wp + c) * C;
                    if (okr[r * Wp + c]) { orc_layernorm(px, C, P->ln1_gamma, P->ln1_beta, P->ln_eps, ln); memcpy(sc + t * C, px, sizeof(float) * C); }
                    else { memset(ln, 0, sizeof(float) * C); memset(sc + t * C, 0, sizeof(float) * C); }
                    for (int k = 0; k < C; ++k) a[t * C + k] = orc_q(ln[k], 1.0f / P->a_qkv_in.scale, P->a_qkv_in.zero_point, bits);
                }
                lin(a, T, C, P->w_qkv, 3 * C, P->a_qkv_in.zero_point, acc);
                for (int t = 0; t < T; ++t)
                    for (int n = 0; n < 3 * C; ++n) {
                        ub_qparam qp = n / C == 0 ? P->a_q : (n / C == 1 ? P->a_k : P->a_v);
                        float f = fmaf((float)acc[t * 3 * C + n], P->a_qkv_in.scale * P->s_qkv[n], P->b_qkv[n]);
                        qkv[t * 3 * C + n] = orc_q(f, 1.0f / qp.scale, qp.zero_point, bits);
                    }
                float m2 = ((P->a_q.scale * P->a_k.scale) * (float)(1.0 / sqrt((double)hd))) * 0x1.715476p+0f;
                for (int h = 0; h < nh; ++h)
                    for (int i = 0; i < T; ++i) {
                        int li = region(wr * ws + i / ws, Hp, ws, s) * 3 + region(wc * ws + i % ws, Wp, ws, s);
                        float mx = -INFINITY;
                        for (int j = 0; j < T; ++j) {
                            int lj = region(wr * ws + j / ws, Hp, ws, s) * 3 + region(wc * ws + j % ws, Wp, ws, s);
                            int32_t d = 0;
                            for (int k = 0; k < hd; ++k) d += qkv[i * 3 * C + h * hd + k] * qkv[j * 3 * C + C + h * hd + k];
                            float bias = P->rel_pos_bias[((size_t)h * T + i) * T + j];
                            if (s > 0 && li != lj) bias = bias + -100.0f;
                            lg[j] = fmaf((float)d, m2, bias * 0x1.715476p+0f);
                            mx = fmaxf(mx, lg[j]);
                        }
                        double den = 0.0;
                        for (int j = 0; j < T; ++j) { ev[j] = orc_exp2_pinned(lg[j] - mx); den += (double)ev[j]; }
                        float rden = 1.0f / (float)den;
                        for (int j = 0; j < T; ++j) pc[j] = orc_q(ev[j] * rden, 1.0f / P->a_p.scale, P->a_p.zero_point, bits);
                        for (int k = 0; k < hd; ++k) {
                            int32_t o = 0;
                            for (int j = 0; j < T; ++j) o += (pc[j] - P->a_p.zero_point) * qkv[j * 3 * C + 2 * C + h * hd + k];
                            ao[i * C + h * hd + k] = orc_q((float)o * (P->a_p.scale * P->a_v.scale), 1.0f / P->a_proj_in.scale, P->a_proj_in.zero_point, bits);
                        }
                    }
                lin(ao, T, C, P->w_proj, C, P->a_proj_in.zero_point, acc);
                for (int i = 0; i < T * C; ++i)
                    hr[i] = fmaf((float)acc[i], P->a_proj_in.scale * P->s_proj[i % C], P->b_proj[i % C]) + sc[i];
                for (int t = 0; t < T; ++t) {
                    orc_layernorm(hr + t * C, C, P->ln2_gamma, P->ln2_beta, P->ln_eps, ln);
                    for (int k = 0; k < C; ++k) a[t * C + k] = orc_q(ln[k], 1.0f / P->a_fc1_in.scale, P->a_fc1_in.zero_point, bits);
                }
                lin(a, T, C, P->w_fc1, F, P->a_fc1_in.zero_point, acc);
                for (int i = 0; i < T * F; ++i) {
                    float f = fmaf((float)acc[i], P->a_fc1_in.scale * P->s_fc1[i % F], P->b_fc1[i % F]);
                    g[i] = orc_q(orc_gelu_pinned(f), 1.0f / P->a_fc2_in.scale, P->a_fc2_in.zero_point, bits);
                }
                lin(g, T, F, P->w_fc2, C, P->a_fc2_in.zero_point, acc);
                /* window reverse into the rolled frame */
                for (int t = 0; t < T; ++t)
                    for (int n = 0; n < C; ++n)
                        outr[((size_t)(wr * ws + t / ws) * Wp + wc * ws + t % ws) * C + n] =
                            fmaf((float)acc[t * C + n], P->a_fc2_in.scale * P->s_fc2[n], P->b_fc2[n]) + hr[t * C + n];
            }
        /* roll back by +s and crop */
        for (int r = 0; r < P->H; ++r)
            for (int c = 0; c < P->W; ++c) {
                int rr = ((r - s) % Hp + Hp) % Hp, cc = ((c - s) % Wp + Wp) % Wp;
                memcpy(y + (((size_t)b * P->H + r) * P->W + c) * C, outr + ((size_t)rr * Wp + cc) * C, sizeof(float) * C);
            }
    }
    free(pad); free(rol); free(outr); free(okp); free(okr); free(a); free(acc); free(qkv); free(ao); free(g);
    free(sc); free(hr); free(ln); free(lg); free(ev); free(pc);
    return 0;
}
