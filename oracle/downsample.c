/*
 * TEST INFRASTRUCTURE ONLY -- CPU oracle for the layers BETWEEN the stages of a
 * Swin backbone, needed to run the four stages of a backbone as one chain.
 * Nothing on the product path may include, link or call this file.
 *
 * The paper keeps these layers outside MixA-Q: its cost model lists them as the
 * layers whose computation the method cannot save (appendix on equivalent
 * activation bits, the constant term beside the per-pair GMACs).  Reading used
 * here: each is ONE uniformly quantized linear layer at a single activation bit
 * width (no windows, no branches) with the arithmetic of the block's linears:
 *
 *   kind 0, patch embedding (Swin: a PxP, stride-P projection of the image, then a
 *     LayerNorm): token (i,j) of the output takes the P*P*Cin values of its patch
 *     in the order (row in patch, column in patch, channel); values outside the
 *     image are 0; v -> codes with (a_in, act_bits); acc = sum_k code*W[n][k];
 *     f = fma(f32(acc - z*colsum[n]), a_in.scale*s_w[n], bias[n]); out = LN(f).
 *   kind 1, patch merging (Swin: the 2x2 neighbours (0,0), (1,0), (0,1), (1,1)
 *     [row offset, column offset] concatenated along the channels, LayerNorm over
 *     the 4C values, linear 4C -> N without bias): positions outside the map are
 *     0 BEFORE the LayerNorm; codes, acc and f as above (bias may be NULL = 0).
 *
 * Layouts: x [B,H,W,Cin] float channels last; out [B,Ho,Wo,N]; W row-major
 * [N][K] int8 codes with per-output-channel scales s_w.  Optional taps: codes
 * [tokens][K] and acc [tokens][N] (acc is the zero-point corrected sum).
 *
 * Parity status: every step is pinned by tests against numpy: gather order
 * (slicing), codes (patch embedding: exact rational quantization of every
 * value; patch merging: within half a step of a float64 LayerNorm), integer
 * sums (int64 matmul), output (float64 dequantization and LayerNorm within
 * binary32 rounding).  The paper prints no worked example, so no stored
 * end-to-end value exists.
 */
#include <stdlib.h>
#include <string.h>
#include "arith.h"

typedef struct { float scale; int32_t zero_point; } ods_qparam;

typedef struct {
    int32_t kind;                    /* 0 patch embedding, 1 patch merging */
    int32_t B, H, W, C_in;           /* input map / image */
    int32_t patch;                   /* kind 0: P (4); kind 1: ignored (2) */
    int32_t N;                       /* output channels */
    int32_t act_bits, weight_bits;
    float   ln_eps;
} ods_desc;

typedef struct {
    const int8_t *w;                 /* [N][K] */
    const float  *s_w;               /* [N] */
    const float  *bias;              /* [N] or NULL */
    const float  *ln_gamma, *ln_beta;/* kind 0: [N] (after the linear); kind 1: [K] (before it) */
    ods_qparam a_in;
} ods_params;

enum { ODS_OK = 0, ODS_E_NULL = -1, ODS_E_SHAPE = -2, ODS_E_BITS = -3 };

static int ods_geometry(const ods_desc *d, int *P, int *K, int *Ho, int *Wo)
{
    if (d->kind != 0 && d->kind != 1) return ODS_E_SHAPE;
    if (d->B < 1 || d->H < 1 || d->W < 1 || d->C_in < 1 || d->N < 1) return ODS_E_SHAPE;
    *P = d->kind == 0 ? d->patch : 2;
    if (*P < 1) return ODS_E_SHAPE;
    *K = *P * *P * d->C_in;
    *Ho = (d->H + *P - 1) / *P;
    *Wo = (d->W + *P - 1) / *P;
    return ODS_OK;
}

int orc_downsample_out_shape(const ods_desc *d, int32_t *Ho, int32_t *Wo, int32_t *K)
{
    if (!d || !Ho || !Wo || !K) return ODS_E_NULL;
    int P, k, ho, wo, rc = ods_geometry(d, &P, &k, &ho, &wo);
    if (rc) return rc;
    *Ho = ho; *Wo = wo; *K = k;
    return ODS_OK;
}

/* the K input values of output token (b,i,j), in the order the weights expect */
static void ods_gather(const ods_desc *d, const float *x, int b, int i, int j, int P, float *v)
{
    const int C = d->C_in;
    if (d->kind == 0) {
        for (int di = 0; di < P; ++di)
            for (int dj = 0; dj < P; ++dj) {
                int r = i * P + di, c = j * P + dj;
                for (int ch = 0; ch < C; ++ch)
                    v[(di * P + dj) * C + ch] = (r < d->H && c < d->W) ? x[(((size_t)b * d->H + r) * d->W + c) * C + ch] : 0.0f;
            }
    } else {
        static const int off[4][2] = {{0, 0}, {1, 0}, {0, 1}, {1, 1}};   /* row offset, column offset */
        for (int q = 0; q < 4; ++q) {
            int r = 2 * i + off[q][0], c = 2 * j + off[q][1];
            for (int ch = 0; ch < C; ++ch)
                v[q * C + ch] = (r < d->H && c < d->W) ? x[(((size_t)b * d->H + r) * d->W + c) * C + ch] : 0.0f;
        }
    }
}

int orc_downsample_forward(const ods_desc *d, const ods_params *p, const float *x, float *out,
                           int8_t *tap_codes, int32_t *tap_acc, int32_t threads)
{
    if (!d || !p || !x || !out || !p->w || !p->s_w || !p->ln_gamma || !p->ln_beta) return ODS_E_NULL;
    if (d->act_bits < 2 || d->act_bits > 8 || d->weight_bits < 2 || d->weight_bits > 8) return ODS_E_BITS;
    int P, K, Ho, Wo, rc = ods_geometry(d, &P, &K, &Ho, &Wo);
    if (rc) return rc;
    const int N = d->N;
    const float inv = 1.0f / p->a_in.scale;
    const int32_t z = p->a_in.zero_point;
    int64_t *colsum = (int64_t *)malloc(sizeof(int64_t) * N);
    if (!colsum) return ODS_E_NULL;
    for (int n = 0; n < N; ++n) {
        int64_t s = 0;
        for (int k = 0; k < K; ++k) s += p->w[(size_t)n * K + k];
        colsum[n] = s;
    }
    const int64_t tokens = (int64_t)d->B * Ho * Wo;
    int failed = 0;
#pragma omp parallel num_threads(threads > 0 ? threads : 1)
    {
        float *v = (float *)malloc(sizeof(float) * K), *u = (float *)malloc(sizeof(float) * K);
        float *f = (float *)malloc(sizeof(float) * N);
        int32_t *code = (int32_t *)malloc(sizeof(int32_t) * K);
        if (!v || !u || !f || !code) {
#pragma omp atomic write
            failed = 1;
        } else {
#pragma omp for schedule(static)
            for (int64_t tok = 0; tok < tokens; ++tok) {      /* tokens are independent */
                const int b = (int)(tok / ((int64_t)Ho * Wo)), i = (int)(tok / Wo % Ho), j = (int)(tok % Wo);
                ods_gather(d, x, b, i, j, P, v);
                const float *src = v;
                if (d->kind == 1) { orc_layernorm(v, K, p->ln_gamma, p->ln_beta, d->ln_eps, u); src = u; }
                for (int k = 0; k < K; ++k) {
                    code[k] = orc_q(src[k], inv, z, d->act_bits);
                    if (tap_codes) tap_codes[tok * K + k] = (int8_t)code[k];
                }
                for (int n = 0; n < N; ++n) {
                    int64_t acc = 0;
                    for (int k = 0; k < K; ++k) acc += (int64_t)code[k] * p->w[(size_t)n * K + k];
                    acc -= (int64_t)z * colsum[n];
                    if (tap_acc) tap_acc[tok * N + n] = (int32_t)acc;
                    f[n] = fmaf((float)(int32_t)acc, p->a_in.scale * p->s_w[n], p->bias ? p->bias[n] : 0.0f);
                }
                if (d->kind == 0) orc_layernorm(f, N, p->ln_gamma, p->ln_beta, d->ln_eps, out + tok * N);
                else memcpy(out + tok * N, f, sizeof(float) * N);
            }
        }
        free(v); free(u); free(f); free(code);
    }
    free(colsum);
    return failed ? ODS_E_NULL : ODS_OK;
}
