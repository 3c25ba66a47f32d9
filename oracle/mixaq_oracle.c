/*
 * TEST INFRASTRUCTURE ONLY -- plain CPU oracle for the MixA-Q Two-Branch Swin
 * Block (paper Sec. 3.2 and Fig. 3).  Only tests/, the smoke check and the
 * benchmark's cpu_baseline leg may load this library; the product path must
 * never call it.  It shares no code with the HIP implementation.
 *
 * What it computes, in the paper's order:
 *   score   : importance of a window = its L2 norm (Sec. 3.2), computed on the
 *             un-shifted window grid of the stage input, shared by the stage;
 *   select  : the windows with the highest scores go to the high-precision
 *             branch, the rest to the low-precision branch (Sec. 3.2); the
 *             compression ratio is one number per pair of blocks (Sec. 3.3);
 *   branches: each branch runs LayerNorm (its own parameters) -> windowed
 *             multi-head attention -> LayerNorm -> FFN with the SHARED weights
 *             and its OWN activation step sizes / zero points (Sec. 3.2);
 *   scatter : outputs of both branches go back to the feature map (Fig. 3).
 * Everything the paper leaves open (padding, shift direction, mask, rounding,
 * quantizer form, where activations are quantized) follows the readings listed
 * in the design notes of this repository; each is marked "reading" below.
 *
 * Parity status: every step is pinned by tests to something other than this
 * file.  Structure: a float Swin block and a uniform block written separately,
 * brute-force mask, library pad/roll/reshape for gather and scatter, sort for
 * the selection.  Values, step by step from the previous step's tap: int64
 * matmuls for every integer sum, exact rational arithmetic for every
 * dequantize / residual / quantize epilogue on samples, float64 LayerNorm and
 * natural-base float64 softmax for the codes they decide (equal except within
 * a stated distance of a rounding tie), libm exp2 and erf for the two pinned
 * routines.  The paper prints no worked example, so no stored end-to-end value
 * exists; none of the pins is a paper-printed number.
 *
 * Layouts.  x, y: [B,H,W,C] float, channels last.  A "slot" is a position in
 * perm: slot g = b*nW + j processes window perm[b*nW+j] of image b; slots with
 * j < k_high belong to the high branch.  Every tap is slot-major:
 * [B*nW, 49, ...].
 */
#include <stdlib.h>
#include <string.h>
#include "arith.h"

typedef struct { float scale; int32_t zero_point; } orc_qparam;

typedef struct {
    int32_t B, H, W, C;
    int32_t window, shift;
    int32_t heads, mlp_ratio;
    int32_t act_bits_high, act_bits_low, weight_bits;
    int32_t score_mode;              /* 0: raw L2, 1: L2 after a scoring LayerNorm */
    float   ln_eps;
} orc_desc;

typedef struct {
    const float *ln1_gamma, *ln1_beta, *ln2_gamma, *ln2_beta;
    const float *b_qkv, *b_proj, *b_fc1, *b_fc2;
    orc_qparam a_qkv_in, a_q, a_k, a_v, a_p, a_proj_in, a_fc1_in, a_fc2_in;
} orc_branch;

typedef struct {
    const int8_t *w_qkv, *w_proj, *w_fc1, *w_fc2;     /* row-major [out,in] */
    const float  *s_qkv, *s_proj, *s_fc1, *s_fc2;     /* per output channel */
    const float  *rel_pos_bias;                       /* [heads,49,49] */
    const float  *score_gamma, *score_beta;           /* [C] (score_mode 1) */
} orc_shared;

typedef struct {                      /* all optional (NULL = not wanted) */
    int8_t  *a_qkv_in;   /* [S,49,C]   */
    int32_t *acc_qkv;    /* [S,49,3C]  */
    int8_t  *qkv;        /* [S,49,3C]  */
    int32_t *acc_s;      /* [S,heads,49,49] */
    int8_t  *p;          /* [S,heads,49,49] */
    int32_t *acc_o;      /* [S,49,C]   zero-point corrected */
    int8_t  *a_proj_in;  /* [S,49,C]   */
    int32_t *acc_proj;   /* [S,49,C]   */
    float   *h;          /* [S,49,C]   */
    int8_t  *a_fc1_in;   /* [S,49,C]   */
    int32_t *acc_fc1;    /* [S,49,4C]  */
    int8_t  *a_fc2_in;   /* [S,49,4C]  */
    int32_t *acc_fc2;    /* [S,49,C]   */
    float   *y_win;      /* [S,49,C]   */
} orc_taps;

enum { ORC_OK = 0, ORC_E_NULL = -1, ORC_E_SHAPE = -2, ORC_E_BITS = -3 };

#define MASK_VALUE (-100.0f)          /* reading: Swin's additive mask value */
#define LOG2E_F    0x1.715476p+0f     /* log2(e) rounded to binary32 */

static int padded(int n, int ws) { return (n + ws - 1) / ws * ws; }

static int check_desc(const orc_desc *d)
{
    if (!d) return ORC_E_NULL;
    if (d->B < 1 || d->H < 1 || d->W < 1 || d->C < 1 || d->window < 1) return ORC_E_SHAPE;
    if (d->heads < 1 || d->C % d->heads) return ORC_E_SHAPE;
    if (d->shift < 0 || d->shift >= d->window) return ORC_E_SHAPE;
    /* the neighbour predicate of the shift mask needs at least two windows per side */
    if (d->shift > 0 && (padded(d->H, d->window) < 2 * d->window || padded(d->W, d->window) < 2 * d->window)) return ORC_E_SHAPE;
    if (d->mlp_ratio < 1) return ORC_E_SHAPE;
    if (d->act_bits_high < 2 || d->act_bits_high > 8) return ORC_E_BITS;
    if (d->act_bits_low < 2 || d->act_bits_low > 8) return ORC_E_BITS;
    if (d->weight_bits < 2 || d->weight_bits > 8) return ORC_E_BITS;
    return ORC_OK;
}

int orc_num_windows(const orc_desc *d, int32_t *nW)
{
    int rc = check_desc(d);
    if (rc) return rc;
    if (!nW) return ORC_E_NULL;
    *nW = (padded(d->H, d->window) / d->window) * (padded(d->W, d->window) / d->window);
    return ORC_OK;
}

/* reading: number of high-branch windows per image = keep ratio times window
 * count, rounded half up (Sec. 3.3 defines the ratio as a share of the windows). */
int orc_keep_count(int32_t nW, double keep_ratio, int32_t *k_high)
{
    if (!k_high) return ORC_E_NULL;
    if (nW < 0 || !(keep_ratio >= 0.0) || !(keep_ratio <= 1.0)) return ORC_E_SHAPE;
    double k = floor(keep_ratio * (double)nW + 0.5);
    if (k < 0) k = 0;
    if (k > nW) k = nW;
    *k_high = (int32_t)k;
    return ORC_OK;
}

/* Where token t of window w comes from.  reading: the map is zero-padded at the
 * bottom/right to multiples of the window, rolled by -shift before partitioning
 * (so rolled[r,c] = padded[(r+s) mod Hp, (c+s) mod Wp]), windows are numbered
 * row-major.  Returns 1 when the source lies inside the H x W map. */
int orc_token_source(const orc_desc *d, int32_t w, int32_t t, int32_t *row, int32_t *col)
{
    int ws = d->window, Hp = padded(d->H, ws), Wp = padded(d->W, ws), nWc = Wp / ws;
    int wr = w / nWc, wc = w % nWc, tr = t / ws, tc = t % ws;
    int pr = (wr * ws + tr + d->shift) % Hp;
    int pc = (wc * ws + tc + d->shift) % Wp;
    *row = pr; *col = pc;
    return pr < d->H && pc < d->W;
}

/* Shifted-window mask: tokens i and j of one rolled window may attend to each
 * other iff they are neighbours in the ORIGINAL padded map, i.e. closer than
 * one window in both directions.  Returns 1 when the pair is masked. */
int orc_mask_pair(const orc_desc *d, int32_t w, int32_t ti, int32_t tj)
{
    if (d->shift == 0) return 0;
    int ri, ci, rj, cj;
    orc_token_source(d, w, ti, &ri, &ci);
    orc_token_source(d, w, tj, &rj, &cj);
    int dr = ri > rj ? ri - rj : rj - ri, dc = ci > cj ? ci - cj : cj - ci;
    return !(dr < d->window && dc < d->window);
}

/* Importance score (Sec. 3.2): squared L2 norm of the window (the square root
 * is monotone and dropped), over in-bounds tokens of the un-shifted grid. */
int orc_score_windows(const orc_desc *d, const orc_shared *sh, const float *x, double *scores)
{
    int rc = check_desc(d);
    if (rc) return rc;
    if (!x || !scores) return ORC_E_NULL;
    if (d->score_mode == 1 && (!sh || !sh->score_gamma || !sh->score_beta)) return ORC_E_NULL;
    orc_desc g = *d; g.shift = 0;
    int32_t nW; orc_num_windows(d, &nW);
    int T = d->window * d->window, C = d->C;
    float *u = (float *)malloc(sizeof(float) * C);
    for (int b = 0; b < d->B; ++b)
        for (int w = 0; w < nW; ++w) {
            double acc = 0.0;
            for (int t = 0; t < T; ++t) {
                int r, c;
                if (!orc_token_source(&g, w, t, &r, &c)) continue;
                const float *px = x + (((size_t)b * d->H + r) * d->W + c) * C;
                if (d->score_mode == 1) orc_layernorm(px, C, sh->score_gamma, sh->score_beta, d->ln_eps, u);
                else memcpy(u, px, sizeof(float) * C);
                for (int ch = 0; ch < C; ++ch) acc += (double)u[ch] * (double)u[ch];
            }
            scores[(size_t)b * nW + w] = acc;
        }
    free(u);
    return ORC_OK;
}

/* Selection (Sec. 3.2): the k_high windows with the highest scores form the
 * high group.  reading: perm lists the windows of an image in order of decreasing
 * score, ties going to the lower window index, so the high group is its first
 * k_high entries and the low group the rest.  reverse != 0 inverts the importance
 * order (the worst-case window selection of the robustness study, Sec. 4.1). */
int orc_select_windows3(const double *scores, int32_t B, int32_t nW, int32_t k_high, int32_t k_low,
                        int32_t reverse, int32_t *perm);

int orc_select_windows(const double *scores, int32_t B, int32_t nW, int32_t k_high,
                       int32_t reverse, int32_t *perm)
{
    return orc_select_windows3(scores, B, nW, k_high, nW - k_high, reverse, perm);
}

/* reading: the paper orders windows by their L2 norm and says nothing of scores that are not numbers
 * (a window holding NaN; Inf under the scoring LayerNorm).  Such a score is outside the order; it is
 * ranked behind every number, infinities included (ties among them by index), so that the list stays a
 * permutation. */
static double rank_key(double s, int reverse)
{
    if (isnan(s)) return reverse ? INFINITY : -INFINITY;
    return s;
}

/* Selection with activation pruning (Sec. 3.4): the windows with the lowest scores are pruned,
 * the rest is split as before.  perm is the same sorted list; its first k_high entries are the high
 * group, the next k_low the low group, the remainder is pruned. */
int orc_select_windows3(const double *scores, int32_t B, int32_t nW, int32_t k_high, int32_t k_low,
                        int32_t reverse, int32_t *perm)
{
    if (!scores || !perm) return ORC_E_NULL;
    if (B < 1 || nW < 1 || k_high < 0 || k_low < 0 || k_high + k_low > nW) return ORC_E_SHAPE;
    for (int b = 0; b < B; ++b) {
        const double *s = scores + (size_t)b * nW;
        int32_t *p = perm + (size_t)b * nW;
        for (int w = 0; w < nW; ++w) {
            double sw = rank_key(s[w], reverse);
            int nw = isnan(s[w]);
            int rank = 0;                         /* windows strictly ahead of w */
            for (int v = 0; v < nW; ++v) {
                if (v == w) continue;
                double sv = rank_key(s[v], reverse);
                int nv = isnan(s[v]);
                int ahead = reverse ? (sv < sw) : (sv > sw);
                /* equal keys: a number goes before a NaN, otherwise the lower index first */
                if (ahead || (sv == sw && (nv != nw ? nw : v < w))) ++rank;
            }
            p[rank] = w;                          /* the rank under a total order is a permutation */
        }
    }
    return ORC_OK;
}

/* Gather (Fig. 3): slot-major copy of the windows, zeros for padded sources. */
int orc_gather_windows(const orc_desc *d, const float *x, const int32_t *perm, float *win, uint8_t *valid)
{
    int rc = check_desc(d);
    if (rc) return rc;
    if (!x || !perm || !win) return ORC_E_NULL;
    int32_t nW; orc_num_windows(d, &nW);
    int T = d->window * d->window, C = d->C;
    for (int b = 0; b < d->B; ++b)
        for (int j = 0; j < nW; ++j)
            for (int t = 0; t < T; ++t) {
                int r, c, ok = orc_token_source(d, perm[(size_t)b * nW + j], t, &r, &c);
                float *dst = win + (((size_t)b * nW + j) * T + t) * C;
                if (ok) memcpy(dst, x + (((size_t)b * d->H + r) * d->W + c) * C, sizeof(float) * C);
                else memset(dst, 0, sizeof(float) * C);
                if (valid) valid[((size_t)b * nW + j) * T + t] = (uint8_t)ok;
            }
    return ORC_OK;
}

/* Scatter (Fig. 3): inverse of the gather; padded targets are dropped. */
int orc_scatter_windows(const orc_desc *d, const float *win, const int32_t *perm, float *y)
{
    int rc = check_desc(d);
    if (rc) return rc;
    if (!win || !perm || !y) return ORC_E_NULL;
    int32_t nW; orc_num_windows(d, &nW);
    int T = d->window * d->window, C = d->C;
    for (int b = 0; b < d->B; ++b)
        for (int j = 0; j < nW; ++j)
            for (int t = 0; t < T; ++t) {
                int r, c;
                if (!orc_token_source(d, perm[(size_t)b * nW + j], t, &r, &c)) continue;
                memcpy(y + (((size_t)b * d->H + r) * d->W + c) * C,
                       win + (((size_t)b * nW + j) * T + t) * C, sizeof(float) * C);
            }
    return ORC_OK;
}

/* Integer linear layer of a shadow layer (Sec. 3.2: shared weights, per-branch
 * step size / zero point): acc[t,n] = sum_k a[t,k]*W[n,k] - z_a*sum_k W[n,k]. */
static void int_linear(const int32_t *a, int T, int K, const int8_t *W, int N, int32_t z_a, int32_t *acc)
{
    for (int t = 0; t < T; ++t)
        for (int n = 0; n < N; ++n) {
            int32_t s = 0, cs = 0;
            for (int k = 0; k < K; ++k) { s += a[t * K + k] * (int32_t)W[(size_t)n * K + k]; cs += W[(size_t)n * K + k]; }
            acc[t * N + n] = s - z_a * cs;
        }
}

/* Softmax of one row of base-2 logits followed by the P quantizer: maximum,
 * pinned 2^x, binary64 sum rounded once, one reciprocal, one product. */
static void softmax2_row(const float *lg, int n, float *prob)
{
    float mx = -INFINITY;
    for (int j = 0; j < n; ++j) if (lg[j] > mx) mx = lg[j];
    double den = 0.0;
    for (int j = 0; j < n; ++j) { prob[j] = orc_exp2_pinned(lg[j] - mx); den += (double)prob[j]; }
    float rden = 1.0f / (float)den;
    for (int j = 0; j < n; ++j) prob[j] = prob[j] * rden;
}

static void process_slot(const orc_desc *d, const orc_shared *sh, const orc_branch *br, int bits,
                         const float *x, int b, int w, size_t slot, float *y, const orc_taps *tp)
{
    const int ws = d->window, T = ws * ws, C = d->C, nh = d->heads, hd = C / nh, F = C * d->mlp_ratio;
    float   *xin  = (float *)calloc((size_t)T * C, sizeof(float));      /* shortcut, 0 on padding */
    float   *ln   = (float *)malloc(sizeof(float) * C);
    int32_t *a1   = (int32_t *)malloc(sizeof(int32_t) * T * C);
    int32_t *aqkv = (int32_t *)malloc(sizeof(int32_t) * T * 3 * C);
    int32_t *cqkv = (int32_t *)malloc(sizeof(int32_t) * T * 3 * C);
    int32_t *ao   = (int32_t *)malloc(sizeof(int32_t) * T * C);
    int32_t *accp = (int32_t *)malloc(sizeof(int32_t) * T * C);
    float   *hres = (float *)malloc(sizeof(float) * T * C);
    int32_t *a2   = (int32_t *)malloc(sizeof(int32_t) * T * C);
    int32_t *acc1 = (int32_t *)malloc(sizeof(int32_t) * T * F);
    int32_t *g    = (int32_t *)malloc(sizeof(int32_t) * T * F);
    int32_t *acc2 = (int32_t *)malloc(sizeof(int32_t) * T * C);
    float   *lg   = (float *)malloc(sizeof(float) * T);
    float   *ev   = (float *)malloc(sizeof(float) * T);
    int     *src_ok = (int *)malloc(sizeof(int) * T), *src_r = (int *)malloc(sizeof(int) * T), *src_c = (int *)malloc(sizeof(int) * T);

    /* gather + LN1 + quantize.  reading: padded tokens enter the attention as
     * LN output 0 (zero-padding after the norm) and carry a zero shortcut. */
    float inv = 1.0f / br->a_qkv_in.scale;
    for (int t = 0; t < T; ++t) {
        src_ok[t] = orc_token_source(d, w, t, &src_r[t], &src_c[t]);
        if (src_ok[t]) {
            const float *px = x + (((size_t)b * d->H + src_r[t]) * d->W + src_c[t]) * C;
            memcpy(xin + (size_t)t * C, px, sizeof(float) * C);
            orc_layernorm(px, C, br->ln1_gamma, br->ln1_beta, d->ln_eps, ln);
        } else {
            for (int c = 0; c < C; ++c) ln[c] = 0.0f;
        }
        for (int c = 0; c < C; ++c) a1[t * C + c] = orc_q(ln[c], inv, br->a_qkv_in.zero_point, bits);
    }
    /* QKV projection; output channel n = which*C + head*hd + dim (reading) */
    int_linear(a1, T, C, sh->w_qkv, 3 * C, br->a_qkv_in.zero_point, aqkv);
    for (int t = 0; t < T; ++t)
        for (int n = 0; n < 3 * C; ++n) {
            const orc_qparam *qp = n < C ? &br->a_q : (n < 2 * C ? &br->a_k : &br->a_v);
            float m = br->a_qkv_in.scale * sh->s_qkv[n];
            float f = fmaf((float)aqkv[t * 3 * C + n], m, br->b_qkv[n]);
            cqkv[t * 3 * C + n] = orc_q(f, 1.0f / qp->scale, qp->zero_point, bits);   /* zero_point is 0 for q,k,v */
        }
    /* attention per head, softmax in base 2: 2^(log2e*l - max) == e^(l - max') */
    float m2 = ((br->a_q.scale * br->a_k.scale) * (float)(1.0 / sqrt((double)hd))) * LOG2E_F;
    float inv_p = 1.0f / br->a_p.scale, m_o = br->a_p.scale * br->a_v.scale, inv_ao = 1.0f / br->a_proj_in.scale;
    int32_t zp = br->a_p.zero_point;
    for (int hh = 0; hh < nh; ++hh) {
        for (int i = 0; i < T; ++i) {
            int32_t pc[64 * 4];                     /* T <= 256 is checked by the caller */
            for (int j = 0; j < T; ++j) {
                int32_t s = 0;
                for (int k = 0; k < hd; ++k)
                    s += cqkv[i * 3 * C + hh * hd + k] * cqkv[j * 3 * C + C + hh * hd + k];
                float bias = sh->rel_pos_bias[((size_t)hh * T + i) * T + j];
                if (orc_mask_pair(d, w, i, j)) bias = bias + MASK_VALUE;
                lg[j] = fmaf((float)s, m2, bias * LOG2E_F);
                if (tp && tp->acc_s) tp->acc_s[((slot * nh + hh) * T + i) * T + j] = s;
            }
            softmax2_row(lg, T, ev);
            for (int j = 0; j < T; ++j) {
                pc[j] = orc_q(ev[j], inv_p, zp, bits);
                if (tp && tp->p) tp->p[((slot * nh + hh) * T + i) * T + j] = (int8_t)pc[j];
            }
            for (int k = 0; k < hd; ++k) {
                int32_t o = 0;
                for (int j = 0; j < T; ++j) o += (pc[j] - zp) * cqkv[j * 3 * C + 2 * C + hh * hd + k];
                float f = (float)o * m_o;
                ao[i * C + hh * hd + k] = orc_q(f, inv_ao, br->a_proj_in.zero_point, bits);
                if (tp && tp->acc_o) tp->acc_o[(slot * T + i) * C + hh * hd + k] = o;
            }
        }
    }
    /* output projection + first residual */
    int_linear(ao, T, C, sh->w_proj, C, br->a_proj_in.zero_point, accp);
    for (int t = 0; t < T; ++t)
        for (int n = 0; n < C; ++n) {
            float f = fmaf((float)accp[t * C + n], br->a_proj_in.scale * sh->s_proj[n], br->b_proj[n]);
            hres[t * C + n] = f + xin[t * C + n];
        }
    /* LN2 + FFN (fc1 -> GELU -> fc2) + second residual */
    inv = 1.0f / br->a_fc1_in.scale;
    for (int t = 0; t < T; ++t) {
        orc_layernorm(hres + (size_t)t * C, C, br->ln2_gamma, br->ln2_beta, d->ln_eps, ln);
        for (int c = 0; c < C; ++c) a2[t * C + c] = orc_q(ln[c], inv, br->a_fc1_in.zero_point, bits);
    }
    int_linear(a2, T, C, sh->w_fc1, F, br->a_fc1_in.zero_point, acc1);
    inv = 1.0f / br->a_fc2_in.scale;
    for (int t = 0; t < T; ++t)
        for (int n = 0; n < F; ++n) {
            float f = fmaf((float)acc1[t * F + n], br->a_fc1_in.scale * sh->s_fc1[n], br->b_fc1[n]);
            g[t * F + n] = orc_q(orc_gelu_pinned(f), inv, br->a_fc2_in.zero_point, bits);
        }
    int_linear(g, T, F, sh->w_fc2, C, br->a_fc2_in.zero_point, acc2);
    for (int t = 0; t < T; ++t)
        for (int n = 0; n < C; ++n) {
            float f = fmaf((float)acc2[t * C + n], br->a_fc2_in.scale * sh->s_fc2[n], br->b_fc2[n]);
            float out = f + hres[t * C + n];
            if (tp && tp->y_win) tp->y_win[(slot * T + t) * C + n] = out;
            if (src_ok[t]) y[(((size_t)b * d->H + src_r[t]) * d->W + src_c[t]) * C + n] = out;   /* scatter */
        }
    if (tp) {
        for (int i = 0; i < T * C; ++i) {
            if (tp->a_qkv_in)  tp->a_qkv_in[slot * T * C + i]  = (int8_t)a1[i];
            if (tp->a_proj_in) tp->a_proj_in[slot * T * C + i] = (int8_t)ao[i];
            if (tp->acc_proj)  tp->acc_proj[slot * T * C + i]  = accp[i];
            if (tp->h)         tp->h[slot * T * C + i]         = hres[i];
            if (tp->a_fc1_in)  tp->a_fc1_in[slot * T * C + i]  = (int8_t)a2[i];
            if (tp->acc_fc2)   tp->acc_fc2[slot * T * C + i]   = acc2[i];
        }
        for (int i = 0; i < T * 3 * C; ++i) {
            if (tp->acc_qkv) tp->acc_qkv[slot * T * 3 * C + i] = aqkv[i];
            if (tp->qkv)     tp->qkv[slot * T * 3 * C + i]     = (int8_t)cqkv[i];
        }
        for (int i = 0; i < T * F; ++i) {
            if (tp->acc_fc1)  tp->acc_fc1[slot * T * F + i]  = acc1[i];
            if (tp->a_fc2_in) tp->a_fc2_in[slot * T * F + i] = (int8_t)g[i];
        }
    }
    free(xin); free(ln); free(a1); free(aqkv); free(cqkv); free(ao); free(accp); free(hres); free(a2);
    free(acc1); free(g); free(acc2); free(lg); free(ev); free(src_ok); free(src_r); free(src_c);
}

static int check_params(const orc_desc *d, const orc_shared *sh, const orc_branch br[2])
{
    if (!sh || !br) return ORC_E_NULL;
    if (!sh->w_qkv || !sh->w_proj || !sh->w_fc1 || !sh->w_fc2 || !sh->s_qkv || !sh->s_proj ||
        !sh->s_fc1 || !sh->s_fc2 || !sh->rel_pos_bias) return ORC_E_NULL;
    for (int i = 0; i < 2; ++i) {
        const orc_branch *p = &br[i];
        if (!p->ln1_gamma || !p->ln1_beta || !p->ln2_gamma || !p->ln2_beta || !p->b_qkv ||
            !p->b_proj || !p->b_fc1 || !p->b_fc2) return ORC_E_NULL;
        const orc_qparam *q = &p->a_qkv_in;
        for (int k = 0; k < 8; ++k) if (!(q[k].scale > 0.0f)) return ORC_E_SHAPE;
        if (p->a_q.zero_point || p->a_k.zero_point || p->a_v.zero_point) return ORC_E_SHAPE;
    }
    if (d->window * d->window > 256) return ORC_E_SHAPE;
    return ORC_OK;
}

/* One Two-Branch Swin Block (Fig. 3).  perm == NULL: score and select here with
 * k_high windows per image in the high branch.  threads > 1 only splits the
 * independent windows over OpenMP threads; the arithmetic is unchanged. */
int orc_block_forward_pruned(const orc_desc *d, const orc_shared *sh, const orc_branch br[2], const float *x,
                             const int32_t *perm, int32_t k_high, int32_t k_low, float *y, const orc_taps *taps,
                             int32_t threads);

int orc_block_forward(const orc_desc *d, const orc_shared *sh, const orc_branch br[2], const float *x,
                      const int32_t *perm, int32_t k_high, float *y, const orc_taps *taps, int32_t threads)
{
    int32_t nW;
    int rc = orc_num_windows(d, &nW);
    if (rc) return rc;
    return orc_block_forward_pruned(d, sh, br, x, perm, k_high, nW - k_high, y, taps, threads);
}

/* Block with activation pruning incorporated (Sec. 3.4): positions k_high+k_low.. of perm are
 * pruned windows; their computation is skipped and their features are forwarded unchanged. */
int orc_block_forward_pruned(const orc_desc *d, const orc_shared *sh, const orc_branch br[2], const float *x,
                             const int32_t *perm, int32_t k_high, int32_t k_low, float *y, const orc_taps *taps,
                             int32_t threads)
{
    int rc = check_desc(d);
    if (rc) return rc;
    if ((rc = check_params(d, sh, br))) return rc;
    if (!x || !y) return ORC_E_NULL;
    int32_t nW; orc_num_windows(d, &nW);
    if (k_high < 0 || k_low < 0 || k_high + k_low > nW) return ORC_E_SHAPE;
    int32_t *own = NULL;
    if (!perm) {
        double *sc = (double *)malloc(sizeof(double) * d->B * nW);
        own = (int32_t *)malloc(sizeof(int32_t) * d->B * nW);
        rc = orc_score_windows(d, sh, x, sc);
        if (!rc) rc = orc_select_windows3(sc, d->B, nW, k_high, k_low, 0, own);
        free(sc);
        if (rc) { free(own); return rc; }
        perm = own;
    }
    long total = (long)d->B * nW;
    if (threads < 1) threads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
    for (long s = 0; s < total; ++s) {
        int b = (int)(s / nW), j = (int)(s % nW);
        int hi = j < k_high;
        if (j < k_high + k_low) {
            process_slot(d, sh, &br[hi ? 0 : 1], hi ? d->act_bits_high : d->act_bits_low, x, b,
                         perm[s], (size_t)s, y, taps);
        } else {                                         /* pruned: forward the features */
            for (int t = 0; t < d->window * d->window; ++t) {
                int r, c;
                if (!orc_token_source(d, perm[s], t, &r, &c)) continue;
                size_t off = (((size_t)b * d->H + r) * d->W + c) * d->C;
                memcpy(y + off, x + off, sizeof(float) * d->C);
            }
        }
    }
    free(own);
    return ORC_OK;
}

/* scalar entry points for the pins */
float   orc_exp2(float y) { return orc_exp2_pinned(y); }
float   orc_gelu(float x) { return orc_gelu_pinned(x); }
int32_t orc_quantize(float v, float scale, int32_t zero_point, int32_t bits) { return orc_q(v, 1.0f / scale, zero_point, bits); }
void    orc_layernorm_token(const float *x, int32_t C, const float *g, const float *b, float eps, float *y) { orc_layernorm(x, C, g, b, eps, y); }
void    orc_softmax2(const float *lg, int32_t n, float *prob) { softmax2_row(lg, n, prob); }
void    orc_exp2_array(const float *y, float *out, int64_t n) { for (int64_t i = 0; i < n; ++i) out[i] = orc_exp2_pinned(y[i]); }
void    orc_gelu_array(const float *x, float *out, int64_t n) { for (int64_t i = 0; i < n; ++i) out[i] = orc_gelu_pinned(x[i]); }
