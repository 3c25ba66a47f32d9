// gfx950 kernels of the Two-Branch Swin Block (paper Sec. 3.2, Fig. 3):
//   score_kernel      window importance = squared L2 norm            (Sec. 3.2)
//   select_kernel     top-k partition into high / low groups         (Sec. 3.2)
//   ln_quant_kernel   gather (shift folded in) + LayerNorm + quantize, also LN2
//   gemm_tile_kernel  int8 MFMA linear layers with fused epilogues   (shadow layers)
//   attn_kernel       per (window, head): QK^T, bias+mask, softmax, P.V
// Arithmetic that decides an integer code follows the pinned binary32 sequences
// of mixaq_dev.h; reductions feeding a code run in binary64.
#include <algorithm>
#include "mixaq_dev.h"
#include "kernels.h"

namespace mixaq {

// ------------------------------------------------------------------ helpers
// sum over a group of W consecutive lanes (the group does not straddle a wave); every lane of the
// group gets the same bits: a butterfly for powers of two, a fixed-order gather otherwise
// (first = the group's first lane).
template <int W>
__device__ __forceinline__ double group_sum(double v, int first = 0)
{
    if ((W & (W - 1)) == 0) {
#pragma unroll
        for (int o = W / 2; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
        return v;
    }
    double tot = __shfl(v, first, 64);
#pragma unroll
    for (int k = 1; k < W; ++k) tot += __shfl(v, first + k, 64);
    return tot;
}

// LayerNorm of one token spread over LPT lanes (NV float4 per lane; channel of
// element e of vector k on lane i: (k*LPT + i)*4 + e).  Mean and variance in
// binary64, rounded once.
template <int LPT, int NV>
__device__ __forceinline__ void token_ln_stats(const float4 (&v)[NV], int C, float eps, float& mean, float& rstd, int first = 0)
{
    double s = 0.0;
#pragma unroll
    for (int k = 0; k < NV; ++k) s += ((double)v[k].x + (double)v[k].y) + ((double)v[k].z + (double)v[k].w);
    s = group_sum<LPT>(s, first);
    mean = (float)(s / (double)C);
    double q = 0.0;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        double a = (double)v[k].x - (double)mean, b = (double)v[k].y - (double)mean;
        double c = (double)v[k].z - (double)mean, d = (double)v[k].w - (double)mean;
        q += (a * a + b * b) + (c * c + d * d);
    }
    q = group_sum<LPT>(q, first);
    const float var = (float)(q / (double)C);
    rstd = 1.0f / sqrtf(var + eps);
}

template <int LPT, int NV>
__device__ __forceinline__ void token_ln_apply(float4 (&v)[NV], float mean, float rstd, const float* __restrict__ gamma,
                                               const float* __restrict__ beta, int sub)
{
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        int ch = (k * LPT + sub) * 4;
        float4 g = *(const float4*)(gamma + ch), b = *(const float4*)(beta + ch);
        v[k].x = fmaf((v[k].x - mean) * rstd, g.x, b.x);
        v[k].y = fmaf((v[k].y - mean) * rstd, g.y, b.y);
        v[k].z = fmaf((v[k].z - mean) * rstd, g.z, b.z);
        v[k].w = fmaf((v[k].w - mean) * rstd, g.w, b.w);
    }
}

template <int LPT, int NV>
__device__ __forceinline__ void token_layernorm(float4 (&v)[NV], int C, float eps, const float* __restrict__ gamma,
                                                const float* __restrict__ beta, int sub, int first = 0)
{
    float mean, rstd;
    token_ln_stats<LPT, NV>(v, C, eps, mean, rstd, first);
    token_ln_apply<LPT, NV>(v, mean, rstd, gamma, beta, sub);
}

// ------------------------------------------------------------------ K0 score
// One workgroup (256 threads) per window of the un-shifted grid.
template <int LPT, int NV>
__global__ __launch_bounds__(256) void score_kernel(Geom G, const float* __restrict__ x, int mode, float eps,
                                                    const float* __restrict__ gamma, const float* __restrict__ beta,
                                                    double* __restrict__ scores)
{
    const int wid = blockIdx.x;                       // b*nW + w
    const int b = wid / G.nW, w = wid - b * G.nW;
    const int wr = w / G.nWc, wc = w - wr * G.nWc;
    const int grp = threadIdx.x / LPT, sub = threadIdx.x % LPT;
    constexpr int TP = 256 / LPT;
    double acc = 0.0;
    constexpr int PASSES = (TOK + TP - 1) / TP;
    constexpr int PC = LPT <= 16 ? PASSES : 2;        // passes whose loads are issued together, before any arithmetic
#pragma unroll 1
    for (int p0 = 0; p0 < PASSES; p0 += PC) {
        float4 v[PC][NV];
        bool in[PC];
#pragma unroll
        for (int p = 0; p < PC; ++p) {
            const int t = grp + (p0 + p) * TP, pr = wr * WS + t / WS, pc = wc * WS + t % WS;
            in[p] = t < TOK && pr < G.H && pc < G.W;  // uniform inside a token group
            if (in[p]) {
                const float* px = x + ((size_t)(b * G.H + pr) * G.W + pc) * G.C;
#pragma unroll
                for (int k = 0; k < NV; ++k) v[p][k] = *(const float4*)(px + (k * LPT + sub) * 4);
            }
        }
#pragma unroll
        for (int p = 0; p < PC; ++p) {
            if (in[p]) {
                if (mode == 1) token_layernorm<LPT, NV>(v[p], G.C, eps, gamma, beta, sub);
#pragma unroll
                for (int k = 0; k < NV; ++k)
                    acc += ((double)v[p][k].x * (double)v[p][k].x + (double)v[p][k].y * (double)v[p][k].y) +
                           ((double)v[p][k].z * (double)v[p][k].z + (double)v[p][k].w * (double)v[p][k].w);
            }
        }
    }
    acc = group_sum<64>(acc);
    __shared__ double part[4];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) scores[wid] = (part[0] + part[1]) + (part[2] + part[3]);
}

// ------------------------------------------------------------------ K1 select
// Rank by counting under the total order (score descending, index ascending): the rank of a
// window is the number of windows ahead of it, which is a permutation, so perm[rank] = window
// lists the windows by decreasing importance; the high group is the first k_hi entries.
// A wave ranks four windows at once, its lanes stride over the candidates held in LDS.
// A score that is not a number (a window holding NaN, or Inf under the scoring LayerNorm) is outside
// the order: it is ranked behind every number (infinities included), so the ranks stay a permutation.
// rank_key maps it to the infinity at the unimportant end; among equal keys a number goes first.
__device__ __forceinline__ double rank_key(double s, int reverse)
{
    const double worst = reverse ? __longlong_as_double(0x7ff0000000000000LL) : __longlong_as_double(0xfff0000000000000LL);
    return s != s ? worst : s;
}
// true when candidate v (raw score rv) is ranked before window w (raw score rw)
__device__ __forceinline__ bool ranked_before(double rv, int v, double rw, int w, int reverse)
{
    const double sv = rank_key(rv, reverse), sw = rank_key(rw, reverse);
    const bool nv = rv != rv, nw = rw != rw;
    const bool ahead = reverse ? (sv < sw) : (sv > sw);
    return ahead || (sv == sw && (nv != nw ? nw : v < w));
}
constexpr int RANK_WPB = 16;                          // windows ranked per workgroup (4 per wave)
__global__ __launch_bounds__(256) void select_rank_kernel(const double* __restrict__ scores, int nW, int reverse,
                                                          int* __restrict__ perm)
{
    extern __shared__ double rsc[];                   // all scores of the image
    const int b = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const double* sc = scores + (size_t)b * nW;
    for (int base = 0; base < nW; base += 2048) {     // eight loads in flight per thread
        double tmp[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) { const int i = base + threadIdx.x + k * 256; tmp[k] = i < nW ? sc[i] : 0.0; }
#pragma unroll
        for (int k = 0; k < 8; ++k) { const int i = base + threadIdx.x + k * 256; if (i < nW) rsc[i] = tmp[k]; }
    }
    __syncthreads();
    constexpr int Q = RANK_WPB / 4;                   // windows per wave, ranked together
    const int w0 = blockIdx.x * RANK_WPB + wave * Q;
    if (w0 >= nW) return;                             // whole wave, after the barrier
    double sw[Q];
    int rank[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) { sw[q] = rsc[min(w0 + q, nW - 1)]; rank[q] = 0; }
    for (int v0 = lane; v0 < nW; v0 += 256) {
        double sv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) { const int v = v0 + 64 * u; sv[u] = rsc[min(v, nW - 1)]; }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int v = v0 + 64 * u;
#pragma unroll
            for (int q = 0; q < Q; ++q) rank[q] += (v < nW && ranked_before(sv[u], v, sw[q], w0 + q, reverse)) ? 1 : 0;
        }
    }
#pragma unroll
    for (int q = 0; q < Q; ++q) {
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) rank[q] += __shfl_xor(rank[q], o, 64);
        if (lane == 0 && w0 + q < nW) perm[(size_t)b * nW + rank[q]] = w0 + q;
    }
}

// ------------------------------------------------------------------ pruned windows
// Activation pruning (paper Sec. 3.4): the windows after the high and low groups in perm are
// skipped by the block and their features are forwarded.  One workgroup per pruned window.
__global__ __launch_bounds__(256) void bypass_kernel(Geom G, const int* __restrict__ perm, const float* __restrict__ x,
                                                     float* __restrict__ y)
{
    const int kept = G.k_hi + G.k_lo, n_pruned = G.nW - kept;
    const int b = blockIdx.x / n_pruned, jpos = kept + blockIdx.x % n_pruned;
    const int w = perm[b * G.nW + jpos];
    const int wr = w / G.nWc, wc = w - wr * G.nWc;
    const int c4 = G.C / 4;
    for (int i = threadIdx.x; i < TOK * c4; i += 256) {
        const int t = i / c4, k = i - t * c4, tr = t / WS, tc = t - tr * WS;
        int pr = wr * WS + tr + G.shift; if (pr >= G.Hp) pr -= G.Hp;
        int pc = wc * WS + tc + G.shift; if (pc >= G.Wp) pc -= G.Wp;
        if (pr < G.H && pc < G.W) {
            const size_t off = ((size_t)(b * G.H + pr) * G.W + pc) * G.C + k * 4;
            *(float4*)(y + off) = *(const float4*)(x + off);
        }
    }
}

// ------------------------------------------------------------------ K2 / K6
// One token per group of LPT lanes.  GATHER: source is the feature map through the
// window / shift / padding index map, and the row bookkeeping is written.
template <int LPT, int NV, bool GATHER>
__global__ __launch_bounds__(256) void ln_quant_kernel(Geom G, LnArgs A)
{
    constexpr int TP = 256 / LPT;
    const int row = blockIdx.x * TP + threadIdx.x / LPT, sub = threadIdx.x % LPT;
    if (row >= G.rows_total) return;
    int branch, canon, pix;
    if (GATHER) {
        RowInfo ri = row_info(G, A.perm, row);
        branch = ri.branch; canon = ri.canon; pix = ri.pix;
        if (sub == 0) { A.row_pix[row] = pix; A.row_canon[row] = canon; }
    } else {
        branch = row >= G.base_lo ? 1 : 0;
        canon = A.row_canon[row];
        pix = 0;
    }
    const QDev q = A.q[branch];
    int8_t* dst = A.out + (size_t)row * G.C;
    float4 v[NV];
    const bool real = canon >= 0 && pix >= 0;
    if (real) {
        const float* src = GATHER ? A.src + (size_t)pix * G.C : A.src + (size_t)row * G.C;
#pragma unroll
        for (int k = 0; k < NV; ++k) v[k] = *(const float4*)(src + (k * LPT + sub) * 4);
        token_layernorm<LPT, NV>(v, G.C, A.eps, A.gamma[branch], A.beta[branch], sub);
    } else {
#pragma unroll
        for (int k = 0; k < NV; ++k) v[k] = make_float4(0.f, 0.f, 0.f, 0.f);   // padding enters as LN output 0
    }
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        int code = pack4(quant_code(v[k].x, q), quant_code(v[k].y, q), quant_code(v[k].z, q), quant_code(v[k].w, q));
        if (canon < 0) code = 0;
        int ch = (k * LPT + sub) * 4;
        *(int*)(dst + ch) = code;
        if (A.tap && canon >= 0) *(int*)(A.tap + (size_t)canon * G.C + ch) = code;
    }
}

// ------------------------------------------------------------------ GEMMs
// out^T = W * act^T on 32x32x32 int8 MFMA: the packed weight fragment is the A
// operand (rows = output channels), the activation rows are the B operand (columns
// = tokens), so a lane owns one token and 16 output channels per 32-channel block.
// A wave computes 64 rows x 32 channels at a time.
template <int EPI>
__device__ __forceinline__ void epilogue(const GemmArgs& A, const Geom& G, int branch, int row, int nb, int g,
                                         const v16i& acc, int pix, int canon, const float4* gelu_lds)
{
    const int N = A.N;
#pragma unroll
    for (int qd = 0; qd < 4; ++qd) {
        const int n0 = nb * 32 + qd * 8 + g * 4;
        const float4 m = *(const float4*)(A.m[branch] + n0);
        const float4 bs = *(const float4*)(A.bias[branch] + n0);
        const int a0 = acc[qd * 4 + 0], a1 = acc[qd * 4 + 1], a2 = acc[qd * 4 + 2], a3 = acc[qd * 4 + 3];
        float f0 = fmaf((float)a0, m.x, bs.x), f1 = fmaf((float)a1, m.y, bs.y);
        float f2 = fmaf((float)a2, m.z, bs.z), f3 = fmaf((float)a3, m.w, bs.w);
        if (A.tap_acc && canon >= 0) *(int4*)(A.tap_acc + (size_t)canon * N + n0) = make_int4(a0, a1, a2, a3);
        if (EPI == EPI_QKV || EPI == EPI_FC1) {
            if (EPI == EPI_FC1) { f0 = gelu_scaled(f0, gelu_lds); f1 = gelu_scaled(f1, gelu_lds); f2 = gelu_scaled(f2, gelu_lds); f3 = gelu_scaled(f3, gelu_lds); }
            const QDev& q = A.q[branch][EPI == EPI_QKV ? n0 / G.C : 0];
            int code = pack4(quant_code(f0, q), quant_code(f1, q), quant_code(f2, q), quant_code(f3, q));
            *(int*)(A.out8 + (size_t)row * N + n0) = code;
            if (A.tap_code && canon >= 0) *(int*)(A.tap_code + (size_t)canon * N + n0) = code;
        } else if (EPI == EPI_PROJ) {
            float4 sc = make_float4(0.f, 0.f, 0.f, 0.f);
            if (pix >= 0) sc = *(const float4*)(A.x + (size_t)pix * N + n0);
            float4 o = make_float4(f0 + sc.x, f1 + sc.y, f2 + sc.z, f3 + sc.w);
            *(float4*)(A.outf + (size_t)row * N + n0) = o;
            if (A.tap_f && canon >= 0) *(float4*)(A.tap_f + (size_t)canon * N + n0) = o;
        } else {   // EPI_FC2: second residual and scatter back to the map
            float4 h = *(const float4*)(A.resid + (size_t)row * N + n0);
            float4 o = make_float4(f0 + h.x, f1 + h.y, f2 + h.z, f3 + h.w);
            if (pix >= 0) *(float4*)(A.y + (size_t)pix * N + n0) = o;
            if (A.tap_f && canon >= 0) *(float4*)(A.tap_f + (size_t)canon * N + n0) = o;
        }
    }
}

// One workgroup per 64-row tile and group of output blocks (all of them once the tiles alone fill the chip; on few
// rows, e.g. 20 row tiles at C = 768 and batch 1, groups of four).  The tile's activation rows are read once, 16 contiguous bytes per lane, and laid out in LDS as
// MFMA operand fragments (the row-major codes read directly as operands are 16 bytes from each of 32 rows per
// load, a quarter of every cache line touched); wave w computes the output blocks first + w, first + w + 4, ...
// of the group: weight fragments stream through a ring of loads in flight, the B operand comes from LDS.
// K up to 2048 stays whole in LDS for a 64-row tile, K up to 4096 for a 32-row tile; longer K passes in chunks.
constexpr int GEMM_TILE_MAX_K = 2048;      // 64 rows x K bytes of LDS
// KMAX: bytes of K the instantiation's LDS holds per row (a longer K goes through in chunks of A.kchunk <= KMAX); RT: rows per tile,
// 64 or, so that a long K fits LDS whole, 32
template <int EPI, int KMAX, int RT = ROW_TILE>
__global__ __launch_bounds__(256) void gemm_tile_kernel(Geom G, GemmArgs A)
{
    constexpr int RB = RT / 32;
    __shared__ v4i afr[RT * KMAX / 16];                                // [row blocks][chunk slabs][64 lanes]
    __shared__ float4 gtab[EPI == EPI_FC1 ? GELU_K : 1];
    constexpr int D = 8;                                               // weight fragments in flight per wave
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, j = lane & 31, g = lane >> 5;
    const int row0 = blockIdx.x * RT;
    const int branch = row0 >= G.base_lo ? 1 : 0;
    const int K = A.K, ks_n = K / 32, NB = A.N / 32;
    const int kch = A.kchunk, cs = kch / 32, n_ch = K / kch, per_row = kch / 16;       // chunk bytes (a divisor of K, at most KMAX), slabs per chunk, chunks
    auto stage = [&](int ch) {     // piece (row r, 16-byte chunk q) -> fragment (r/32, q/2), lane (r%32, q%2)
        for (int p = tid; p < RT * per_row; p += 256) {
            const int r = p / per_row, q = p - r * per_row;
            afr[((r >> 5) * cs + (q >> 1)) * 64 + (q & 1) * 32 + (r & 31)] = *(const v4i*)(A.A + (size_t)(row0 + r) * K + ch * kch + q * 16);
        }
    };
    if (EPI == EPI_FC1) gelu_stage_table(gtab, A.gelu_tab, tid, 256);
    const float4* gelu_lds = gtab;
    int pix[RB], canon[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        canon[rb] = A.row_canon[row0 + rb * 32 + j];
        pix[rb] = (EPI == EPI_PROJ || EPI == EPI_FC2) ? A.row_pix[row0 + rb * 32 + j] : 0;
    }
    if (n_ch == 1) stage(0);                                           // the whole K stays for every output block
    __syncthreads();
    const int nb_lo = blockIdx.y * A.nb_per_block, nb_hi = min(nb_lo + A.nb_per_block, NB);
    for (int nb0 = nb_lo; nb0 < nb_hi; nb0 += 4) {                     // the same trips for every wave: barriers inside
        const int nb = min(nb0 + wave, NB - 1);
        const bool active = nb0 + wave < nb_hi;
        const v4i* wp = A.Wp + (size_t)nb * ks_n * 64 + lane;
        v4i rw[D];
#pragma unroll
        for (int d = 0; d < D; ++d) rw[d] = wp[min(d, ks_n - 1) * 64];  // K may hold fewer than D slabs: the last one again (unused)
        v16i c0, c1;                                                     // c1: the second row block (RT = 64)
        {   // accumulators start at -zp_in * colsum(W[n,:])
            const int* nc = A.negcorr[branch] + nb * 32 + g * 4;
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                int4 t = *(const int4*)(nc + qd * 8);
                c0[qd * 4 + 0] = t.x; c0[qd * 4 + 1] = t.y; c0[qd * 4 + 2] = t.z; c0[qd * 4 + 3] = t.w;
            }
            c1 = c0;
        }
#pragma unroll 1
        for (int ch = 0; ch < n_ch; ++ch) {
            if (n_ch > 1) {
                if (ch > 0 || nb0 > nb_lo) __syncthreads();             // the previous chunk is no longer read
                stage(ch);
                __syncthreads();
            }
#pragma unroll 1
            for (int k0 = 0; k0 < cs; k0 += D) {
#pragma unroll
                for (int d = 0; d < D; ++d) {
                    const v4i w = rw[d];
                    rw[d] = wp[min(ch * cs + k0 + D + d, ks_n - 1) * 64]; // past the end: the last slab again (unused)
                    if (k0 + d < cs) {                                   // wave-uniform: the last turn may be partial
                        c0 = mfma32(w, afr[(k0 + d) * 64 + lane], c0);
                        if (RB == 2) c1 = mfma32(w, afr[(cs + k0 + d) * 64 + lane], c1);
                    }
                }
            }
        }
        if (active) {
            epilogue<EPI>(A, G, branch, row0 + j, nb, g, c0, pix[0], canon[0], gelu_lds);
            if (RB == 2) epilogue<EPI>(A, G, branch, row0 + 32 + j, nb, g, c1, pix[RB - 1], canon[RB - 1], gelu_lds);
        }
    }
}

// ------------------------------------------------------------------ attention core
// For one (window, head) held by one wave.  S^T = K Q^T (A operand = key rows, B operand =
// query columns) leaves a lane with one query per query block and the keys in registers,
// so the softmax reduces in registers; the packed P codes are then directly the B operand
// of O^T = V^T P^T.  qf/kf: lane = token tb*32+j, 16 bytes = the lane half's 16 dims (any
// mapping, the same for q and k).  vt: lane = dim j, byte r of slab kb = V[kb*32 +
// mfma_row(r,g)][j], zero for keys >= 49.  Returns the raw P.V sums (lane = query, register
// r = dim mfma_row(r,g)).  The wave runs NIB query blocks starting at block ib0 (both, or one of the
// two when a pair of waves shares the head).
struct AttnCore {
    const PolyCoef* poly;
    const float* bq;          // (bias + mask) * log2e of query j of query block ib0 at key g*4, in the [49 keys][64 queries]
                              // table of this head and mask type: key k + g*4, query block ib0 + ib is bq[k * 64 + ib * 32]
    float m2;
    QDev qp;
    int32_t* tap_s;           // already offset to this (slot, head): [49][49]
    int8_t* tap_p;
};

template <bool TAPS, int NIB>
__device__ __forceinline__ void attention_core(const v4i (&qf)[NIB], const v4i (&kf)[2], const v4i (&vt)[2],
                                               const AttnCore& A, int j, int g, int ib0, v16i (&o)[NIB])
{
    const v16i zero16 = {0};
#pragma unroll
    for (int ib = 0; ib < NIB; ++ib) {
        const int qi = (ib0 + ib) * 32 + j;                               // this lane's query
        v16i s[2];                                                        // S^T tiles of this query block, per key block
        s[0] = mfma32(kf[0], qf[ib], zero16);
        s[1] = mfma32(kf[1], qf[ib], zero16);
        float lg[2][16];
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = kb * 32 + (r >> 2) * 8 + (r & 3);         // + g*4
                float v = -INFINITY;
                if (key < TOK) {                                          // valid for at least one half
                    const int kk = key + g * 4;
                    if (kk < TOK) v = fmaf((float)s[kb][r], A.m2, A.bq[key * 64 + ib * 32]);
                    mx = fmaxf(mx, v);
                    if (TAPS && kk < TOK && qi < TOK && A.tap_s) A.tap_s[qi * TOK + kk] = s[kb][r];
                }
                lg[kb][r] = v;
            }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        double den = 0.0;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = kb * 32 + (r >> 2) * 8 + (r & 3);
                if (key < TOK) {
                    const int kk = key + g * 4;
                    float e = kk < TOK ? exp2_pinned(lg[kb][r] - mx, *A.poly) : 0.0f;
                    lg[kb][r] = e;
                    den += (double)e;
                }
            }
        den += __shfl_xor(den, 32, 64);
        const float rden = 1.0f / (float)den;
        v4i pk[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            int wd[4];
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                int c[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int r = qd * 4 + e, key = kb * 32 + qd * 8 + e;
                    c[e] = 0;
                    if (key < TOK) {
                        const int kk = key + g * 4;
                        if (kk < TOK) {
                            c[e] = quant_code(lg[kb][r] * rden, A.qp);
                            if (TAPS && qi < TOK && A.tap_p) A.tap_p[qi * TOK + kk] = (int8_t)c[e];
                        }
                    }
                }
                wd[qd] = pack4(c[0], c[1], c[2], c[3]);
            }
            pk[kb] = (v4i){wd[0], wd[1], wd[2], wd[3]};
        }
        o[ib] = mfma32(vt[0], pk[0], zero16);
        o[ib] = mfma32(vt[1], pk[1], o[ib]);
    }
}

// zero-point correction, dequantization and requantization of the P.V sums; writes the codes
// of head `head` for the window's tokens to out[row0 + token][C] (and the taps).  zcsum[d] = zp * sum of
// the V codes of dim d over the keys, formed once per dim by the caller (an integer multiply is a
// quarter-rate instruction; inside the loop it would be one per output element).
template <bool TAPS, int NIB>
__device__ __forceinline__ void attention_store(const v16i (&o)[NIB], const int* zcsum, const QDev& qo, float m_o,
                                                int j, int g, int ib0, int head, int C, int8_t* out, int row0, int32_t* tap_o,
                                                int8_t* tap_code, size_t canon_row0, int pack = 0)
{
#pragma unroll
    for (int ib = 0; ib < NIB; ++ib) {
        const int qi = (ib0 + ib) * 32 + j;
        if (qi < TOK) {
            int code[4];
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                const int d0 = qd * 8 + g * 4;
                const int4 cz = *(const int4*)(zcsum + d0);
                int a0 = o[ib][qd * 4 + 0] - cz.x, a1 = o[ib][qd * 4 + 1] - cz.y;
                int a2 = o[ib][qd * 4 + 2] - cz.z, a3 = o[ib][qd * 4 + 3] - cz.w;
                code[qd] = pack4(quant_code((float)a0 * m_o, qo), quant_code((float)a1 * m_o, qo),
                                 quant_code((float)a2 * m_o, qo), quant_code((float)a3 * m_o, qo));
                const int ch = head * HD + d0;
                if (pack == 0) *(int*)(out + (size_t)(row0 + qi) * C + ch) = code[qd];
                size_t ci = (canon_row0 + qi) * C + ch;
                if (TAPS && tap_o) *(int4*)(tap_o + ci) = make_int4(a0, a1, a2, a3);
                if (TAPS && tap_code) *(int*)(tap_code + ci) = code[qd];
            }
            if (pack == 1) {                       // out = first packed row of the region, row0 = row inside it
                int8_t* rowp = out + (size_t)(row0 + qi) * (C / 2) + head * 16 + g * 4;
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    const int lo = (code[2 * p] ^ 0x08080808) & 0x0f0f0f0f, hi = (code[2 * p + 1] ^ 0x08080808) & 0x0f0f0f0f;
                    *(int*)(rowp + p * 8) = lo | (hi << 4);
                }
            } else if (pack == 2) {
                int w = 0;
#pragma unroll
                for (int qd = 0; qd < 4; ++qd) w |= ((code[qd] ^ 0x02020202) & 0x03030303) << (2 * qd);
                *(int*)(out + (size_t)(row0 + qi) * (C / 4) + head * 8 + g * 4) = w;
            }
        }
    }
}

// slot (high group of all images first, then the low group) -> branch, first row, canonical slot
__device__ __forceinline__ void slot_info(const Geom& G, int slot, int& branch, int& row0, int& canon_slot)
{
    const int n_hi = G.B * G.k_hi;
    if (slot < n_hi) { int b = slot / G.k_hi; branch = 0; row0 = slot * TOK; canon_slot = b * G.nW + (slot - b * G.k_hi); }
    else { int s = slot - n_hi, b = s / G.k_lo; branch = 1; row0 = G.base_lo + s * TOK; canon_slot = b * G.nW + G.k_hi + (s - b * G.k_lo); }
}

__device__ __forceinline__ int mask_type(const Geom& G, int w)
{
    if (G.shift == 0) return 0;
    int wr = w / G.nWc, wc = w - wr * G.nWc;
    return (wr == G.Hp / WS - 1 ? 2 : 0) + (wc == G.nWc - 1 ? 1 : 0);
}

// ------------------------------------------------------------------ K4 attention (unfused path)
// One wave per (window slot, head); q, k, v codes come from the row-major QKV buffer, V^T
// fragments from a transposing read of V staged in LDS.
__global__ __launch_bounds__(256) void attn_kernel(Geom G, AttnArgs A)
{
    __shared__ __attribute__((aligned(16))) int8_t vs[4][64 * HD];       // V tile per wave, [key][dim]
    __shared__ __attribute__((aligned(16))) int csum[4][HD];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, j = lane & 31, g = lane >> 5;
    const int item = blockIdx.x * 4 + wave;                              // slot * heads + head
    if (item >= G.n_slots * G.heads) return;
    const int slot = item / G.heads, head = item - slot * G.heads;
    int branch, row0, canon_slot;
    slot_info(G, slot, branch, row0, canon_slot);
    const int mtype = mask_type(G, A.perm[canon_slot]);
    const int C3 = 3 * G.C;
    const int8_t* base = A.qkv + (size_t)row0 * C3 + head * HD + g * 16;
    const v4i zero4 = {0, 0, 0, 0};
    v4i qf[2], kf[2];
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        int t = tb * 32 + j;
        qf[tb] = t < TOK ? *(const v4i*)(base + (size_t)t * C3) : zero4;
        kf[tb] = t < TOK ? *(const v4i*)(base + (size_t)t * C3 + G.C) : zero4;
        v4i vv = t < TOK ? *(const v4i*)(base + (size_t)t * C3 + 2 * G.C) : zero4;
        *(v4i*)(&vs[wave][t * HD + g * 16]) = vv;
    }
    __builtin_amdgcn_s_waitcnt(0);
    __builtin_amdgcn_wave_barrier();
    v4i vt[2];
    int cs = 0;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
        int wd[4];
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            int c[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) c[e] = vs[wave][(kb * 32 + qd * 8 + g * 4 + e) * HD + j];
            wd[qd] = pack4(c[0], c[1], c[2], c[3]);
            cs = __builtin_amdgcn_sdot4(wd[qd], 0x01010101, cs, false);
        }
        vt[kb] = (v4i){wd[0], wd[1], wd[2], wd[3]};
    }
    cs += __shfl_xor(cs, 32, 64);
    if (g == 0) csum[wave][j] = A.qp[branch].zp * cs;
    AttnCore core;
    core.poly = &A.poly;
    core.bq = A.bias2 + ((size_t)(mtype * G.heads + head) * TOK) * 64 + g * 4 * 64 + j;
    core.m2 = A.m2[branch];
    core.qp = A.qp[branch];
    const size_t tb = ((size_t)canon_slot * G.heads + head) * TOK * TOK;
    core.tap_s = A.tap_s ? A.tap_s + tb : nullptr;
    core.tap_p = A.tap_p ? A.tap_p + tb : nullptr;
    v16i o[2];
    attention_core<true, 2>(qf, kf, vt, core, j, g, 0, o);
    __builtin_amdgcn_s_waitcnt(0);
    __builtin_amdgcn_wave_barrier();
    attention_store<true, 2>(o, csum[wave], A.qo[branch], A.m_o[branch], j, g, 0, head, G.C, A.out, row0, A.tap_o, A.tap_code,
                    (size_t)canon_slot * TOK);
}

// ------------------------------------------------------------------ fused window kernel
// One workgroup per window slot (HG = 1) or per half of a window's heads (HG = 2: few windows, or more heads
// than a workgroup has waves; both halves repeat the gather + LN1 phase), one wave per head (QS = 1, NH waves)
// or a pair of waves per head (QS = 2: each wave projects one 32-token block to q, k and v, the pair exchanges
// k and v through LDS, and each runs the attention of its own query block: half the chain of dependent steps):
//   gather (shift folded into the index map) + LN1 + quantize, shared through LDS as MFMA
//   fragments -> per head: q, k (transposed product, lane = token) and v (plain product, lane =
//   dim) straight into operand registers -> attention core -> codes of the attention output.
constexpr int WIN_WAVES_PER_EU = 3;
template <int NH, int HG, int QS>
struct WinCfg {
    // lanes per token in the LN phase: one per wave (3 ... 16), so that the 49 tokens fit one pass
    // with about three quarters of the lanes busy; a wave holds 64/LPT whole groups
    static constexpr int LPT = NH * QS;
    static constexpr int GPW = 64 / LPT;                             // groups (tokens) per wave
    static constexpr int NV = NH * HG * 32 / (4 * LPT);              // float4 per lane = 8 * HG / QS
};
constexpr int win_waves_per_eu(int NH, int HG, int QS) { return QS == 2 ? (NH * HG > 8 ? 3 : 4) : (HG == 2 && NH <= 8) ? 2 : WIN_WAVES_PER_EU; }

// word offsets inside the window kernel's parameter block of one branch (see WinArgs::params)
template <int C> struct WinPrm {
    static constexpr int LN_G = 0, LN_B = C, M = 2 * C, B = 5 * C, NC = 8 * C, WORDS = 11 * C;
};

template <int NH, bool TAPS, bool SCORED, int HG = 1, int QS = 1>
__global__ __launch_bounds__(NH * QS * 64) __attribute__((amdgpu_waves_per_eu(win_waves_per_eu(NH, HG, QS)))) void window_kernel(Geom G, WinArgs A)
{
    constexpr int NHT = NH * HG;                                         // heads of the block; this workgroup runs NH of them
    constexpr int NW = NH * QS, NTB = 2 / QS;                            // waves; token blocks a wave projects and attends for
    constexpr int C = NHT * 32, KS = NHT, LPT = WinCfg<NH, HG, QS>::LPT, NV = WinCfg<NH, HG, QS>::NV, NT = NW * 64;
    constexpr int GPW = WinCfg<NH, HG, QS>::GPW;
    using PR = WinPrm<C>;
    const int widx = HG == 1 ? blockIdx.x : blockIdx.x / HG, hg = HG == 1 ? 0 : blockIdx.x % HG;
    static_assert(NW * GPW >= TOK, "one pass must cover the window");
    __shared__ v4i a1s[2 * KS * 64];                                     // LN1 codes as fragments [token block][k slab][lane]
    __shared__ __attribute__((aligned(16))) float prm[PR::WORDS];        // this branch's LN1 affine and QKV epilogue constants
    __shared__ __attribute__((aligned(16))) int csum[NW][HD];
    __shared__ v4i kvx[QS == 2 ? NH * 4 * 64 : 1];                       // k and v operands of a wave pair [head][k|v][token block][lane]
    __shared__ int csp[QS == 2 ? NH * 2 * HD : 1];                       // V column sums of each token block [head][block][dim]
    __shared__ int red[NW];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, j = lane & 31, g = lane >> 5;
    const int hw = QS == 1 ? wave : wave >> 1, tb0 = QS == 1 ? 0 : wave & 1;   // head inside the workgroup, first token block
    const int head = hg * NH + hw;
    constexpr bool HOIST = KS <= 8;
    constexpr int RING = 6;
    auto weights_of = [&](int which) { return A.Wqkv + (size_t)(which * NHT + head) * KS * 64 + lane; };
    // SCORED: the workgroup is given a window and finds its own place in the selection (its rank
    // under the total order of the scores); otherwise it is given a slot and looks the window up.
    int branch = 0, row0 = 0, canon_slot = 0, w, bimg;
    if (SCORED) {
        bimg = widx / G.nW;
        w = widx - bimg * G.nW;
    } else if (widx < G.n_slots) {
        slot_info(G, widx, branch, row0, canon_slot);
        w = A.perm[canon_slot];
        bimg = canon_slot / G.nW;
    } else {                              // workgroups past the computed slots: pruned windows (Sec. 3.4), features forwarded
        if (hg != 0) return;
        const int kept = G.k_hi + G.k_lo, q = widx - G.n_slots, b = q / (G.nW - kept);
        const int wp = A.perm[b * G.nW + kept + (q - b * (G.nW - kept))];
        const int wr = wp / G.nWc, wc = wp - wr * G.nWc;
        for (int i = tid; i < TOK * (C / 4); i += NT) {
            const int tt = i / (C / 4), k = i - tt * (C / 4), tr = tt / WS, tc = tt - tr * WS;
            int pr = wr * WS + tr + G.shift; if (pr >= G.Hp) pr -= G.Hp;
            int pc = wc * WS + tc + G.shift; if (pc >= G.Wp) pc -= G.Wp;
            if (pr < G.H && pc < G.W) {
                const size_t off = ((size_t)(b * G.H + pr) * G.W + pc) * C + k * 4;
                *(float4*)(A.y + off) = *(const float4*)(A.x + off);
            }
        }
        return;
    }
    // The rows that pad each region to whole tiles belong to no window: the first workgroup marks them
    // (pixel -1, slot-major row -1) for the kernels of the seven-kernel path, which read the marks of every row.
    if (blockIdx.x == 0) {
        for (int r = G.rows_hi + tid; r < G.base_lo; r += NT) { A.row_pix[r] = -1; A.row_canon[r] = -1; }
        for (int r = G.base_lo + G.rows_lo + tid; r < G.rows_total; r += NT) { A.row_pix[r] = -1; A.row_canon[r] = -1; }
    }
    int* a1w = (int*)a1s;
    // dword index of (token slot s, channel c with c%4==0) in the fragment layout (k = channel, natural order)
    auto frag_dw = [&](int s, int c) { return ((((s >> 5) * KS + (c >> 5)) * 64 + ((c & 31) >> 4) * 32 + (s & 31)) << 2) + ((c & 15) >> 2); };
    for (int i = tid; i < 15 * (C / 4); i += NT) a1w[frag_dw(TOK + i / (C / 4), (i % (C / 4)) * 4)] = 0;
    const int grp = lane / LPT, sub = lane - grp * LPT, first = lane - sub;
    const int t = grp < GPW ? wave * GPW + grp : TOK;                    // lanes beyond the last whole group idle
    int pix = -1;
    float4 v[NV];
    if (t < TOK) {                                                       // gather: the loads need the window only
        const int wr = w / G.nWc, wc = w - wr * G.nWc, tr = t / WS, tc = t - tr * WS;
        int pr = wr * WS + tr + G.shift; if (pr >= G.Hp) pr -= G.Hp;
        int pc = wc * WS + tc + G.shift; if (pc >= G.Wp) pc -= G.Wp;
        pix = (pr < G.H && pc < G.W) ? (bimg * G.H + pr) * G.W + pc : -1;
        if (pix >= 0) {
            const float* src = A.x + (size_t)pix * C;
#pragma unroll
            for (int k = 0; k < NV; ++k) v[k] = *(const float4*)(src + (k * LPT + sub) * 4);
        }
    }
    if (SCORED) {
        const double* sc = A.scores + (size_t)bimg * G.nW;
        const double sw = sc[w];
        int cnt = 0;
        for (int base = 0; base < G.nW; base += 8 * NT) {                // eight loads in flight per thread
            double sv[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) { const int u = base + tid + k * NT; sv[k] = sc[min(u, G.nW - 1)]; }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int u = base + tid + k * NT;
                cnt += (u < G.nW && ranked_before(sv[k], u, sw, w, 0)) ? 1 : 0;
            }
        }
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) cnt += __shfl_xor(cnt, o, 64);
        if (lane == 0) red[wave] = cnt;
        __syncthreads();
        int rank = 0;
#pragma unroll
        for (int k = 0; k < NW; ++k) rank += red[k];
        rank = __builtin_amdgcn_readfirstlane(rank);                      // the same in every lane: what follows from it stays scalar
        if (tid == 0 && hg == 0) A.perm_out[(size_t)bimg * G.nW + rank] = w;
        if (rank >= G.k_hi + G.k_lo) {                                    // pruned (Sec. 3.4): forward the features
            if (pix >= 0 && hg == 0) {
                float* dst = A.y + (size_t)pix * C;
#pragma unroll
                for (int k = 0; k < NV; ++k) *(float4*)(dst + (k * LPT + sub) * 4) = v[k];
            }
            return;                                                       // the whole workgroup
        }
        canon_slot = bimg * G.nW + rank;
        if (rank < G.k_hi) { branch = 0; row0 = (bimg * G.k_hi + rank) * TOK; }
        else { branch = 1; row0 = G.base_lo + (bimg * G.k_lo + rank - G.k_hi) * TOK; }
    }
    {   // the branch is known: its parameter block goes to LDS (requested now, so that it travels with the map)
        const float4* src = (const float4*)A.params[branch];
        constexpr int PV = PR::WORDS / 4, PVT = (PV + NT - 1) / NT;
        float4 pv[PVT];
#pragma unroll
        for (int k = 0; k < PVT; ++k) pv[k] = src[min(tid + k * NT, PV - 1)];
#pragma unroll
        for (int k = 0; k < PVT; ++k) if (tid + k * NT < PV) ((float4*)prm)[tid + k * NT] = pv[k];
    }
    __syncthreads();                                                     // parameter block visible
    const int* prmi = (const int*)prm;
    if (t < TOK) {
        const int canon = canon_slot * TOK + t;
        if (sub == 0 && hg == 0) { A.row_pix[row0 + t] = pix; A.row_canon[row0 + t] = canon; }
        if (pix >= 0) {
            token_layernorm<LPT, NV>(v, C, A.eps, prm + PR::LN_G, prm + PR::LN_B, sub, first);
        } else {
#pragma unroll
            for (int k = 0; k < NV; ++k) v[k] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        const QDev q = A.q_in[branch];
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const int ch = (k * LPT + sub) * 4;
            int code = pack4(quant_code(v[k].x, q), quant_code(v[k].y, q), quant_code(v[k].z, q), quant_code(v[k].w, q));
            a1w[frag_dw(t, ch)] = code;
            if (TAPS && A.tap_a1 && hg == 0) *(int*)(A.tap_a1 + (size_t)canon * C + ch) = code;
        }
    }
    __syncthreads();
    // Operand handling.  Up to eight heads the LN1 fragments of both token blocks and the weight
    // fragments of one output block sit in registers; beyond that the B operand is read from LDS
    // inside the chain and the weight fragments stream through a short ring.
    v4i bf[NTB][HOIST ? KS : 1];
    if (HOIST) {
#pragma unroll
        for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) bf[tb][ks] = a1s[((tb0 + tb) * KS + ks) * 64 + lane];
    }
    // streaming form: acc[tb] += (weights as A operand ? W * act^T : act * W^T) over the whole K
    auto chain = [&](const v4i* wp, v16i* acc, bool weights_first) {
        v4i ring[RING];
#pragma unroll
        for (int d = 0; d < RING; ++d) ring[d] = wp[d * 64];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const v4i wv = ring[ks % RING];
            if (ks + RING < KS) ring[ks % RING] = wp[(ks + RING) * 64];
#pragma unroll
            for (int tb = 0; tb < NTB; ++tb) {
                const v4i xv = a1s[((tb0 + tb) * KS + ks) * 64 + lane];
                acc[tb] = weights_first ? mfma32(wv, xv, acc[tb]) : mfma32(xv, wv, acc[tb]);
            }
        }
    };
    const size_t canon_row0 = (size_t)canon_slot * TOK;
    v4i qk[2][NTB];                                                      // [q|k][token block]
#pragma unroll
    for (int which = 0; which < 2; ++which) {
        const int nb = which * NHT + head;
        const QDev qq = A.q_qkv[branch][which];
        const v4i* wp = weights_of(which);
        auto start = [&](v16i& acc) {                                     // accumulators start at -zp * colsum
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                const int4 t4 = *(const int4*)(prmi + PR::NC + nb * 32 + qd * 8 + g * 4);
                acc[qd * 4 + 0] = t4.x; acc[qd * 4 + 1] = t4.y; acc[qd * 4 + 2] = t4.z; acc[qd * 4 + 3] = t4.w;
            }
        };
        auto finish = [&](int tb, const v16i& acc) {                      // dequantize, requantize, keep as operand
            int wd[4];
            const int tok = (tb0 + tb) * 32 + j;
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                const int n0 = nb * 32 + qd * 8 + g * 4;
                const float4 m = *(const float4*)(prm + PR::M + n0), bs = *(const float4*)(prm + PR::B + n0);
                const int a0 = acc[qd * 4 + 0], a1 = acc[qd * 4 + 1], a2 = acc[qd * 4 + 2], a3 = acc[qd * 4 + 3];
                wd[qd] = pack4(quant_code(fmaf((float)a0, m.x, bs.x), qq), quant_code(fmaf((float)a1, m.y, bs.y), qq),
                               quant_code(fmaf((float)a2, m.z, bs.z), qq), quant_code(fmaf((float)a3, m.w, bs.w), qq));
                if (TAPS && tok < TOK) {
                    if (A.tap_acc) *(int4*)(A.tap_acc + (canon_row0 + tok) * (3 * C) + n0) = make_int4(a0, a1, a2, a3);
                    if (A.tap_qkv) *(int*)(A.tap_qkv + (canon_row0 + tok) * (3 * C) + n0) = wd[qd];
                }
            }
            qk[which][tb] = (v4i){wd[0], wd[1], wd[2], wd[3]};
        };
        if (HOIST) {
            v4i wf[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) wf[ks] = wp[ks * 64];
#pragma unroll
            for (int tb = 0; tb < NTB; ++tb) {
                v16i acc;
                start(acc);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) acc = mfma32(wf[ks], bf[tb][ks], acc);
                finish(tb, acc);
            }
        } else {
            v16i acc[NTB];
            start(acc[0]);
            if (NTB == 2) acc[NTB - 1] = acc[0];
            chain(wp, acc, true);
#pragma unroll
            for (int tb = 0; tb < NTB; ++tb) finish(tb, acc[tb]);
        }
    }
    v4i vt[2];
    {
        const int nb = 2 * NHT + head, n = nb * 32 + j;                   // this lane's output channel (dim j of the head)
        const v4i* wp = weights_of(2);
        const float m = prm[PR::M + n], bs = prm[PR::B + n];
        const int nc = prmi[PR::NC + n];
        const QDev qv = A.q_qkv[branch][2];
        int cs = 0;
        auto finish = [&](int tb, const v16i& acc) {
            int wd[4];
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                int c[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int tok = (tb0 + tb) * 32 + qd * 8 + g * 4 + e;
                    c[e] = 0;
                    if (QS == 2 || tb * 32 + qd * 8 + e < TOK) {      // known at compile time when the wave runs both blocks
                        if (tok < TOK) {
                            c[e] = quant_code(fmaf((float)acc[qd * 4 + e], m, bs), qv);
                            if (TAPS && A.tap_acc) A.tap_acc[(canon_row0 + tok) * (3 * C) + n] = acc[qd * 4 + e];
                            if (TAPS && A.tap_qkv) A.tap_qkv[(canon_row0 + tok) * (3 * C) + n] = (int8_t)c[e];
                        }
                    }
                }
                wd[qd] = pack4(c[0], c[1], c[2], c[3]);
                cs = __builtin_amdgcn_sdot4(wd[qd], 0x01010101, cs, false);
            }
            vt[tb] = (v4i){wd[0], wd[1], wd[2], wd[3]};
        };
        if (HOIST) {
            v4i wf[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) wf[ks] = wp[ks * 64];
#pragma unroll
            for (int tb = 0; tb < NTB; ++tb) {
                v16i acc;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[r] = nc;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) acc = mfma32(bf[tb][ks], wf[ks], acc);      // rows = tokens, columns = dims
                finish(tb, acc);
            }
        } else {
            v16i acc[NTB];
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[0][r] = nc;
            if (NTB == 2) acc[NTB - 1] = acc[0];
            chain(wp, acc, false);
#pragma unroll
            for (int tb = 0; tb < NTB; ++tb) finish(tb, acc[tb]);
        }
        cs += __shfl_xor(cs, 32, 64);
        if (QS == 1) {
            if (g == 0) csum[wave][j] = A.qp[branch].zp * cs;
        } else {                                                          // the pair exchanges its halves of K, V and the sums
            kvx[((hw * 2 + 0) * 2 + tb0) * 64 + lane] = qk[1][0];
            kvx[((hw * 2 + 1) * 2 + tb0) * 64 + lane] = vt[0];
            if (g == 0) csp[(hw * 2 + tb0) * HD + j] = cs;
            __syncthreads();
            if (g == 0) csum[wave][j] = A.qp[branch].zp * (csp[(hw * 2) * HD + j] + csp[(hw * 2 + 1) * HD + j]);
        }
    }
    v4i kf[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
        kf[kb] = QS == 1 ? qk[1][kb % NTB] : kvx[((hw * 2 + 0) * 2 + kb) * 64 + lane];
        if (QS == 2) vt[kb] = kvx[((hw * 2 + 1) * 2 + kb) * 64 + lane];
    }
    AttnCore core;
    core.poly = &A.poly;
    core.bq = A.bias2 + ((size_t)(mask_type(G, w) * NHT + head) * TOK) * 64 + g * 4 * 64 + tb0 * 32 + j;
    core.m2 = A.m2[branch];
    core.qp = A.qp[branch];
    const size_t tbase = ((size_t)canon_slot * NHT + head) * TOK * TOK;
    core.tap_s = A.tap_s ? A.tap_s + tbase : nullptr;
    core.tap_p = A.tap_p ? A.tap_p + tbase : nullptr;
    v16i o[NTB];
    attention_core<TAPS, NTB>(qk[0], kf, vt, core, j, g, tb0, o);
    __builtin_amdgcn_s_waitcnt(0);
    __builtin_amdgcn_wave_barrier();
    const int pack = branch ? A.out_pack : 0;                            // the low region's rows may be packed (dense, after the high region)
    if (pack) attention_store<TAPS, NTB>(o, csum[wave], A.qo[branch], A.m_o[branch], j, g, tb0, head, C, A.out + (size_t)G.base_lo * C,
                                         row0 - G.base_lo, A.tap_o, A.tap_code, canon_row0, pack);
    else attention_store<TAPS, NTB>(o, csum[wave], A.qo[branch], A.m_o[branch], j, g, tb0, head, C, A.out, row0, A.tap_o, A.tap_code, canon_row0);
}

// ------------------------------------------------------------------ fused token kernel
// One workgroup per tile of 32 gathered rows, one wave per 32-channel block (NH = C/32 = 3, 4 or 8 waves; six and
// twelve waves run the wide form below):
//   proj + first residual (wave w owns channels 32w..32w+31, h stays in registers) -> LN2 with
//   statistics exchanged through LDS -> quantize -> FC1 (each wave 4 hidden blocks) + GELU +
//   quantize, codes to LDS as fragments -> FC2 + second residual -> scatter to the map.
// Latency is hidden by issuing loads a phase ahead: the per-branch parameter block (epilogue
// constants, LN2 affine) is staged in LDS once, weight fragments of the next MFMA chain are
// requested before the current epilogue starts.
// waves per SIMD the token kernel is compiled for: two workgroups per CU with eight waves each, four and five with
// four and three waves; measured: one more resident workgroup at eight waves takes the kernel from 122 to 96 us
// on 70756 rows, five waves per SIMD at three waves per workgroup gain nothing
constexpr int tok_waves_per_eu(int) { return 4; }
// word offsets inside the parameter block of one branch (see TokArgs::params)
template <int C> struct TokPrm {
    static constexpr int F = 4 * C;
    static constexpr int P_M = 0, P_B = C, P_NC = 2 * C, LN_G = 3 * C, LN_B = 4 * C, F2_M = 5 * C, F2_B = 6 * C,
                         F2_NC = 7 * C, F1_M = 8 * C, F1_B = 8 * C + F, F1_NC = 8 * C + 2 * F, WORDS = 8 * C + 3 * F;
};

template <int NH, bool TAPS>
__global__ __launch_bounds__(NH * 64) __attribute__((amdgpu_waves_per_eu(tok_waves_per_eu(NH), tok_waves_per_eu(NH)))) void token_kernel(Geom G, TokArgs A)
{
    constexpr int C = NH * 32, KS = NH, HB = 4 * NH, F = 4 * C, NT = NH * 64;
    using PR = TokPrm<C>;
    constexpr int PV = PR::WORDS / 4, PVT = (PV + NT - 1) / NT;       // float4 of the block, per thread
    constexpr int D2 = 4;                                            // FC2 weight fragments in flight
    constexpr bool EARLY_W1 = NH <= 4;                               // first FC1 weights requested at entry (register room permitting)
    __shared__ v4i a2s[KS * 64];
    __shared__ v4i gs[HB * 64];
    __shared__ double part[2][NH][32];
    __shared__ __attribute__((aligned(16))) float prm[PR::WORDS];
    __shared__ float4 gtab[GELU_K];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, j = lane & 31, g = lane >> 5;
    const int tile = blockIdx.x;
    const int row = tile * 32 + j;
    const int branch = tile * 32 >= G.base_lo ? 1 : 0;                 // a tile never straddles the regions: scalar
    const bool valid = branch ? (row - G.base_lo < G.rows_lo) : (row < G.rows_hi);
    const int nb = wave;
    // ---- loads that depend on nothing: parameter block, attention codes, first weight fragments
    static_assert(PVT <= 3, "the parameter block is staged with at most three loads per thread");
    const float4* psrc = (const float4*)A.params[branch];
    const float4 pv0 = psrc[tid];                                     // PV >= NT always; out-of-range threads re-read the last vector
    const float4 pv1 = psrc[min(tid + NT, PV - 1)];
    const float4 pv2 = psrc[min(tid + 2 * NT, PV - 1)];
    const int pix = valid ? A.row_pix[row] : -1;
    const size_t canon = (TAPS && valid) ? (size_t)A.row_canon[row] : 0;
    const bool tap_ok = TAPS && valid;
    v4i aof[KS], wpf[KS], w1f[KS];
    {
        const int pack = branch ? A.ao_pack : 0;                       // packed low-branch codes: scalar per tile
        const int8_t* ap = A.ao + (size_t)row * C + g * 16;
        const int8_t* pp = A.ao + (size_t)G.base_lo * C + (size_t)(row - G.base_lo) * (C >> pack);
        const v4i* wp = A.Wproj + (size_t)nb * KS * 64 + lane;
        const v4i* w1 = A.W1 + (size_t)wave * KS * 64 + lane;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            aof[ks] = pack ? unpack_codes(pp, pack, ks, g) : *(const v4i*)(ap + ks * 32);
            wpf[ks] = wp[ks * 64];
            if (EARLY_W1) w1f[ks] = w1[ks * 64];
        }
    }
    gelu_stage_table(gtab, A.gelu_tab, tid, NT);
    const float4* gelu_lds = gtab;
    ((float4*)prm)[tid] = pv0;
    if (PVT > 1 && tid + NT < PV) ((float4*)prm)[tid + NT] = pv1;
    if (PVT > 2 && tid + 2 * NT < PV) ((float4*)prm)[tid + 2 * NT] = pv2;
    float4 sc[4];
#pragma unroll
    for (int qd = 0; qd < 4; ++qd)
        sc[qd] = pix >= 0 ? *(const float4*)(A.x + (size_t)pix * C + nb * 32 + qd * 8 + g * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
    __syncthreads();                                                  // parameter block visible
    const int* prmi = (const int*)prm;
    float h[16];
    {   // output projection + first residual
        v16i acc;
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            const int4 t4 = *(const int4*)(prmi + PR::P_NC + nb * 32 + qd * 8 + g * 4);
            acc[qd * 4 + 0] = t4.x; acc[qd * 4 + 1] = t4.y; acc[qd * 4 + 2] = t4.z; acc[qd * 4 + 3] = t4.w;
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) acc = mfma32(wpf[ks], aof[ks], acc);
        if (!EARLY_W1) {                                              // wide blocks: the first FC1 weights follow the projection chain
            const v4i* w1 = A.W1 + (size_t)wave * KS * 64 + lane;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) w1f[ks] = w1[ks * 64];
        }
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            const int n0 = nb * 32 + qd * 8 + g * 4;
            const float4 m = *(const float4*)(prm + PR::P_M + n0), bs = *(const float4*)(prm + PR::P_B + n0);
            h[qd * 4 + 0] = fmaf((float)acc[qd * 4 + 0], m.x, bs.x) + sc[qd].x;
            h[qd * 4 + 1] = fmaf((float)acc[qd * 4 + 1], m.y, bs.y) + sc[qd].y;
            h[qd * 4 + 2] = fmaf((float)acc[qd * 4 + 2], m.z, bs.z) + sc[qd].z;
            h[qd * 4 + 3] = fmaf((float)acc[qd * 4 + 3], m.w, bs.w) + sc[qd].w;
            if (tap_ok) {
                if (A.tap_acc_proj) *(int4*)(A.tap_acc_proj + canon * C + n0) = make_int4(acc[qd * 4], acc[qd * 4 + 1], acc[qd * 4 + 2], acc[qd * 4 + 3]);
                if (A.tap_h) *(float4*)(A.tap_h + canon * C + n0) = make_float4(h[qd * 4], h[qd * 4 + 1], h[qd * 4 + 2], h[qd * 4 + 3]);
            }
        }
    }
    {   // LN2: binary64 partial sums per (wave, token) through LDS, then normalise and quantize
        double s = 0.0;
#pragma unroll
        for (int r = 0; r < 16; r += 4) s += ((double)h[r] + (double)h[r + 1]) + ((double)h[r + 2] + (double)h[r + 3]);
        s += __shfl_xor(s, 32, 64);
        if (g == 0) part[0][wave][j] = s;
        __syncthreads();
        double tot = 0.0;
#pragma unroll
        for (int w2 = 0; w2 < NH; ++w2) tot += part[0][w2][j];
        const float mean = (float)(tot / (double)C);
        double q = 0.0;
#pragma unroll
        for (int r = 0; r < 16; r += 4) {
            double a = (double)h[r] - (double)mean, b = (double)h[r + 1] - (double)mean;
            double c = (double)h[r + 2] - (double)mean, d = (double)h[r + 3] - (double)mean;
            q += (a * a + b * b) + (c * c + d * d);
        }
        q += __shfl_xor(q, 32, 64);
        if (g == 0) part[1][wave][j] = q;
        __syncthreads();
        tot = 0.0;
#pragma unroll
        for (int w2 = 0; w2 < NH; ++w2) tot += part[1][w2][j];
        const float var = (float)(tot / (double)C);
        const float rstd = 1.0f / sqrtf(var + A.eps);
        const QDev qa = A.q_fc1in[branch];
        int wd[4];
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            const int n0 = nb * 32 + qd * 8 + g * 4;
            const float4 gm = *(const float4*)(prm + PR::LN_G + n0), bt = *(const float4*)(prm + PR::LN_B + n0);
            wd[qd] = pack4(quant_code(fmaf((h[qd * 4 + 0] - mean) * rstd, gm.x, bt.x), qa),
                           quant_code(fmaf((h[qd * 4 + 1] - mean) * rstd, gm.y, bt.y), qa),
                           quant_code(fmaf((h[qd * 4 + 2] - mean) * rstd, gm.z, bt.z), qa),
                           quant_code(fmaf((h[qd * 4 + 3] - mean) * rstd, gm.w, bt.w), qa));
            if (tap_ok && A.tap_a2) *(int*)(A.tap_a2 + canon * C + n0) = wd[qd];
        }
        a2s[nb * 64 + lane] = (v4i){wd[0], wd[1], wd[2], wd[3]};       // k slab nb, byte r = channel 32nb + mfma_row(r,g)
    }
    __syncthreads();
    v4i w2q[D2];                                                      // first FC2 weight fragments, requested during FC1
    const v4i* w2p = A.W2 + (size_t)nb * HB * 64 + lane;
    {   // FC1 + GELU + quantize for hidden blocks wave, wave+NH, ...
        v4i af[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) af[ks] = a2s[ks * 64 + lane];
        const QDev qg = A.q_fc2in[branch];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int hb = wave + NH * i;
            v16i acc;
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                const int4 t4 = *(const int4*)(prmi + PR::F1_NC + hb * 32 + qd * 8 + g * 4);
                acc[qd * 4 + 0] = t4.x; acc[qd * 4 + 1] = t4.y; acc[qd * 4 + 2] = t4.z; acc[qd * 4 + 3] = t4.w;
            }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) acc = mfma32(w1f[ks], af[ks], acc);
            if (i < 3) {                                              // weights of the next hidden block
                const v4i* w1 = A.W1 + (size_t)(hb + NH) * KS * 64 + lane;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) w1f[ks] = w1[ks * 64];
            } else {
#pragma unroll
                for (int d = 0; d < D2; ++d) w2q[d] = w2p[d * 64];
            }
            int wd[4];
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                const int n0 = hb * 32 + qd * 8 + g * 4;
                const float4 m = *(const float4*)(prm + PR::F1_M + n0), bs = *(const float4*)(prm + PR::F1_B + n0);
                wd[qd] = pack4(quant_code(gelu_scaled(fmaf((float)acc[qd * 4 + 0], m.x, bs.x), gelu_lds), qg),
                               quant_code(gelu_scaled(fmaf((float)acc[qd * 4 + 1], m.y, bs.y), gelu_lds), qg),
                               quant_code(gelu_scaled(fmaf((float)acc[qd * 4 + 2], m.z, bs.z), gelu_lds), qg),
                               quant_code(gelu_scaled(fmaf((float)acc[qd * 4 + 3], m.w, bs.w), gelu_lds), qg));
                if (tap_ok) {
                    if (A.tap_acc_fc1) *(int4*)(A.tap_acc_fc1 + canon * F + n0) = make_int4(acc[qd * 4], acc[qd * 4 + 1], acc[qd * 4 + 2], acc[qd * 4 + 3]);
                    if (A.tap_g) *(int*)(A.tap_g + canon * F + n0) = wd[qd];
                }
            }
            gs[hb * 64 + lane] = (v4i){wd[0], wd[1], wd[2], wd[3]};
        }
    }
    __syncthreads();
    {   // FC2 + second residual + scatter
        v16i acc;
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            const int4 t4 = *(const int4*)(prmi + PR::F2_NC + nb * 32 + qd * 8 + g * 4);
            acc[qd * 4 + 0] = t4.x; acc[qd * 4 + 1] = t4.y; acc[qd * 4 + 2] = t4.z; acc[qd * 4 + 3] = t4.w;
        }
#pragma unroll
        for (int hb = 0; hb < HB; ++hb) {
            const v4i w = w2q[hb % D2];
            if (hb + D2 < HB) w2q[hb % D2] = w2p[(hb + D2) * 64];
            acc = mfma32(w, gs[hb * 64 + lane], acc);
        }
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            const int n0 = nb * 32 + qd * 8 + g * 4;
            const float4 m = *(const float4*)(prm + PR::F2_M + n0), bs = *(const float4*)(prm + PR::F2_B + n0);
            float4 o4 = make_float4(fmaf((float)acc[qd * 4 + 0], m.x, bs.x) + h[qd * 4 + 0], fmaf((float)acc[qd * 4 + 1], m.y, bs.y) + h[qd * 4 + 1],
                                    fmaf((float)acc[qd * 4 + 2], m.z, bs.z) + h[qd * 4 + 2], fmaf((float)acc[qd * 4 + 3], m.w, bs.w) + h[qd * 4 + 3]);
            if (pix >= 0) *(float4*)(A.y + (size_t)pix * C + n0) = o4;
            if (tap_ok) {
                if (A.tap_acc_fc2) *(int4*)(A.tap_acc_fc2 + canon * C + n0) = make_int4(acc[qd * 4], acc[qd * 4 + 1], acc[qd * 4 + 2], acc[qd * 4 + 3]);
                if (A.tap_y) *(float4*)(A.tap_y + canon * C + n0) = o4;
            }
        }
    }
}

// ------------------------------------------------------------------ fused token kernel, wide form
// For six and twelve waves (C = 192, 384): one workgroup per tile of 32*RB gathered rows (RB 32-row blocks share
// every weight fragment, which divides the L2 -> CU weight traffic per row by RB), one wave per 32-channel block.
// Built for a small register footprint: the per-branch parameter block sits in LDS, the weight fragments of the whole kernel form ONE stream
// per wave (projection block, then per chunk the FC1 block and the FC2 fragments) that is requested RING
// fragments ahead across every phase boundary, and with twelve waves h is parked in the output map between the
// first and the second residual (the same thread writes and re-reads the same address) instead of in registers.
// The FFN runs in four chunks of NH hidden blocks: FC1 + GELU + quantize of a chunk goes to one of two LDS buffers,
// then FC2 accumulates that chunk.
template <int NH, int RB, bool TAPS>
__global__ __launch_bounds__(NH * 64) void token_wide_kernel(Geom G, TokArgs A)
{
    constexpr int C = NH * 32, KS = NH, HB = 4 * NH, F = 4 * C, NT = NH * 64;
    constexpr int RING = NH == 6 ? 6 : 8;                              // fragments in flight per wave
    constexpr bool PARK_H = (NH >= 12 || RB >= 4) && !TAPS;          // taps need h of padded tokens too, which have no pixel
    static_assert((2 * KS) % RING == 0 && RING <= KS, "phases 2k start at ring slot 0, phases 2k+1 at slot KS % RING");
    constexpr int SLOT_ODD = KS % RING;
    using PR = TokPrm<C>;
    __shared__ v4i actf[RB * KS * 64];                                 // [row block][k slab][lane]
    __shared__ v4i gs[2][NH * RB * 64];                                // [buffer][hidden block of the chunk][row block][lane]
    __shared__ double part[2][NH][32 * RB];
    __shared__ __attribute__((aligned(16))) float prm[PR::WORDS];
    __shared__ float4 gtab[GELU_K];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, j = lane & 31, g = lane >> 5;
    const int row_base = blockIdx.x * (32 * RB);
    const int branch = row_base >= G.base_lo ? 1 : 0;                 // a tile never straddles the regions: scalar
    const int nb = wave;
    const int* prmi = (const int*)prm;
    // The wave's weight stream, phase by phase (every phase has KS = NH fragments): projection block, FC1 block of
    // chunk 0, then per chunk c = 1..3 the FC1 block of chunk c followed by the FC2 fragments of chunk c-1, and the
    // FC2 fragments of chunk 3 at the end.  FC2 of a chunk is issued one chunk late so that its matrix work runs
    // under the GELU arithmetic of the next chunk.
    const v4i* wproj = A.Wproj + (size_t)nb * KS * 64 + lane;
    auto w1_of = [&](int chunk) { return A.W1 + ((size_t)(chunk * NH + wave) * KS) * 64 + lane; };
    auto w2_of = [&](int chunk) { return A.W2 + ((size_t)nb * HB + chunk * NH) * 64 + lane; };
    v4i ring[RING];
#pragma unroll
    for (int d = 0; d < RING; ++d) ring[d] = wproj[d * 64];            // the stream starts before anything else
    int pix[RB];
    bool valid[RB];
    size_t canon[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int row = row_base + rb * 32 + j;
        valid[rb] = branch ? (row - G.base_lo < G.rows_lo) : (row < G.rows_hi);
        pix[rb] = valid[rb] ? A.row_pix[row] : -1;
        canon[rb] = (TAPS && valid[rb]) ? (size_t)A.row_canon[row] : 0;
    }
    // stage the attention codes of the tile: piece p = (row r, 16-byte chunk q) -> fragment (r/32, q/2), lane (r%32, q%2)
    const int pack = branch ? A.ao_pack : 0;                           // packed low-branch codes: scalar per tile
    for (int p = tid; p < 32 * RB * (C / 16); p += NT) {
        const int r = p / (C / 16), q = p - r * (C / 16);
        actf[((r >> 5) * KS + (q >> 1)) * 64 + (q & 1) * 32 + (r & 31)] =
            pack ? unpack_codes(A.ao + (size_t)G.base_lo * C + (size_t)(row_base - G.base_lo + r) * (C >> pack), pack, q >> 1, q & 1)
                 : *(const v4i*)(A.ao + (size_t)(row_base + r) * C + q * 16);
    }
    {
        const float4* psrc = (const float4*)A.params[branch];
        for (int p = tid; p < PR::WORDS / 4; p += NT) ((float4*)prm)[p] = psrc[p];
    }
    gelu_stage_table(gtab, A.gelu_tab, tid, NT);
    // acc[rb] += W * operand^T over one phase.  Weights come from the ring (slot0 = ring slot of the phase's first
    // fragment); after fragment i is used, the fragment RING places further down the stream is requested: from this
    // phase (cur) or from the start of the next one (nxt, NULL at the end of the stream).  Operand fragment i of
    // row block rb: b[(rb*rb_stride + i*i_stride)*64 + lane].
    auto run = [&](int slot0, const v4i* cur, const v4i* nxt, const v4i* b, int rb_stride, int i_stride, v16i* acc) {
#pragma unroll
        for (int i = 0; i < KS; ++i) {
            const v4i wv = ring[(slot0 + i) % RING];
            if (i + RING < KS) ring[(slot0 + i) % RING] = cur[(i + RING) * 64];
            else if (nxt) ring[(slot0 + i) % RING] = nxt[(i + RING - KS) * 64];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) acc[rb] = mfma32(wv, b[(rb * rb_stride + i * i_stride) * 64 + lane], acc[rb]);
        }
    };
    auto start = [&](v16i* acc, int off) {                             // accumulators start at -zp * colsum
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            const int4 t4 = *(const int4*)(prmi + off + qd * 8 + g * 4);
            acc[0][qd * 4 + 0] = t4.x; acc[0][qd * 4 + 1] = t4.y; acc[0][qd * 4 + 2] = t4.z; acc[0][qd * 4 + 3] = t4.w;
        }
#pragma unroll
        for (int rb = 1; rb < RB; ++rb) acc[rb] = acc[0];
    };
    float4 sc[RB][4];                                                  // shortcut of the first residual, in flight during the projection
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int qd = 0; qd < 4; ++qd)
            sc[rb][qd] = pix[rb] >= 0 ? *(const float4*)(A.x + (size_t)pix[rb] * C + nb * 32 + qd * 8 + g * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
    __syncthreads();                                                  // staged codes, parameters and table visible
    float h[RB][16];
    {   // output projection + first residual
        v16i acc[RB];
        start(acc, PR::P_NC + nb * 32);
        run(0, wproj, w1_of(0), actf, KS, 1, acc);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                const int n0 = nb * 32 + qd * 8 + g * 4;
                const float4 m = *(const float4*)(prm + PR::P_M + n0), bs = *(const float4*)(prm + PR::P_B + n0);
                h[rb][qd * 4 + 0] = fmaf((float)acc[rb][qd * 4 + 0], m.x, bs.x) + sc[rb][qd].x;
                h[rb][qd * 4 + 1] = fmaf((float)acc[rb][qd * 4 + 1], m.y, bs.y) + sc[rb][qd].y;
                h[rb][qd * 4 + 2] = fmaf((float)acc[rb][qd * 4 + 2], m.z, bs.z) + sc[rb][qd].z;
                h[rb][qd * 4 + 3] = fmaf((float)acc[rb][qd * 4 + 3], m.w, bs.w) + sc[rb][qd].w;
                if (PARK_H && pix[rb] >= 0)
                    *(float4*)(A.y + (size_t)pix[rb] * C + n0) = make_float4(h[rb][qd * 4], h[rb][qd * 4 + 1], h[rb][qd * 4 + 2], h[rb][qd * 4 + 3]);
                if (TAPS && valid[rb]) {
                    if (A.tap_acc_proj) *(int4*)(A.tap_acc_proj + canon[rb] * C + n0) = make_int4(acc[rb][qd * 4], acc[rb][qd * 4 + 1], acc[rb][qd * 4 + 2], acc[rb][qd * 4 + 3]);
                    if (A.tap_h) *(float4*)(A.tap_h + canon[rb] * C + n0) = make_float4(h[rb][qd * 4], h[rb][qd * 4 + 1], h[rb][qd * 4 + 2], h[rb][qd * 4 + 3]);
                }
            }
    }
    {   // LN2: binary64 partial sums per (wave, token) through LDS, then normalise and quantize
        float mean[RB];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            double s = 0.0;
#pragma unroll
            for (int r = 0; r < 16; r += 4) s += ((double)h[rb][r] + (double)h[rb][r + 1]) + ((double)h[rb][r + 2] + (double)h[rb][r + 3]);
            s += __shfl_xor(s, 32, 64);
            if (g == 0) part[0][wave][rb * 32 + j] = s;
        }
        __syncthreads();                                              // also: every wave is done reading the attention codes
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            double tot = 0.0;
#pragma unroll
            for (int w2i = 0; w2i < NH; ++w2i) tot += part[0][w2i][rb * 32 + j];
            mean[rb] = (float)(tot / (double)C);
            double q = 0.0;
#pragma unroll
            for (int r = 0; r < 16; r += 4) {
                double a = (double)h[rb][r] - (double)mean[rb], b = (double)h[rb][r + 1] - (double)mean[rb];
                double c = (double)h[rb][r + 2] - (double)mean[rb], d = (double)h[rb][r + 3] - (double)mean[rb];
                q += (a * a + b * b) + (c * c + d * d);
            }
            q += __shfl_xor(q, 32, 64);
            if (g == 0) part[1][wave][rb * 32 + j] = q;
        }
        __syncthreads();
        const QDev qa = A.q_fc1in[branch];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            double tot = 0.0;
#pragma unroll
            for (int w2i = 0; w2i < NH; ++w2i) tot += part[1][w2i][rb * 32 + j];
            const float var = (float)(tot / (double)C);
            const float rstd = 1.0f / sqrtf(var + A.eps);
            int wd[4];
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                const int n0 = nb * 32 + qd * 8 + g * 4;
                const float4 gm = *(const float4*)(prm + PR::LN_G + n0), bt = *(const float4*)(prm + PR::LN_B + n0);
                wd[qd] = pack4(quant_code(fmaf((h[rb][qd * 4 + 0] - mean[rb]) * rstd, gm.x, bt.x), qa),
                               quant_code(fmaf((h[rb][qd * 4 + 1] - mean[rb]) * rstd, gm.y, bt.y), qa),
                               quant_code(fmaf((h[rb][qd * 4 + 2] - mean[rb]) * rstd, gm.z, bt.z), qa),
                               quant_code(fmaf((h[rb][qd * 4 + 3] - mean[rb]) * rstd, gm.w, bt.w), qa));
                if (TAPS && valid[rb] && A.tap_a2) *(int*)(A.tap_a2 + canon[rb] * C + n0) = wd[qd];
            }
            actf[(rb * KS + nb) * 64 + lane] = (v4i){wd[0], wd[1], wd[2], wd[3]};   // k slab nb, byte r = channel 32nb + mfma_row(r,g)
        }
    }
    __syncthreads();
    v16i acc2[RB];
    start(acc2, PR::F2_NC + nb * 32);
    const QDev qg = A.q_fc2in[branch];
    // GELU + quantize of the FC1 sums of hidden block ch*NH + wave -> LDS buffer ch & 1
    auto gelu_chunk = [&](int ch, const v16i* acc) {
        const int hb = ch * NH + wave;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            int wd[4];
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                const int n0 = hb * 32 + qd * 8 + g * 4;
                const float4 m = *(const float4*)(prm + PR::F1_M + n0), bs = *(const float4*)(prm + PR::F1_B + n0);
                wd[qd] = pack4(quant_code(gelu_scaled(fmaf((float)acc[rb][qd * 4 + 0], m.x, bs.x), gtab), qg),
                               quant_code(gelu_scaled(fmaf((float)acc[rb][qd * 4 + 1], m.y, bs.y), gtab), qg),
                               quant_code(gelu_scaled(fmaf((float)acc[rb][qd * 4 + 2], m.z, bs.z), gtab), qg),
                               quant_code(gelu_scaled(fmaf((float)acc[rb][qd * 4 + 3], m.w, bs.w), gtab), qg));
                if (TAPS && valid[rb]) {
                    if (A.tap_acc_fc1) *(int4*)(A.tap_acc_fc1 + canon[rb] * F + n0) = make_int4(acc[rb][qd * 4], acc[rb][qd * 4 + 1], acc[rb][qd * 4 + 2], acc[rb][qd * 4 + 3]);
                    if (A.tap_g) *(int*)(A.tap_g + canon[rb] * F + n0) = wd[qd];
                }
            }
            gs[ch & 1][(wave * RB + rb) * 64 + lane] = (v4i){wd[0], wd[1], wd[2], wd[3]};
        }
    };
    {   // chunk 0: FC1 + GELU
        v16i acc[RB];
        start(acc, PR::F1_NC + wave * 32);
        run(SLOT_ODD, w1_of(0), w1_of(1), actf, KS, 1, acc);
        gelu_chunk(0, acc);
    }
    __syncthreads();                                                  // chunk 0 of the hidden codes complete
#pragma unroll 1
    for (int ch = 1; ch < 4; ++ch) {
        v16i acc[RB];
        start(acc, PR::F1_NC + (ch * NH + wave) * 32);
        run(0, w1_of(ch), w2_of(ch - 1), actf, KS, 1, acc);                                   // FC1 of chunk ch
        run(SLOT_ODD, w2_of(ch - 1), ch < 3 ? w1_of(ch + 1) : w2_of(3), gs[(ch - 1) & 1], 1, RB, acc2);   // FC2 of chunk ch-1, under ...
        gelu_chunk(ch, acc);                                                                  // ... this arithmetic
        __syncthreads();                                              // chunk ch complete, chunk ch-1 no longer read
    }
    run(0, w2_of(3), nullptr, gs[1], 1, RB, acc2);                     // FC2 of the last chunk
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {   // second residual + scatter
            const int n0 = nb * 32 + qd * 8 + g * 4;
            const float4 m = *(const float4*)(prm + PR::F2_M + n0), bs = *(const float4*)(prm + PR::F2_B + n0);
            float4 hh = make_float4(h[rb][qd * 4], h[rb][qd * 4 + 1], h[rb][qd * 4 + 2], h[rb][qd * 4 + 3]);
            if (PARK_H) hh = pix[rb] >= 0 ? *(const float4*)(A.y + (size_t)pix[rb] * C + n0) : make_float4(0.f, 0.f, 0.f, 0.f);
            float4 o4 = make_float4(fmaf((float)acc2[rb][qd * 4 + 0], m.x, bs.x) + hh.x, fmaf((float)acc2[rb][qd * 4 + 1], m.y, bs.y) + hh.y,
                                    fmaf((float)acc2[rb][qd * 4 + 2], m.z, bs.z) + hh.z, fmaf((float)acc2[rb][qd * 4 + 3], m.w, bs.w) + hh.w);
            if (pix[rb] >= 0) *(float4*)(A.y + (size_t)pix[rb] * C + n0) = o4;
            if (TAPS && valid[rb]) {
                if (A.tap_acc_fc2) *(int4*)(A.tap_acc_fc2 + canon[rb] * C + n0) = make_int4(acc2[rb][qd * 4], acc2[rb][qd * 4 + 1], acc2[rb][qd * 4 + 2], acc2[rb][qd * 4 + 3]);
                if (A.tap_y) *(float4*)(A.tap_y + canon[rb] * C + n0) = o4;
            }
        }
}

// ------------------------------------------------------------------ launchers
template <int LPT, int NV>
static void launch_score_t(const Geom& G, const float* x, int mode, float eps, const float* gm, const float* bt,
                           double* scores, hipStream_t st)
{
    hipLaunchKernelGGL((score_kernel<LPT, NV>), dim3(G.B * G.nW), dim3(256), 0, st, G, x, mode, eps, gm, bt, scores);
}
template <int LPT, int NV>
static void launch_ln_t(const Geom& G, const LnArgs& A, bool gather, hipStream_t st)
{
    constexpr int TP = 256 / LPT;
    if (G.rows_total == 0) return;
    dim3 grid((G.rows_total + TP - 1) / TP);
    if (gather) hipLaunchKernelGGL((ln_quant_kernel<LPT, NV, true>), grid, dim3(256), 0, st, G, A);
    else hipLaunchKernelGGL((ln_quant_kernel<LPT, NV, false>), grid, dim3(256), 0, st, G, A);
}

#define MIXAQ_DISPATCH_C(C, CALL)                                             \
    switch (C) {                                                              \
        case 96: CALL(8, 3); break;                                           \
        case 128: CALL(8, 4); break;                                          \
        case 192: CALL(16, 3); break;                                         \
        case 256: CALL(16, 4); break;                                         \
        case 384: CALL(32, 3); break;                                         \
        case 512: CALL(32, 4); break;                                         \
        case 768: CALL(64, 3); break;                                         \
        case 1024: CALL(64, 4); break;                                        \
        default: return false;                                                \
    }

bool channels_supported(int C)
{
    return C == 96 || C == 128 || C == 192 || C == 256 || C == 384 || C == 512 || C == 768 || C == 1024;
}

bool launch_score(const Geom& G, const float* x, int mode, float eps, const float* gm, const float* bt, double* scores,
                  hipStream_t st)
{
#define CALL(L, N) launch_score_t<L, N>(G, x, mode, eps, gm, bt, scores, st)
    MIXAQ_DISPATCH_C(G.C, CALL)
#undef CALL
    return true;
}

void launch_bypass(const Geom& G, const int* perm, const float* x, float* y, hipStream_t st)
{
    const int n_pruned = G.nW - G.k_hi - G.k_lo;
    if (n_pruned > 0) hipLaunchKernelGGL(bypass_kernel, dim3(G.B * n_pruned), dim3(256), 0, st, G, perm, x, y);
}

void launch_select(const double* scores, int B, int nW, int reverse, int* perm, hipStream_t st)
{
    hipLaunchKernelGGL(select_rank_kernel, dim3((nW + RANK_WPB - 1) / RANK_WPB, B), dim3(256), (size_t)nW * 8, st, scores, nW, reverse,
                       perm);
}

bool launch_ln_quant(const Geom& G, const LnArgs& A, bool gather, hipStream_t st)
{
#define CALL(L, N) launch_ln_t<L, N>(G, A, gather, st)
    MIXAQ_DISPATCH_C(G.C, CALL)
#undef CALL
    return true;
}

template <int EPI>
static void launch_gemm_e(const Geom& G, const GemmArgs& A0, hipStream_t st)
{
    GemmArgs A = A0;
    if (G.rows_total == 0) return;
    const int tiles = G.rows_total / ROW_TILE, NB = A.N / 32;
    // the activation tile through LDS, output blocks over the waves and, while the grid is small, in groups over workgroups
    // 32-row tiles: a long K stays whole in LDS (K = 3072 on 19 row tiles: 16.3 us; 64-row tiles in chunks of 1024: 27.8 us);
    // a narrow layer on few rows gets twice the workgroups (the projection at C = 768 on 19 row tiles: 8.1 instead of 10.7 us;
    // with 72 or 96 output blocks the wider layers have workgroups enough and lose: 13.2 and 13.8 instead of 12.4 and 13.2 us)
    const bool half = (A.K > GEMM_TILE_MAX_K && A.K <= 4096) || (tiles <= 32 && NB <= 32 && A.K > 384 && A.K <= 1024);
    A.kchunk = A.K;
    if (A.K > 4096)                                                   // chunks of whole ring turns (256 bytes of K each): the largest such size up to
        for (A.kchunk = 1024; A.kchunk > 256 && A.K % A.kchunk; A.kchunk -= 256) {}   // 1024 that divides K (K = 768 r or 1024 r here: 256 always does)
    const int nt = half ? G.rows_total / 32 : tiles;
    const int groups = std::max(1, std::min((NB + 3) / 4, (512 + nt - 1) / nt));
    A.nb_per_block = ((NB + groups - 1) / groups + 3) / 4 * 4;
    const dim3 grid(nt, (NB + A.nb_per_block - 1) / A.nb_per_block);
    if (half && A.K <= 1024) hipLaunchKernelGGL((gemm_tile_kernel<EPI, 1024, 32>), grid, dim3(256), 0, st, G, A);
    else if (half && A.K <= 3072) hipLaunchKernelGGL((gemm_tile_kernel<EPI, 3072, 32>), grid, dim3(256), 0, st, G, A);
    else if (half) hipLaunchKernelGGL((gemm_tile_kernel<EPI, 4096, 32>), grid, dim3(256), 0, st, G, A);
    else if (A.K <= 384) hipLaunchKernelGGL((gemm_tile_kernel<EPI, 384>), grid, dim3(256), 0, st, G, A);
    else if (A.K <= 1024 || A.K > GEMM_TILE_MAX_K) hipLaunchKernelGGL((gemm_tile_kernel<EPI, 1024>), grid, dim3(256), 0, st, G, A);   // above 4096: chunks of 1024
    else hipLaunchKernelGGL((gemm_tile_kernel<EPI, GEMM_TILE_MAX_K>), grid, dim3(256), 0, st, G, A);
}

void launch_gemm(const Geom& G, const GemmArgs& A, int epi, hipStream_t st)
{
    switch (epi) {
        case EPI_QKV: launch_gemm_e<EPI_QKV>(G, A, st); break;
        case EPI_PROJ: launch_gemm_e<EPI_PROJ>(G, A, st); break;
        case EPI_FC1: launch_gemm_e<EPI_FC1>(G, A, st); break;
        default: launch_gemm_e<EPI_FC2>(G, A, st); break;
    }
}

// the window kernel (gather + LN1 + QKV + attention) and the token kernel (proj + LN2 + FFN + scatter) are chosen separately
// (a window kernel for C = 768, two workgroups of twelve heads per window, was measured at 37.5 us against 42 us for the three
// kernels it replaces on 24 windows, and the whole stage came out slower: not enabled)
bool fused_window_supported(int C) { return C == 96 || C == 128 || C == 192 || C == 256 || C == 384; }
bool fused_token_supported(int C, int mlp_ratio) { return (C == 96 || C == 128 || C == 192 || C == 256 || C == 384) && mlp_ratio == 4; }

// C = 384: up to this many windows, two workgroups share a window's heads, each with a pair of waves per head (twelve
// waves: 15.7 instead of 16.8 us on 96 windows with one wave per head, and 22.8 us for one twelve-head workgroup per window)
constexpr int WINDOW_SPLIT_SMALL = 128;
// Up to this many windows a pair of waves shares a head.  The pair form has the shorter chain of dependent steps
// (a workgroup alone on its CU: 9.5 instead of 11.2 us at C = 96) but 15 % more vector and 80 % more scalar
// instructions per window, so it loses once the CUs are full (1392 windows at C = 96: 31 instead of 28.3 us;
// 5476 at C = 128: 113 instead of 101 us).  At C = 192 it wins on 360 windows (22.8 instead of 25.4 us); at
// C = 256 it measures the same on 1444 windows and is not instantiated.
constexpr int WINDOW_PAIR_SMALL = 256, WINDOW_PAIR_SMALL_6 = 512;
void launch_window(const Geom& G, const WinArgs& A, hipStream_t st)
{
    // every window gets a workgroup: with scores it finds its own rank (and may turn out pruned), otherwise
    // the computed slots come first and the pruned windows of the list after them
    const int n_wg = G.B * G.nW;
    if (n_wg == 0) return;
#define WIN_CASE(NH, HG, QS)                                                                                              \
    {                                                                                                                     \
        const dim3 grid(n_wg * HG), block(NH * QS * 64);                                                                  \
        if (A.scores) {   /* no entry point takes scores and taps together */                                            \
            hipLaunchKernelGGL((window_kernel<NH, false, true, HG, QS>), grid, block, 0, st, G, A);                       \
        } else {                                                                                                          \
            if (A.taps) hipLaunchKernelGGL((window_kernel<NH, true, false, HG, QS>), grid, block, 0, st, G, A);           \
            else hipLaunchKernelGGL((window_kernel<NH, false, false, HG, QS>), grid, block, 0, st, G, A);                 \
        }                                                                                                                 \
    }                                                                                                                     \
    break
    switch (G.C / 32) {
        case 3:
            if (n_wg <= WINDOW_PAIR_SMALL) { WIN_CASE(3, 1, 2); }
            WIN_CASE(3, 1, 1);
        case 4:
            if (n_wg <= WINDOW_PAIR_SMALL) { WIN_CASE(4, 1, 2); }
            WIN_CASE(4, 1, 1);
        case 6:
            if (n_wg <= WINDOW_PAIR_SMALL_6) { WIN_CASE(6, 1, 2); }
            WIN_CASE(6, 1, 1);
        case 8: WIN_CASE(8, 1, 1);
        case 12:
            if (n_wg <= WINDOW_SPLIT_SMALL) { WIN_CASE(6, 2, 2); }
            WIN_CASE(12, 1, 1);
        default: break;
    }
#undef WIN_CASE
}

constexpr int TOKEN_WIDE_SMALL = 128;        // C = 384: up to this many 64-row tiles the wide token kernel runs on 32-row tiles
void launch_token(const Geom& G, const TokArgs& A, hipStream_t st)
{
    if (G.rows_total == 0) return;
    const int NHr = G.C / 32;
#define TOK_CASE(NH)                                                                                              \
    if (A.taps) hipLaunchKernelGGL((token_kernel<NH, true>), dim3(G.rows_total / 32), dim3(NH * 64), 0, st, G, A); \
    else hipLaunchKernelGGL((token_kernel<NH, false>), dim3(G.rows_total / 32), dim3(NH * 64), 0, st, G, A);      \
    break
    // twelve heads: the wide form, 64-row tiles once there are enough of them to give every second CU one, else 32-row tiles
    if (NHr == 12 && G.rows_total / 64 > TOKEN_WIDE_SMALL) {
        if (A.taps) hipLaunchKernelGGL((token_wide_kernel<12, 2, true>), dim3(G.rows_total / 64), dim3(12 * 64), 0, st, G, A);
        else hipLaunchKernelGGL((token_wide_kernel<12, 2, false>), dim3(G.rows_total / 64), dim3(12 * 64), 0, st, G, A);
    } else if (NHr == 12) {
        if (A.taps) hipLaunchKernelGGL((token_wide_kernel<12, 1, true>), dim3(G.rows_total / 32), dim3(12 * 64), 0, st, G, A);
        else hipLaunchKernelGGL((token_wide_kernel<12, 1, false>), dim3(G.rows_total / 32), dim3(12 * 64), 0, st, G, A);
    } else if (NHr == 6) {    // six waves: the wide form on 32-row tiles (28.9 instead of 32.3 us on 552 tiles; at 3, 4 and 8 waves the plain kernel wins)
        if (A.taps) hipLaunchKernelGGL((token_wide_kernel<6, 1, true>), dim3(G.rows_total / 32), dim3(6 * 64), 0, st, G, A);
        else hipLaunchKernelGGL((token_wide_kernel<6, 1, false>), dim3(G.rows_total / 32), dim3(6 * 64), 0, st, G, A);
    } else {
        switch (NHr) {
            case 3: TOK_CASE(3);
            case 4: TOK_CASE(4);
            default: TOK_CASE(8);
        }
    }
#undef TOK_CASE
}

void launch_attn(const Geom& G, const AttnArgs& A, hipStream_t st)
{
    const int items = G.n_slots * G.heads;
    if (items == 0) return;
    hipLaunchKernelGGL(attn_kernel, dim3((items + 3) / 4), dim3(256), 0, st, G, A);
}

}  // namespace mixaq
