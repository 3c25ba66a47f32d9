// The layers between the stages of a Swin backbone (patch embedding, patch merging) as one
// uniformly quantized linear layer each: gather + (LayerNorm) + quantize + int8 MFMA +
// dequantize + (LayerNorm), one kernel.  The paper keeps these layers outside MixA-Q (its cost
// model lists them as the part the method cannot save, appendix on equivalent activation bits);
// they are here so that the four stages of a backbone run as one chain on the GPU.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/mixaq.h"
#include "mixaq_dev.h"

namespace mixaq { int fail(int code, const char* fmt, ...); }
using namespace mixaq;

namespace {

struct DsArgs {
    const float* x;
    float* y;
    int B, H, W, Cin, P, K, Kp, N, Ho, Wo, tokens;
    const v4i* Wp;                    // [N/32][Kp/32][64 lanes] x 16 bytes, natural k order, zero beyond K
    const float* m;                   // a_in.scale * s_w[n]
    const float* bias;                // [N] (zeros when the layer has none)
    const int* negcorr;               // -zp * sum_k W[n,k]
    const float* gamma;               // kind 0: [N], kind 1: [K]
    const float* beta;
    QDev q;
    float eps;
    int8_t* tap_codes;                // [tokens][K] or NULL
    int32_t* tap_acc;                 // [tokens][N] or NULL
};

__device__ __forceinline__ double sum8(double v)      // over the 8 lanes of a token
{
    v += __shfl_xor(v, 4, 64);
    v += __shfl_xor(v, 2, 64);
    v += __shfl_xor(v, 1, 64);
    return v;
}

// the four input values k0..k0+3 of output token (b,i,j); zero outside the map and beyond K
// (PC, CC: patch size and input channels when known at compile time, so that the index divisions are by constants; 0 = from A)
template <int KIND, int PC = 0, int CC = 0>
__device__ __forceinline__ float4 ds_values(const DsArgs& A, int b, int i, int j, int k0)
{
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (k0 >= A.K) return v;
    const int P = PC ? PC : A.P, Cin = CC ? CC : A.Cin;
    if (KIND == 1) {                  // 2x2 neighbours in the order (0,0), (1,0), (0,1), (1,1) [row, column offset]
        const int q = k0 / A.Cin, ch = k0 - q * A.Cin;
        const int r = 2 * i + (q & 1), c = 2 * j + (q >> 1);
        if (r < A.H && c < A.W) v = *(const float4*)(A.x + (((size_t)b * A.H + r) * A.W + c) * A.Cin + ch);
    } else {                          // patch values in the order (row in patch, column in patch, channel)
        float e[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int k = k0 + t, pc = k / Cin, ch = k - pc * Cin, di = pc / P, dj = pc - di * P;
            const int r = i * P + di, c = j * P + dj;
            e[t] = (r < A.H && c < A.W) ? A.x[(((size_t)b * A.H + r) * A.W + c) * Cin + ch] : 0.f;
        }
        v = make_float4(e[0], e[1], e[2], e[3]);
    }
    return v;
}

// Patch merging of the usual widths (C_in = 4 LPT NV4, LPT lanes per token, 4 NV4 = NV float4 per lane: C_in a
// multiple of 48 or 64 up to 512).  One workgroup (4 waves) per 32 output tokens and per group of output blocks.
// Phase 1: LPT lanes hold the 4 C_in inputs of a token in registers (NV independent 16-byte loads per lane, the
// neighbour of each known at compile time), LayerNorm statistics in binary64 over the lane group, quantize, codes
// to LDS as MFMA operand fragments; 256 / LPT tokens per pass.  Phase 2: wave w computes the output blocks
// first + w, first + w + 4, ... of its group: the weight fragments stream through a ring of loads in flight.
template <int LPT, int NV, bool TAPS>
__global__ __launch_bounds__(256) void merge_kernel(DsArgs A, int blocks_per_group)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int TP = 256 / LPT, PER = NV / 4, KSN = NV * LPT / 8, RING = KSN % 8 == 0 ? 8 : 6;
    static_assert(NV % 4 == 0 && (LPT & (LPT - 1)) == 0 && LPT <= 64 && KSN % RING == 0, "lane groups inside a wave, whole ring turns");
    v4i* frag = (v4i*)smem;                                   // [KSN][64]
    int* fragw = (int*)smem;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int grp = tid / LPT, sub = tid % LPT;
#pragma unroll 1
    for (int p0 = 0; p0 < 32; p0 += TP) {
        const int jt = p0 + grp, tok = blockIdx.x * 32 + jt;
        const bool valid = tok < A.tokens;
        const int b = tok / (A.Ho * A.Wo), rem = tok - b * (A.Ho * A.Wo), i = rem / A.Wo, j = rem - i * A.Wo;
        float4 v[NV];
#pragma unroll
        for (int k = 0; k < NV; ++k) {                        // element k of the lane: neighbour k / PER, channels ((k % PER) LPT + sub) 4 ..
            const int q = k / PER, r = 2 * i + (q & 1), c = 2 * j + (q >> 1);
            v[k] = (valid && r < A.H && c < A.W)
                       ? *(const float4*)(A.x + (((size_t)b * A.H + r) * A.W + c) * A.Cin + ((k % PER) * LPT + sub) * 4)
                       : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        double s = 0.0;
#pragma unroll
        for (int k = 0; k < NV; ++k) s += ((double)v[k].x + (double)v[k].y) + ((double)v[k].z + (double)v[k].w);
#pragma unroll
        for (int o = LPT / 2; o >= 1; o >>= 1) s += __shfl_xor(s, o, 64);
        const float mean = (float)(s / (double)A.K);
        double qv = 0.0;
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const double a0 = (double)v[k].x - (double)mean, a1 = (double)v[k].y - (double)mean;
            const double a2 = (double)v[k].z - (double)mean, a3 = (double)v[k].w - (double)mean;
            qv += (a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3);
        }
#pragma unroll
        for (int o = LPT / 2; o >= 1; o >>= 1) qv += __shfl_xor(qv, o, 64);
        const float var = (float)(qv / (double)A.K);
        const float rstd = 1.0f / sqrtf(var + A.eps);
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const int k0 = (k * LPT + sub) * 4;
            int code = 0;
            if (valid) {
                const float4 gm = *(const float4*)(A.gamma + k0), bt = *(const float4*)(A.beta + k0);
                code = pack4(quant_code(fmaf((v[k].x - mean) * rstd, gm.x, bt.x), A.q), quant_code(fmaf((v[k].y - mean) * rstd, gm.y, bt.y), A.q),
                             quant_code(fmaf((v[k].z - mean) * rstd, gm.z, bt.z), A.q), quant_code(fmaf((v[k].w - mean) * rstd, gm.w, bt.w), A.q));
                if (TAPS && A.tap_codes && blockIdx.y == 0) *(int*)(A.tap_codes + (size_t)tok * A.K + k0) = code;
            }
            fragw[(((k0 >> 5) * 64 + ((k0 & 31) >> 4) * 32 + jt) << 2) + ((k0 & 15) >> 2)] = code;
        }
    }
    __syncthreads();
    const int j = lane & 31, g = lane >> 5;
    const int tok = blockIdx.x * 32 + j;
    const bool valid = tok < A.tokens;
    const int first = blockIdx.y * blocks_per_group, last = min(first + blocks_per_group, A.N / 32);
    for (int nb = first + wave; nb < last; nb += 4) {
        const v4i* wp = A.Wp + (size_t)nb * KSN * 64 + lane;
        v4i ring[RING];
#pragma unroll
        for (int d = 0; d < RING; ++d) ring[d] = wp[d * 64];
        v16i acc;
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            const int4 t4 = *(const int4*)(A.negcorr + nb * 32 + qd * 8 + g * 4);
            acc[qd * 4 + 0] = t4.x; acc[qd * 4 + 1] = t4.y; acc[qd * 4 + 2] = t4.z; acc[qd * 4 + 3] = t4.w;
        }
#pragma unroll 1
        for (int k0 = 0; k0 < KSN; k0 += RING) {
#pragma unroll
            for (int d = 0; d < RING; ++d) {
                const v4i wv = ring[d];
                ring[d] = wp[min(k0 + RING + d, KSN - 1) * 64];           // past the end: the last fragment again, unused
                acc = mfma32(wv, frag[(k0 + d) * 64 + lane], acc);
            }
        }
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            const int n0 = nb * 32 + qd * 8 + g * 4;
            const float4 m = *(const float4*)(A.m + n0), bs = *(const float4*)(A.bias + n0);
            if (valid) {
                *(float4*)(A.y + (size_t)tok * A.N + n0) =
                    make_float4(fmaf((float)acc[qd * 4 + 0], m.x, bs.x), fmaf((float)acc[qd * 4 + 1], m.y, bs.y),
                                fmaf((float)acc[qd * 4 + 2], m.z, bs.z), fmaf((float)acc[qd * 4 + 3], m.w, bs.w));
                if (TAPS && A.tap_acc) *(int4*)(A.tap_acc + (size_t)tok * A.N + n0) = make_int4(acc[qd * 4], acc[qd * 4 + 1], acc[qd * 4 + 2], acc[qd * 4 + 3]);
            }
        }
    }
}

// The general form (patch embedding; patch merging of other widths).
// One workgroup (4 waves) per 32 output tokens.  Phase 1: eight lanes per token gather the K inputs
// (kind 1: LayerNorm over them, binary64 sums), quantize, and lay the codes out in LDS as MFMA
// operand fragments.  Phase 2: wave w computes the output blocks w, w+4, ...: W * codes^T, lane =
// token, 16 channels per block; dequantize; kind 1 stores, kind 0 goes through LDS for the
// LayerNorm over the N outputs of a token.
template <int KIND, int PC = 0, int CC = 0>
__global__ __launch_bounds__(256) void downsample_kernel(DsArgs A)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    v4i* frag = (v4i*)smem;                                   // [Kp/32][64]
    float* fo = (float*)(smem + (size_t)A.Kp * 32);           // kind 0: [32][N]
    int* fragw = (int*)smem;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    {
        const int jt = tid >> 3, sub = tid & 7;
        const int tok = blockIdx.x * 32 + jt;
        const bool valid = tok < A.tokens;
        const int b = tok / (A.Ho * A.Wo), rem = tok - b * (A.Ho * A.Wo), i = rem / A.Wo, j = rem - i * A.Wo;
        const int nch = A.Kp / 4, nreal = A.K / 4;
        float mean = 0.f, rstd = 1.f;
        if (KIND == 1) {
            double s = 0.0;
            if (valid)
                for (int c4 = sub; c4 < nreal; c4 += 8) {
                    const float4 v = ds_values<KIND, PC, CC>(A, b, i, j, c4 * 4);
                    s += ((double)v.x + (double)v.y) + ((double)v.z + (double)v.w);
                }
            s = sum8(s);
            mean = (float)(s / (double)A.K);
            double qv = 0.0;
            if (valid)
                for (int c4 = sub; c4 < nreal; c4 += 8) {
                    const float4 v = ds_values<KIND, PC, CC>(A, b, i, j, c4 * 4);
                    const double a0 = (double)v.x - (double)mean, a1 = (double)v.y - (double)mean;
                    const double a2 = (double)v.z - (double)mean, a3 = (double)v.w - (double)mean;
                    qv += (a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3);
                }
            qv = sum8(qv);
            const float var = (float)(qv / (double)A.K);
            rstd = 1.0f / sqrtf(var + A.eps);
        }
        for (int c4 = sub; c4 < nch; c4 += 8) {
            const int k0 = c4 * 4;
            int code = 0;
            if (valid && k0 < A.K) {
                float4 v = ds_values<KIND, PC, CC>(A, b, i, j, k0);
                if (KIND == 1) {
                    const float4 gm = *(const float4*)(A.gamma + k0), bt = *(const float4*)(A.beta + k0);
                    v.x = fmaf((v.x - mean) * rstd, gm.x, bt.x);
                    v.y = fmaf((v.y - mean) * rstd, gm.y, bt.y);
                    v.z = fmaf((v.z - mean) * rstd, gm.z, bt.z);
                    v.w = fmaf((v.w - mean) * rstd, gm.w, bt.w);
                }
                code = pack4(quant_code(v.x, A.q), quant_code(v.y, A.q), quant_code(v.z, A.q), quant_code(v.w, A.q));
                if (A.tap_codes) *(int*)(A.tap_codes + (size_t)tok * A.K + k0) = code;
            }
            // fragment (k slab, lane = half*32 + token): 16 bytes = the half's 16 consecutive k
            fragw[(((k0 >> 5) * 64 + ((k0 & 31) >> 4) * 32 + jt) << 2) + ((k0 & 15) >> 2)] = code;
        }
    }
    __syncthreads();
    const int j = lane & 31, g = lane >> 5, ksn = A.Kp / 32;
    const int tok = blockIdx.x * 32 + j;
    const bool valid = tok < A.tokens;
    for (int nb = wave; nb < A.N / 32; nb += 4) {
        v16i acc;
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            const int4 t4 = *(const int4*)(A.negcorr + nb * 32 + qd * 8 + g * 4);
            acc[qd * 4 + 0] = t4.x; acc[qd * 4 + 1] = t4.y; acc[qd * 4 + 2] = t4.z; acc[qd * 4 + 3] = t4.w;
        }
        const v4i* wp = A.Wp + (size_t)nb * ksn * 64 + lane;
        for (int ks = 0; ks < ksn; ++ks) acc = mfma32(wp[ks * 64], frag[ks * 64 + lane], acc);
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            const int n0 = nb * 32 + qd * 8 + g * 4;
            const float4 m = *(const float4*)(A.m + n0), bs = *(const float4*)(A.bias + n0);
            const float4 f = make_float4(fmaf((float)acc[qd * 4 + 0], m.x, bs.x), fmaf((float)acc[qd * 4 + 1], m.y, bs.y),
                                         fmaf((float)acc[qd * 4 + 2], m.z, bs.z), fmaf((float)acc[qd * 4 + 3], m.w, bs.w));
            if (valid && A.tap_acc) *(int4*)(A.tap_acc + (size_t)tok * A.N + n0) = make_int4(acc[qd * 4], acc[qd * 4 + 1], acc[qd * 4 + 2], acc[qd * 4 + 3]);
            if (KIND == 1) {
                if (valid) *(float4*)(A.y + (size_t)tok * A.N + n0) = f;
            } else {
                *(float4*)(fo + j * A.N + n0) = f;
            }
        }
    }
    if (KIND == 0) {                  // LayerNorm over the N outputs of a token, eight lanes per token
        __syncthreads();
        const int jt = tid >> 3, sub = tid & 7, tk = blockIdx.x * 32 + jt, nch = A.N / 4;
        const float* row = fo + jt * A.N;
        double s = 0.0;
        for (int c4 = sub; c4 < nch; c4 += 8) {
            const float4 v = *(const float4*)(row + c4 * 4);
            s += ((double)v.x + (double)v.y) + ((double)v.z + (double)v.w);
        }
        s = sum8(s);
        const float mean = (float)(s / (double)A.N);
        double qv = 0.0;
        for (int c4 = sub; c4 < nch; c4 += 8) {
            const float4 v = *(const float4*)(row + c4 * 4);
            const double a0 = (double)v.x - (double)mean, a1 = (double)v.y - (double)mean;
            const double a2 = (double)v.z - (double)mean, a3 = (double)v.w - (double)mean;
            qv += (a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3);
        }
        qv = sum8(qv);
        const float var = (float)(qv / (double)A.N);
        const float rstd = 1.0f / sqrtf(var + A.eps);
        if (tk < A.tokens)
            for (int c4 = sub; c4 < nch; c4 += 8) {
                const float4 v = *(const float4*)(row + c4 * 4);
                const float4 gm = *(const float4*)(A.gamma + c4 * 4), bt = *(const float4*)(A.beta + c4 * 4);
                *(float4*)(A.y + (size_t)tk * A.N + c4 * 4) =
                    make_float4(fmaf((v.x - mean) * rstd, gm.x, bt.x), fmaf((v.y - mean) * rstd, gm.y, bt.y),
                                fmaf((v.z - mean) * rstd, gm.z, bt.z), fmaf((v.w - mean) * rstd, gm.w, bt.w));
            }
    }
}

#define HIP_TRY(expr)                                                                                   \
    do {                                                                                                \
        hipError_t e_ = (expr);                                                                         \
        if (e_ != hipSuccess) return fail(MIXAQ_E_HIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

}  // namespace

struct mixaq_downsample {
    mixaq_downsample_desc d;
    int P = 0, K = 0, Kp = 0, Ho = 0, Wo = 0;
    std::vector<void*> owned;
    v4i* Wp = nullptr;
    float *m = nullptr, *bias = nullptr, *gamma = nullptr, *beta = nullptr;
    int* negcorr = nullptr;
    QDev q;
    ~mixaq_downsample() { for (void* p : owned) (void)hipFree(p); }
};

namespace {

int ds_geometry(const mixaq_downsample_desc* d, int* P, int* K, int* Ho, int* Wo)
{
    if (!d) return fail(MIXAQ_E_NULL, "descriptor is NULL");
    if (d->kind != 0 && d->kind != 1) return fail(MIXAQ_E_SHAPE, "kind must be 0 (patch embedding) or 1 (patch merging)");
    if (d->B < 1 || d->H < 1 || d->W < 1 || d->C_in < 1) return fail(MIXAQ_E_SHAPE, "B, H, W, C_in must be positive");
    *P = d->kind == 0 ? d->patch : 2;
    if (*P < 1 || *P > 16) return fail(MIXAQ_E_SHAPE, "patch must be in 1..16");
    *K = *P * *P * d->C_in;
    if (*K % 4 != 0 || *K > 8192) return fail(MIXAQ_E_SHAPE, "inputs per token (%d) must be a multiple of 4, at most 8192", *K);
    if (d->kind == 1 && d->C_in % 4 != 0) return fail(MIXAQ_E_SHAPE, "patch merging needs C_in %% 4 == 0");
    if (d->N < 32 || d->N % 32 != 0 || d->N > 4096) return fail(MIXAQ_E_SHAPE, "N must be a multiple of 32 in 32..4096");
    if (d->act_bits < 2 || d->act_bits > 8 || d->weight_bits < 2 || d->weight_bits > 8)
        return fail(MIXAQ_E_BITS, "bit widths must be in 2..8");
    if (!(d->ln_eps > 0.0f)) return fail(MIXAQ_E_SHAPE, "ln_eps must be positive");
    *Ho = (d->H + *P - 1) / *P;
    *Wo = (d->W + *P - 1) / *P;
    if ((long long)d->B * *Ho * *Wo > (1LL << 30)) return fail(MIXAQ_E_SHAPE, "map too large for 32-bit token indexing");
    return MIXAQ_OK;
}

template <typename T>
int ds_upload(mixaq_downsample* h, const std::vector<T>& host, T** dev)
{
    void* p = nullptr;
    HIP_TRY(hipMalloc(&p, host.size() * sizeof(T) + 16));
    h->owned.push_back(p);
    HIP_TRY(hipMemcpy(p, host.data(), host.size() * sizeof(T), hipMemcpyHostToDevice));
    *dev = (T*)p;
    return MIXAQ_OK;
}

size_t ds_lds_bytes(const mixaq_downsample* h) { return (size_t)h->Kp * 32 + (h->d.kind == 0 ? (size_t)32 * h->d.N * 4 : 0); }

int ds_forward(const mixaq_downsample* h, const float* x, float* y, void* stream, int8_t* tap_codes, int32_t* tap_acc)
{
    if (!h) return fail(MIXAQ_E_NULL, "handle is NULL");
    if (!x || !y) return fail(MIXAQ_E_NULL, "x or y is NULL");
    DsArgs A = {};
    A.x = x; A.y = y;
    A.B = h->d.B; A.H = h->d.H; A.W = h->d.W; A.Cin = h->d.C_in; A.P = h->P; A.K = h->K; A.Kp = h->Kp; A.N = h->d.N;
    A.Ho = h->Ho; A.Wo = h->Wo; A.tokens = h->d.B * h->Ho * h->Wo;
    A.Wp = h->Wp; A.m = h->m; A.bias = h->bias; A.negcorr = h->negcorr; A.gamma = h->gamma; A.beta = h->beta;
    A.q = h->q; A.eps = h->d.ln_eps; A.tap_codes = tap_codes; A.tap_acc = tap_acc;
    const dim3 grid((A.tokens + 31) / 32);
    const size_t lds = ds_lds_bytes(h);
    hipStream_t st = (hipStream_t)stream;
    // patch merging of the usual widths: lanes per token and registers per lane from C_in; the output blocks are split
    // into groups of at least four (one per wave) over more workgroups while the grid has fewer than about 512
    int lpt = 0, nv = 0;
    if (h->d.kind == 1) {
        for (int n : {12, 16})
            for (int l : {8, 16, 32})
                if (!lpt && A.Cin == n * l) { lpt = l; nv = n; }
    }
    if (lpt) {
        const int NB = A.N / 32, tiles = (int)grid.x;
        int groups = std::max(1, std::min(NB / 4, (512 + tiles - 1) / tiles));
        const int per = ((NB + groups - 1) / groups + 3) / 4 * 4;
        groups = (NB + per - 1) / per;
        const dim3 grid2(tiles, groups);
        const bool taps = tap_codes || tap_acc;
#define MERGE_CASE(L, V)                                                                                          \
    if (lpt == L && nv == V) {                                                                                    \
        if (taps) hipLaunchKernelGGL((merge_kernel<L, V, true>), grid2, dim3(256), (size_t)A.Kp * 32, st, A, per);  \
        else hipLaunchKernelGGL((merge_kernel<L, V, false>), grid2, dim3(256), (size_t)A.Kp * 32, st, A, per);     \
    }
        MERGE_CASE(8, 12) MERGE_CASE(16, 12) MERGE_CASE(32, 12) MERGE_CASE(8, 16) MERGE_CASE(16, 16) MERGE_CASE(32, 16)
#undef MERGE_CASE
    } else if (h->d.kind == 0 && A.P == 4 && A.Cin == 3) hipLaunchKernelGGL((downsample_kernel<0, 4, 3>), grid, dim3(256), lds, st, A);
    else if (h->d.kind == 0) hipLaunchKernelGGL(downsample_kernel<0>, grid, dim3(256), lds, st, A);
    else hipLaunchKernelGGL(downsample_kernel<1>, grid, dim3(256), lds, st, A);
    HIP_TRY(hipGetLastError());
    return MIXAQ_OK;
}

}  // namespace

extern "C" {

int mixaq_downsample_out_shape(const mixaq_downsample_desc* desc, int32_t* Ho, int32_t* Wo, int32_t* K)
{
    if (!Ho || !Wo || !K) return fail(MIXAQ_E_NULL, "an output pointer is NULL");
    int P, k, ho, wo, rc = ds_geometry(desc, &P, &k, &ho, &wo);
    if (rc) return rc;
    *Ho = ho; *Wo = wo; *K = k;
    return MIXAQ_OK;
}

static int downsample_create(const mixaq_downsample_desc* desc, const mixaq_downsample_params* p, mixaq_downsample** out);

// No C++ exception leaves the library: host containers that fail to allocate become an error code.
int mixaq_downsample_create(const mixaq_downsample_desc* desc, const mixaq_downsample_params* p, mixaq_downsample** out)
{
    try {
        return downsample_create(desc, p, out);
    } catch (const std::bad_alloc&) {
        return fail(MIXAQ_E_HIP, "out of host memory while preparing the layer");
    } catch (...) {
        return fail(MIXAQ_E_HIP, "unexpected C++ exception while preparing the layer");
    }
}

namespace {
struct LayerOwner {                      // frees a half-built layer on every early return and on an exception
    mixaq_downsample* h;
    ~LayerOwner() { delete h; }
};
}  // namespace

static int downsample_create(const mixaq_downsample_desc* desc, const mixaq_downsample_params* p, mixaq_downsample** out)
{
    if (!out) return fail(MIXAQ_E_NULL, "out is NULL");
    *out = nullptr;
    int P, K, Ho, Wo, rc = ds_geometry(desc, &P, &K, &Ho, &Wo);
    if (rc) return rc;
    if (!p || !p->w || !p->s_w || !p->ln_gamma || !p->ln_beta) return fail(MIXAQ_E_NULL, "a required parameter pointer is NULL");
    if (!(p->a_in.scale > 0.0f) || !std::isfinite(p->a_in.scale)) return fail(MIXAQ_E_SHAPE, "input scale must be positive");
    const int qmin = -(1 << (desc->act_bits - 1)), qmax = (1 << (desc->act_bits - 1)) - 1;
    if (p->a_in.zero_point < qmin || p->a_in.zero_point > qmax) return fail(MIXAQ_E_BITS, "zero point outside the code range");
    const int N = desc->N, Kp = (K + 31) / 32 * 32, n_ln = desc->kind == 0 ? N : K;
    if (desc->kind == 0 && (size_t)Kp * 32 + (size_t)32 * N * 4 > 64 * 1024) return fail(MIXAQ_E_SHAPE, "patch embedding too wide for one workgroup's LDS");
    if ((size_t)Kp * 32 > 64 * 1024) return fail(MIXAQ_E_SHAPE, "too many inputs per token for one workgroup's LDS");
    mixaq_downsample* h = new (std::nothrow) mixaq_downsample();
    if (!h) return fail(MIXAQ_E_HIP, "out of host memory");
    LayerOwner owner{h};
    auto bail = [&](int code) { return code; };          // the owner frees the layer
    h->d = *desc; h->P = P; h->K = K; h->Kp = Kp; h->Ho = Ho; h->Wo = Wo;
    std::vector<int8_t> w((size_t)N * K);
    std::vector<float> s(N), bias(N, 0.0f), ln_g(n_ln), ln_b(n_ln);
    if (hipMemcpy(w.data(), p->w, w.size(), hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(s.data(), p->s_w, (size_t)N * 4, hipMemcpyDeviceToHost) != hipSuccess ||
        (p->bias && hipMemcpy(bias.data(), p->bias, (size_t)N * 4, hipMemcpyDeviceToHost) != hipSuccess) ||
        hipMemcpy(ln_g.data(), p->ln_gamma, (size_t)n_ln * 4, hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(ln_b.data(), p->ln_beta, (size_t)n_ln * 4, hipMemcpyDeviceToHost) != hipSuccess)
        return bail(fail(MIXAQ_E_HIP, "copy of the parameters to the host failed"));
    const int wmax = (1 << (desc->weight_bits - 1)) - 1, wmin = -(1 << (desc->weight_bits - 1));
    std::vector<float> m(N);
    std::vector<int> nc(N);
    for (int n = 0; n < N; ++n) {
        if (!(s[n] > 0.0f) || !std::isfinite(s[n])) return bail(fail(MIXAQ_E_SHAPE, "weight scale %d is not positive", n));
        long long cs = 0;
        for (int k = 0; k < K; ++k) {
            const int v = w[(size_t)n * K + k];
            if (v < wmin || v > wmax) return bail(fail(MIXAQ_E_BITS, "weight code %d outside the %d-bit range", v, desc->weight_bits));
            cs += v;
        }
        m[n] = p->a_in.scale * s[n];
        nc[n] = (int)(-(long long)p->a_in.zero_point * cs);
    }
    const int NB = N / 32, KS = Kp / 32;
    std::vector<int8_t> packed((size_t)N * Kp, 0);
    for (int nb = 0; nb < NB; ++nb)
        for (int ks = 0; ks < KS; ++ks)
            for (int lane = 0; lane < 64; ++lane)
                for (int e = 0; e < 16; ++e) {
                    const int k = ks * 32 + (lane / 32) * 16 + e;
                    if (k < K) packed[(((size_t)nb * KS + ks) * 64 + lane) * 16 + e] = w[(size_t)(nb * 32 + lane % 32) * K + k];
                }
    int8_t* wp = nullptr;
    if ((rc = ds_upload(h, packed, &wp)) || (rc = ds_upload(h, m, &h->m)) || (rc = ds_upload(h, bias, &h->bias)) ||
        (rc = ds_upload(h, nc, &h->negcorr)) || (rc = ds_upload(h, ln_g, &h->gamma)) || (rc = ds_upload(h, ln_b, &h->beta)))
        return bail(rc);
    h->Wp = (v4i*)wp;
    h->q.scale = p->a_in.scale;
    h->q.zp = p->a_in.zero_point;
    h->q.inv_s = 1.0f / p->a_in.scale;
    h->q.magic = RND_MAGIC + (float)p->a_in.zero_point;
    h->q.lo = RND_MAGIC + (float)qmin;
    h->q.hi = RND_MAGIC + (float)qmax;
    owner.h = nullptr;
    *out = h;
    return MIXAQ_OK;
}

int mixaq_downsample_destroy(mixaq_downsample* h)
{
    delete h;
    return MIXAQ_OK;
}

int mixaq_downsample_forward(const mixaq_downsample* h, const float* x, float* y, void* stream)
{
    return ds_forward(h, x, y, stream, nullptr, nullptr);
}

int mixaq_downsample_forward_taps(const mixaq_downsample* h, const float* x, float* y, void* stream, int8_t* tap_codes,
                                  int32_t* tap_acc)
{
    return ds_forward(h, x, y, stream, tap_codes, tap_acc);
}

}  // extern "C"
