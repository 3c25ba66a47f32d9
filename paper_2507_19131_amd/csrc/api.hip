// C ABI of the Two-Branch Swin Block library (see include/mixaq.h): validation,
// parameter packing at create time, workspace layout and the launch sequence.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <utility>
#include <vector>

#include "../../include/mixaq.h"
#include "kernels.h"

using namespace mixaq;

namespace mixaq {
thread_local char g_err[512] = "";

// records the calling thread's error message and returns `code`
int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}
// Cubic coefficients of the GELU remainder H(a) = (a/2) erfc(a / sqrt 2): on interval i the cubic in the
// local coordinate d in [0,1) passes through H at the interval's ends and thirds.  Binary64 throughout,
// one rounding to binary32 per coefficient (then the exact power-of-two factor of the scaled evaluation).
void gelu_table(float* tab)
{
    static const double lagrange[3][4] = {{-11.0, 18.0, -9.0, 2.0}, {18.0, -45.0, 36.0, -9.0}, {-9.0, 27.0, -27.0, 9.0}};
    const double nodes_per_unit = 3.0 * (double)(1 << GELU_LOG2K);
    for (int i = 0; i < GELU_K; ++i) {
        double y[4];
        for (int j = 0; j < 4; ++j) {
            const double a = (double)(3 * i + j) / nodes_per_unit;
            y[j] = (0.5 * a) * std::erfc(a * 0.70710678118654752440);
        }
        tab[4 * i] = (float)y[0];
        for (int k = 0; k < 3; ++k) {
            double acc = lagrange[k][0] * y[0];
            for (int j = 1; j < 4; ++j) acc += lagrange[k][j] * y[j];
            tab[4 * i + 1 + k] = (float)(acc * 0.5);
        }
    }
    // the kernels work on values scaled by GELU_SCALE (see gelu_scaled): exact, a power of two
    for (int e = 0; e < 4 * GELU_K; ++e) tab[e] *= GELU_SCALE;
}
}  // namespace mixaq

namespace {

#define HIP_TRY(expr)                                                                                   \
    do {                                                                                                \
        hipError_t e_ = (expr);                                                                         \
        if (e_ != hipSuccess) return fail(MIXAQ_E_HIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

int round_up(int v, int m) { return (v + m - 1) / m * m; }
size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

int check_desc(const mixaq_block_desc* d)
{
    if (!d) return fail(MIXAQ_E_NULL, "descriptor is NULL");
    if (d->B < 1 || d->H < 1 || d->W < 1) return fail(MIXAQ_E_SHAPE, "B, H, W must be positive");
    if (d->window != WS) return fail(MIXAQ_E_SHAPE, "window must be 7 (got %d)", d->window);
    if (!channels_supported(d->C)) return fail(MIXAQ_E_SHAPE, "C=%d unsupported (96,128,192,256,384,512,768,1024)", d->C);
    if (d->heads < 1 || d->C != d->heads * HD) return fail(MIXAQ_E_SHAPE, "C/heads must be 32 (C=%d heads=%d)", d->C, d->heads);
    if (d->shift < 0 || d->shift >= WS) return fail(MIXAQ_E_SHAPE, "shift must be in 0..6");
    if (d->shift > 0 && (round_up(d->H, WS) < 2 * WS || round_up(d->W, WS) < 2 * WS))
        return fail(MIXAQ_E_SHAPE, "shift > 0 needs a padded map of at least 14x14");
    if (d->mlp_ratio < 1 || d->mlp_ratio > 8) return fail(MIXAQ_E_SHAPE, "mlp_ratio must be in 1..8");
    if (d->act_bits_high < 2 || d->act_bits_high > 8 || d->act_bits_low < 2 || d->act_bits_low > 8 ||
        d->weight_bits < 2 || d->weight_bits > 8)
        return fail(MIXAQ_E_BITS, "bit widths must be in 2..8");
    if (d->score_mode != 0 && d->score_mode != 1) return fail(MIXAQ_E_SHAPE, "score_mode must be 0 or 1");
    if (!(d->ln_eps > 0.0f)) return fail(MIXAQ_E_SHAPE, "ln_eps must be positive");
    long long nW = (long long)(round_up(d->H, WS) / WS) * (round_up(d->W, WS) / WS);
    if (nW > 4096) return fail(MIXAQ_E_SHAPE, "at most 4096 windows per image (got %lld)", nW);
    if ((long long)d->B * nW * TOK > (1LL << 30)) return fail(MIXAQ_E_SHAPE, "map too large for 32-bit row indexing");
    return MIXAQ_OK;
}

QDev make_qdev(mixaq_qparam p, int bits)
{
    QDev q;
    int qmin = -(1 << (bits - 1)), qmax = (1 << (bits - 1)) - 1;
    q.scale = p.scale;
    q.zp = p.zero_point;
    q.inv_s = 1.0f / p.scale;
    q.magic = RND_MAGIC + (float)p.zero_point;
    q.lo = RND_MAGIC + (float)qmin;
    q.hi = RND_MAGIC + (float)qmax;
    return q;
}

// device buffer owned by a block
template <typename T>
int upload(std::vector<void*>& owned, const std::vector<T>& host, T** dev)
{
    void* p = nullptr;
    size_t bytes = host.size() * sizeof(T);
    HIP_TRY(hipMalloc(&p, bytes ? bytes : 16));
    owned.push_back(p);
    if (bytes) HIP_TRY(hipMemcpy(p, host.data(), bytes, hipMemcpyHostToDevice));
    *dev = (T*)p;
    return MIXAQ_OK;
}

template <typename T>
int download(const T* dev, size_t n, std::vector<T>& host)
{
    host.resize(n);
    HIP_TRY(hipMemcpy(host.data(), dev, n * sizeof(T), hipMemcpyDeviceToHost));
    return MIXAQ_OK;
}

struct Linear {           // one shadow layer prepared for the device
    int K = 0, N = 0;
    v4i* Wp = nullptr;         // k bytes of a lane half in natural order (operand read from row-major memory)
    v4i* Wp_reg = nullptr;     // k bytes in the order of MFMA result registers (operand chained from registers)
    float* m[2] = {nullptr, nullptr};
    float* bias[2] = {nullptr, nullptr};
    int* negcorr[2] = {nullptr, nullptr};
    std::vector<int> colsum;   // sum_k W[n,k], kept on the host
};

}  // namespace

struct mixaq_block {
    mixaq_block_desc d;
    int Hp, Wp, nWc, nW;
    std::vector<void*> owned;
    Linear qkv, proj, fc1, fc2;
    float* ln_gamma[2][2];     // [which LN][branch]
    float* ln_beta[2][2];
    float* score_gamma = nullptr;
    float* score_beta = nullptr;
    float* bias2 = nullptr;
    QDev q_in[2], q_qkv[2][3], q_p[2], q_ao[2], q_fc1in[2], q_fc2in[2];
    float m2[2], m_o[2];
    float* tok_params[2] = {nullptr, nullptr};   // parameter blocks of the fused token kernel
    float* win_params[2] = {nullptr, nullptr};   // parameter blocks of the fused window kernel
    int ao_pack = 0;           // packing of the low branch's attention-output codes between the two fused kernels
    const float4* gelu_tab = nullptr;            // cubic coefficients of the pinned GELU
    size_t ws_bytes = 0;
    size_t ws_fused_bytes = 0; // what the two fused kernels alone need
    // Small maps in a batch (see mixaq_stage_forward): the stage runs as two chains, one per half of the images,
    // the second on this stream between the two events; created with the block when the shape qualifies.
    hipStream_t side_stream = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    bool fused_window = false; // the window kernel instead of gather/LN1 + QKV + attention kernels
    bool fused_token = false;  // the token kernel instead of proj + LN2 + FC1 + FC2 kernels
};

// ---- scratch of the entry point that allocates nothing -------------------------------------------
// One array per GPU the library runs on, held until the process ends.  Host code never uses the
// array's name as an address: static_scratch() asks the runtime for the device address once per
// device and every later use goes through that pointer.
static __device__ __align__(256) unsigned char scratch[MIXAQ_STATIC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;

int static_scratch(void** out)
{
    static std::mutex mu;
    static void* ptr[MAX_DEVICES] = {};
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(MIXAQ_E_HIP, "device %d outside 0..%d", dev, MAX_DEVICES - 1);
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(MIXAQ_E_HIP, "the runtime returned no address for the static scratch");
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return MIXAQ_OK;
}

// packs W[N,K] (row-major int8) into MFMA A-operand order and builds the per-branch epilogue constants
int prepare_linear(mixaq_block* blk, Linear& L, const int8_t* w_dev, const float* s_dev, int N, int K,
                   const float* const bias_dev[2], const mixaq_qparam in_q[2], int weight_bits, bool reg_order,
                   float out_scale = 1.0f)   // a power of two folded into the epilogue constants (exact; see gelu_scaled)
{
    std::vector<int8_t> w;
    std::vector<float> s, b;
    int rc;
    if ((rc = download(w_dev, (size_t)N * K, w))) return rc;
    if ((rc = download(s_dev, (size_t)N, s))) return rc;
    const int wmax = (1 << (weight_bits - 1)) - 1, wmin = -(1 << (weight_bits - 1));
    std::vector<int> colsum(N, 0);
    for (int n = 0; n < N; ++n) {
        if (!(s[n] > 0.0f) || !std::isfinite(s[n])) return fail(MIXAQ_E_SHAPE, "weight scale %d is not positive", n);
        for (int k = 0; k < K; ++k) {
            int v = w[(size_t)n * K + k];
            if (v < wmin || v > wmax) return fail(MIXAQ_E_BITS, "weight code %d outside the %d-bit range", v, weight_bits);
            colsum[n] += v;
        }
    }
    const int NB = N / 32, KS = K / 32;
    std::vector<int8_t> packed((size_t)N * K);
    for (int nb = 0; nb < NB; ++nb)
        for (int ks = 0; ks < KS; ++ks)
            for (int lane = 0; lane < 64; ++lane) {
                const int8_t* src = &w[(size_t)(nb * 32 + lane % 32) * K + ks * 32 + (lane / 32) * 16];
                memcpy(&packed[(((size_t)nb * KS + ks) * 64 + lane) * 16], src, 16);
            }
    L.K = K;
    L.N = N;
    L.colsum = colsum;
    int8_t* wp = nullptr;
    if ((rc = upload(blk->owned, packed, &wp))) return rc;
    L.Wp = (v4i*)wp;
    if (reg_order) {
        for (int nb = 0; nb < NB; ++nb)
            for (int ks = 0; ks < KS; ++ks)
                for (int lane = 0; lane < 64; ++lane)
                    for (int r = 0; r < 16; ++r) {
                        int k = ks * 32 + (r / 4) * 8 + (lane / 32) * 4 + r % 4;
                        packed[(((size_t)nb * KS + ks) * 64 + lane) * 16 + r] = w[(size_t)(nb * 32 + lane % 32) * K + k];
                    }
        if ((rc = upload(blk->owned, packed, &wp))) return rc;
        L.Wp_reg = (v4i*)wp;
    }
    for (int br = 0; br < 2; ++br) {
        if ((rc = download(bias_dev[br], (size_t)N, b))) return rc;
        std::vector<float> m(N);
        std::vector<int> nc(N);
        for (int n = 0; n < N; ++n) {
            m[n] = (in_q[br].scale * s[n]) * out_scale;
            b[n] *= out_scale;
            nc[n] = -in_q[br].zero_point * colsum[n];
        }
        if ((rc = upload(blk->owned, m, &L.m[br]))) return rc;
        if ((rc = upload(blk->owned, b, &L.bias[br]))) return rc;
        if ((rc = upload(blk->owned, nc, &L.negcorr[br]))) return rc;
    }
    return MIXAQ_OK;
}

// original padded coordinates of token t of window (wr,wc) in the rolled frame
void token_src(const mixaq_block* b, int wr, int wc, int t, int* r, int* c)
{
    *r = (wr * WS + t / WS + b->d.shift) % b->Hp;
    *c = (wc * WS + t % WS + b->d.shift) % b->Wp;
}

int check_qparam(const mixaq_qparam& q, int bits, const char* name)
{
    if (!(q.scale > 0.0f) || !std::isfinite(q.scale)) return fail(MIXAQ_E_SHAPE, "%s: scale must be positive", name);
    if (q.zero_point < -(1 << (bits - 1)) || q.zero_point > (1 << (bits - 1)) - 1)
        return fail(MIXAQ_E_SHAPE, "%s: zero point outside the %d-bit range", name, bits);
    return MIXAQ_OK;
}

// Two chains pay while the kernels of the stage leave CUs idle for part of their time: a batch of at least two maps
// with at most this many windows in all, on the fused kernels (config 3, 2 x 96 windows at C = 384: 0.36 instead of
// 0.41 ms per stage pass; 2 x 1392 windows at C = 96: 10 % faster; 4 x 1392: 4 %, no longer taken).
constexpr int STAGE_SPLIT_MAX_WINDOWS = 4096;
bool stage_splits(const mixaq_block* b)
{
    return b->d.B >= 2 && b->d.B * b->nW <= STAGE_SPLIT_MAX_WINDOWS && b->fused_window && b->fused_token;
}

void make_geom(const mixaq_block* b, int k_hi, int k_lo, Geom* G, int images = 0)
{
    const int nB = images > 0 ? images : b->d.B;
    G->B = nB; G->H = b->d.H; G->W = b->d.W; G->C = b->d.C; G->shift = b->d.shift; G->heads = b->d.heads;
    G->Hp = b->Hp; G->Wp = b->Wp; G->nWc = b->nWc; G->nW = b->nW;
    G->k_hi = k_hi; G->k_lo = k_lo; G->n_slots = nB * (k_hi + k_lo);
    G->rows_hi = nB * k_hi * TOK;
    G->rows_lo = nB * G->k_lo * TOK;
    G->base_lo = round_up(G->rows_hi, REGION_ALIGN);
    G->rows_total = G->base_lo + round_up(G->rows_lo, REGION_ALIGN);
}

struct Workspace {
    double* scores; int* perm; int* row_pix; int* row_canon;
    int8_t *a1, *qkv, *ao, *a2, *g; float* h;
};

// fused_only: only what the window kernel and the token kernel exchange (scores, list, row bookkeeping,
// attention-output codes); the buffers of the seven-kernel path stay NULL
int rows_max_of(const mixaq_block* b, int images) { return round_up(images * b->nW * TOK, REGION_ALIGN) + REGION_ALIGN; }

size_t carve(const mixaq_block* b, char* base, Workspace* w, bool fused_only = false, int images = 0)
{
    size_t off = 0;
    const int nB = images > 0 ? images : b->d.B;
    const size_t R = rows_max_of(b, nB), C = b->d.C, S = (size_t)nB * b->nW, F = C * b->d.mlp_ratio;
    auto take = [&](size_t bytes) { char* p = base ? base + off : nullptr; off += align256(bytes); return p; };
    *w = Workspace{};
    w->scores = (double*)take(S * 8);
    w->perm = (int*)take(S * 4);
    w->row_pix = (int*)take(R * 4);
    w->row_canon = (int*)take(R * 4);
    w->ao = (int8_t*)take(R * C);
    if (fused_only) return off;
    w->a1 = (int8_t*)take(R * C);
    w->qkv = (int8_t*)take(R * 3 * C);
    w->h = (float*)take(R * C * 4);
    w->a2 = (int8_t*)take(R * C);
    w->g = (int8_t*)take(R * F);
    return off;
}

// optional per-kernel timing: one event before every launch and one after the last
struct Prof {
    hipEvent_t ev[MIXAQ_NUM_KERNELS + 1];
    int idx[MIXAQ_NUM_KERNELS + 1];
    int n = 0;
    int repeats = 1;          // every kernel is launched this many times between its two events
};

// a run of images of the batch handled by one call of forward_impl (images = 0: the whole batch), and where its
// part of the workspace starts
struct Part { int first = 0, images = 0; size_t ws_offset = 0; };

int forward_impl(const mixaq_block* blk, const float* x, const int32_t* perm, const double* scores, int32_t k_high,
                 int32_t k_low, float* y, void* workspace, size_t workspace_bytes, void* stream, const mixaq_taps* taps,
                 Prof* prof = nullptr, int32_t* perm_out = nullptr, bool fused_only = false, Part part = Part())
{
    if (!blk) return fail(MIXAQ_E_NULL, "block is NULL");
    if (!x || !y) return fail(MIXAQ_E_NULL, "x or y is NULL");
    if (!workspace) return fail(MIXAQ_E_NULL, "workspace is NULL");
    if (k_low < 0) k_low = blk->nW - k_high;      // no pruning
    if (k_high < 0 || k_low < 0 || k_high + k_low > blk->nW)
        return fail(MIXAQ_E_SHAPE, "k_high=%d, k_low=%d do not fit %d windows", k_high, k_low, blk->nW);
    if (fused_only && !(blk->fused_window && blk->fused_token))
        return fail(MIXAQ_E_SHAPE, "this call needs the fused kernels (C <= 384, mlp_ratio 4, not switched off)");
    Workspace ws;
    const size_t ws_need = part.images ? part.ws_offset + carve(blk, nullptr, &ws, fused_only, part.images)
                                       : (fused_only ? blk->ws_fused_bytes : blk->ws_bytes);
    if (workspace_bytes < ws_need) return fail(MIXAQ_E_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, ws_need);
    if ((uintptr_t)workspace & 255) return fail(MIXAQ_E_WORKSPACE, "workspace must be 256-byte aligned");
    {
        const char *xa = (const char*)x, *ya = (const char*)y;
        size_t bytes = (size_t)blk->d.B * blk->d.H * blk->d.W * blk->d.C * 4;
        if (xa < ya + bytes && ya < xa + bytes) return fail(MIXAQ_E_SHAPE, "x and y overlap");
    }
    hipStream_t st = (hipStream_t)stream;
    const mixaq_block_desc& d = blk->d;
    Geom G;
    make_geom(blk, k_high, k_low, &G, part.images);
    carve(blk, (char*)workspace + part.ws_offset, &ws, fused_only, part.images);
    if (part.first) {                       // the part's images in the map, the scores and the lists
        const size_t px = (size_t)part.first * d.H * d.W * d.C, lw = (size_t)part.first * blk->nW;
        x += px; y += px;
        if (perm) perm += lw;
        if (scores) scores += lw;
        if (perm_out) perm_out += lw;
    }
    static const mixaq_taps no_taps = {};
    const mixaq_taps& tp = taps ? *taps : no_taps;

    const int reps = prof ? prof->repeats : 1;
    auto mark = [&](int kernel) {
        if (prof) { prof->idx[prof->n] = kernel; (void)hipEventRecord(prof->ev[prof->n++], st); }
    };
    if (!perm && !scores) {     // score here (single-block use)
        mark(0);
        for (int r = 0; r < reps; ++r) launch_score(G, x, d.score_mode, d.ln_eps, blk->score_gamma, blk->score_beta, ws.scores, st);
        scores = ws.scores;
    }
    // the fused window kernel ranks the windows itself when it is given scores; the other path selects first
    const bool fw = blk->fused_window, ft = blk->fused_token;
    const bool in_kernel_select = !perm && fw;
    if (!perm && !in_kernel_select) {
        mark(1);
        for (int r = 0; r < reps; ++r) launch_select(scores, d.B, blk->nW, 0, perm_out ? perm_out : ws.perm, st);
        perm = perm_out ? perm_out : ws.perm;
    }
    auto fill = [&](GemmArgs& a, const Linear& L, const int8_t* act) {
        a = GemmArgs{};
        a.A = act; a.Wp = L.Wp; a.K = L.K; a.N = L.N;
        for (int br = 0; br < 2; ++br) { a.m[br] = L.m[br]; a.bias[br] = L.bias[br]; a.negcorr[br] = L.negcorr[br]; }
        a.row_pix = ws.row_pix; a.row_canon = ws.row_canon;
        a.gelu_tab = blk->gelu_tab;
    };
    GemmArgs ga;
    LnArgs la = {};
    // ---- first half: gather + LN1 + quantize, QKV, windowed attention -> attention-output codes, row bookkeeping
    if (fw) {
        WinArgs wa = {};
        wa.x = x; wa.perm = perm; wa.scores = in_kernel_select ? scores : nullptr; wa.perm_out = perm_out ? perm_out : ws.perm;
        wa.y = y; wa.eps = d.ln_eps; wa.Wqkv = blk->qkv.Wp; wa.bias2 = blk->bias2; wa.out = ws.ao;
        wa.row_pix = ws.row_pix; wa.row_canon = ws.row_canon;
        wa.out_pack = ft ? blk->ao_pack : 0;
        for (int br = 0; br < 2; ++br) {
            wa.params[br] = blk->win_params[br]; wa.q_in[br] = blk->q_in[br];
            for (int k = 0; k < 3; ++k) wa.q_qkv[br][k] = blk->q_qkv[br][k];
            wa.m2[br] = blk->m2[br]; wa.m_o[br] = blk->m_o[br]; wa.qp[br] = blk->q_p[br]; wa.qo[br] = blk->q_ao[br];
        }
        wa.tap_a1 = tp.a_qkv_in; wa.tap_acc = tp.acc_qkv; wa.tap_qkv = tp.qkv; wa.tap_s = tp.acc_s; wa.tap_p = tp.p;
        wa.tap_o = tp.acc_o; wa.tap_code = tp.a_proj_in;
        wa.poly = pinned_coefficients();
        wa.taps = taps != nullptr;
        mark(9);
        for (int r = 0; r < reps; ++r) launch_window(G, wa, st);       // also forwards pruned windows
    } else {
        launch_bypass(G, perm, x, y, st);                              // pruned windows (if any) are forwarded
        la.perm = perm; la.src = x; la.eps = d.ln_eps; la.out = ws.a1; la.row_pix = ws.row_pix; la.row_canon = ws.row_canon;
        la.tap = tp.a_qkv_in;
        for (int br = 0; br < 2; ++br) { la.gamma[br] = blk->ln_gamma[0][br]; la.beta[br] = blk->ln_beta[0][br]; la.q[br] = blk->q_in[br]; }
        mark(2);
        for (int r = 0; r < reps; ++r) launch_ln_quant(G, la, true, st);
        fill(ga, blk->qkv, ws.a1);
        for (int br = 0; br < 2; ++br) for (int k = 0; k < 3; ++k) ga.q[br][k] = blk->q_qkv[br][k];
        ga.out8 = ws.qkv; ga.tap_acc = tp.acc_qkv; ga.tap_code = tp.qkv;
        mark(3);
        for (int r = 0; r < reps; ++r) launch_gemm(G, ga, EPI_QKV, st);
        AttnArgs aa = {};
        aa.qkv = ws.qkv; aa.perm = perm; aa.bias2 = blk->bias2; aa.out = ws.ao;
        for (int br = 0; br < 2; ++br) { aa.m2[br] = blk->m2[br]; aa.m_o[br] = blk->m_o[br]; aa.qp[br] = blk->q_p[br]; aa.qo[br] = blk->q_ao[br]; }
        aa.poly = pinned_coefficients();
        aa.tap_s = tp.acc_s; aa.tap_p = tp.p; aa.tap_o = tp.acc_o; aa.tap_code = tp.a_proj_in;
        mark(4);
        for (int r = 0; r < reps; ++r) launch_attn(G, aa, st);
    }
    // ---- second half: projection + residual, LN2, FFN, second residual, scatter
    if (ft) {
        TokArgs ta = {};
        ta.ao = ws.ao; ta.x = x; ta.y = y; ta.row_pix = ws.row_pix; ta.row_canon = ws.row_canon; ta.eps = d.ln_eps;
        ta.Wproj = blk->proj.Wp; ta.W1 = blk->fc1.Wp_reg; ta.W2 = blk->fc2.Wp_reg;
        ta.ao_pack = blk->ao_pack;
        for (int br = 0; br < 2; ++br) {
            ta.params[br] = blk->tok_params[br];
            ta.q_fc1in[br] = blk->q_fc1in[br]; ta.q_fc2in[br] = blk->q_fc2in[br];
        }
        ta.tap_acc_proj = tp.acc_proj; ta.tap_h = tp.h; ta.tap_a2 = tp.a_fc1_in; ta.tap_acc_fc1 = tp.acc_fc1;
        ta.tap_g = tp.a_fc2_in; ta.tap_acc_fc2 = tp.acc_fc2; ta.tap_y = tp.y_win;
        ta.gelu_tab = blk->gelu_tab;
        ta.taps = taps != nullptr;
        mark(10);
        for (int r = 0; r < reps; ++r) launch_token(G, ta, st);
        mark(-1);
        HIP_TRY(hipGetLastError());
        return MIXAQ_OK;
    }
    // output projection + first residual
    fill(ga, blk->proj, ws.ao);
    ga.outf = ws.h; ga.x = x; ga.tap_acc = tp.acc_proj; ga.tap_f = tp.h;
    mark(5);
    for (int r = 0; r < reps; ++r) launch_gemm(G, ga, EPI_PROJ, st);
    // LN2 + quantize
    la = LnArgs{};
    la.eps = d.ln_eps; la.row_pix = ws.row_pix; la.row_canon = ws.row_canon;
    la.perm = nullptr; la.src = ws.h; la.out = ws.a2; la.tap = tp.a_fc1_in;
    for (int br = 0; br < 2; ++br) { la.gamma[br] = blk->ln_gamma[1][br]; la.beta[br] = blk->ln_beta[1][br]; la.q[br] = blk->q_fc1in[br]; }
    mark(6);
    for (int r = 0; r < reps; ++r) launch_ln_quant(G, la, false, st);
    // FFN
    fill(ga, blk->fc1, ws.a2);
    for (int br = 0; br < 2; ++br) ga.q[br][0] = blk->q_fc2in[br];
    ga.out8 = ws.g; ga.tap_acc = tp.acc_fc1; ga.tap_code = tp.a_fc2_in;
    mark(7);
    for (int r = 0; r < reps; ++r) launch_gemm(G, ga, EPI_FC1, st);
    fill(ga, blk->fc2, ws.g);
    ga.resid = ws.h; ga.y = y; ga.tap_acc = tp.acc_fc2; ga.tap_f = tp.y_win;
    mark(8);
    for (int r = 0; r < reps; ++r) launch_gemm(G, ga, EPI_FC2, st);
    mark(-1);
    HIP_TRY(hipGetLastError());
    return MIXAQ_OK;
}

}  // namespace

extern "C" {

int mixaq_version(void) { return 100; }

const char* mixaq_last_error(void) { return g_err; }

int mixaq_num_windows(const mixaq_block_desc* desc, int32_t* nW)
{
    int rc = check_desc(desc);
    if (rc) return rc;
    if (!nW) return fail(MIXAQ_E_NULL, "nW_per_image is NULL");
    *nW = (round_up(desc->H, WS) / WS) * (round_up(desc->W, WS) / WS);
    return MIXAQ_OK;
}

int mixaq_keep_count(int32_t nW, double keep_ratio, int32_t* k_high)
{
    if (!k_high) return fail(MIXAQ_E_NULL, "k_high is NULL");
    if (nW < 0 || !(keep_ratio >= 0.0) || !(keep_ratio <= 1.0)) return fail(MIXAQ_E_SHAPE, "need nW >= 0 and 0 <= keep_ratio <= 1");
    double k = std::floor(keep_ratio * (double)nW + 0.5);
    if (k < 0) k = 0;
    if (k > nW) k = nW;
    *k_high = (int32_t)k;
    return MIXAQ_OK;
}

static int block_create(const mixaq_block_desc* desc, const mixaq_shared_params* sh, const mixaq_branch_params branch[2],
                        void* stream, mixaq_block** out);

// No C++ exception leaves the library: host containers that fail to allocate become an error code.
int mixaq_block_create(const mixaq_block_desc* desc, const mixaq_shared_params* sh, const mixaq_branch_params branch[2],
                       void* stream, mixaq_block** out)
{
    try {
        return block_create(desc, sh, branch, stream, out);
    } catch (const std::bad_alloc&) {
        return fail(MIXAQ_E_HIP, "out of host memory while preparing the block");
    } catch (...) {
        return fail(MIXAQ_E_HIP, "unexpected C++ exception while preparing the block");
    }
}

namespace {
struct BlockOwner {                      // destroys a half-built block on every early return and on an exception
    mixaq_block* b;
    ~BlockOwner() { if (b) mixaq_block_destroy(b); }
};
}  // namespace

static int block_create(const mixaq_block_desc* desc, const mixaq_shared_params* sh, const mixaq_branch_params branch[2],
                        void* stream, mixaq_block** out)
{
    int rc = check_desc(desc);
    if (rc) return rc;
    if (!sh || !branch || !out) return fail(MIXAQ_E_NULL, "shared, branch or out is NULL");
    if (!sh->w_qkv || !sh->w_proj || !sh->w_fc1 || !sh->w_fc2 || !sh->s_qkv || !sh->s_proj || !sh->s_fc1 || !sh->s_fc2 ||
        !sh->rel_pos_bias)
        return fail(MIXAQ_E_NULL, "a shared parameter pointer is NULL");
    if (desc->score_mode == 1 && (!sh->score_gamma || !sh->score_beta)) return fail(MIXAQ_E_NULL, "score_mode 1 needs score_gamma/beta");
    for (int br = 0; br < 2; ++br) {
        const mixaq_branch_params& p = branch[br];
        if (!p.ln1_gamma || !p.ln1_beta || !p.ln2_gamma || !p.ln2_beta || !p.b_qkv || !p.b_proj || !p.b_fc1 || !p.b_fc2)
            return fail(MIXAQ_E_NULL, "a parameter pointer of branch %d is NULL", br);
        int bits = br == 0 ? desc->act_bits_high : desc->act_bits_low;
        const mixaq_qparam* q = &p.a_qkv_in;
        static const char* names[8] = {"a_qkv_in", "a_q", "a_k", "a_v", "a_p", "a_proj_in", "a_fc1_in", "a_fc2_in"};
        for (int k = 0; k < 8; ++k) if ((rc = check_qparam(q[k], bits, names[k]))) return rc;
        if (p.a_q.zero_point || p.a_k.zero_point || p.a_v.zero_point) return fail(MIXAQ_E_SHAPE, "zero points of q, k, v must be 0");
    }
    HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    mixaq_block* b = new (std::nothrow) mixaq_block();
    if (!b) return fail(MIXAQ_E_HIP, "out of host memory");
    b->d = *desc;
    b->Hp = round_up(desc->H, WS); b->Wp = round_up(desc->W, WS);
    b->nWc = b->Wp / WS; b->nW = (b->Hp / WS) * b->nWc;
    const int C = desc->C, F = C * desc->mlp_ratio, heads = desc->heads;
    BlockOwner owner{b};
    auto bail = [&](int code) { return code; };          // the owner destroys the block
    mixaq_qparam qi[2];
    const float* bias[2];
    qi[0] = branch[0].a_qkv_in; qi[1] = branch[1].a_qkv_in; bias[0] = branch[0].b_qkv; bias[1] = branch[1].b_qkv;
    if ((rc = prepare_linear(b, b->qkv, sh->w_qkv, sh->s_qkv, 3 * C, C, bias, qi, desc->weight_bits, false))) return bail(rc);
    qi[0] = branch[0].a_proj_in; qi[1] = branch[1].a_proj_in; bias[0] = branch[0].b_proj; bias[1] = branch[1].b_proj;
    if ((rc = prepare_linear(b, b->proj, sh->w_proj, sh->s_proj, C, C, bias, qi, desc->weight_bits, false))) return bail(rc);
    qi[0] = branch[0].a_fc1_in; qi[1] = branch[1].a_fc1_in; bias[0] = branch[0].b_fc1; bias[1] = branch[1].b_fc1;
    if ((rc = prepare_linear(b, b->fc1, sh->w_fc1, sh->s_fc1, F, C, bias, qi, desc->weight_bits, true, GELU_SCALE))) return bail(rc);
    qi[0] = branch[0].a_fc2_in; qi[1] = branch[1].a_fc2_in; bias[0] = branch[0].b_fc2; bias[1] = branch[1].b_fc2;
    if ((rc = prepare_linear(b, b->fc2, sh->w_fc2, sh->s_fc2, C, F, bias, qi, desc->weight_bits, true))) return bail(rc);
    std::vector<float> tmp;
    for (int br = 0; br < 2; ++br) {
        const float* src[4] = {branch[br].ln1_gamma, branch[br].ln1_beta, branch[br].ln2_gamma, branch[br].ln2_beta};
        float** dst[4] = {&b->ln_gamma[0][br], &b->ln_beta[0][br], &b->ln_gamma[1][br], &b->ln_beta[1][br]};
        for (int k = 0; k < 4; ++k) {
            if ((rc = download(src[k], (size_t)C, tmp))) return bail(rc);
            if ((rc = upload(b->owned, tmp, dst[k]))) return bail(rc);
        }
        int bits = br == 0 ? desc->act_bits_high : desc->act_bits_low;
        b->q_in[br] = make_qdev(branch[br].a_qkv_in, bits);
        b->q_qkv[br][0] = make_qdev(branch[br].a_q, bits);
        b->q_qkv[br][1] = make_qdev(branch[br].a_k, bits);
        b->q_qkv[br][2] = make_qdev(branch[br].a_v, bits);
        b->q_p[br] = make_qdev(branch[br].a_p, bits);
        b->q_ao[br] = make_qdev(branch[br].a_proj_in, bits);
        b->q_fc1in[br] = make_qdev(branch[br].a_fc1_in, bits);
        b->q_fc2in[br] = make_qdev(branch[br].a_fc2_in, bits);
        b->q_fc2in[br].inv_s /= GELU_SCALE;              // it quantizes the scaled GELU output (exact, a power of two)
        b->m2[br] = ((branch[br].a_q.scale * branch[br].a_k.scale) * (float)(1.0 / std::sqrt((double)HD))) * LOG2E_F;
        b->m_o[br] = branch[br].a_p.scale * branch[br].a_v.scale;
    }
    if (desc->score_mode == 1) {
        if ((rc = download(sh->score_gamma, (size_t)C, tmp))) return bail(rc);
        if ((rc = upload(b->owned, tmp, &b->score_gamma))) return bail(rc);
        if ((rc = download(sh->score_beta, (size_t)C, tmp))) return bail(rc);
        if ((rc = upload(b->owned, tmp, &b->score_beta))) return bail(rc);
    }
    // (relative position bias + shift mask) * log2(e), transposed to [type][head][key][query 64]
    {
        std::vector<float> rpb;
        if ((rc = download(sh->rel_pos_bias, (size_t)heads * TOK * TOK, rpb))) return bail(rc);
        std::vector<float> tab((size_t)4 * heads * TOK * 64, 0.0f);
        const int nWr = b->Hp / WS;
        for (int type = 0; type < 4; ++type) {
            int wr = (type & 2) ? nWr - 1 : 0, wc = (type & 1) ? b->nWc - 1 : 0;
            for (int h = 0; h < heads; ++h)
                for (int i = 0; i < TOK; ++i)
                    for (int j = 0; j < TOK; ++j) {
                        float v = rpb[((size_t)h * TOK + i) * TOK + j];
                        if (desc->shift > 0) {
                            int ri, ci, rj, cj;
                            token_src(b, wr, wc, i, &ri, &ci);
                            token_src(b, wr, wc, j, &rj, &cj);
                            if (!(std::abs(ri - rj) < WS && std::abs(ci - cj) < WS)) v = v + MASK_VALUE;
                        }
                        tab[(((size_t)type * heads + h) * TOK + j) * 64 + i] = v * LOG2E_F;
                    }
        }
        if ((rc = upload(b->owned, tab, &b->bias2))) return bail(rc);
    }
    {
        std::vector<float> tab((size_t)GELU_K * 4);
        gelu_table(tab.data());
        float* dev = nullptr;
        if ((rc = upload(b->owned, tab, &dev))) return bail(rc);
        b->gelu_tab = (const float4*)dev;
    }
    b->fused_window = fused_window_supported(C);
    b->fused_token = fused_token_supported(C, desc->mlp_ratio);
    auto gather_block = [&](const std::vector<std::pair<const void*, int>>& parts, float** dst) {
        size_t words = 0;
        for (auto& pt : parts) words += pt.second;
        std::vector<float> blkp(words);
        size_t off = 0;
        for (auto& pt : parts) {
            if (hipMemcpy(blkp.data() + off, pt.first, (size_t)pt.second * 4, hipMemcpyDeviceToHost) != hipSuccess)
                return fail(MIXAQ_E_HIP, "copy of a parameter block failed");
            off += pt.second;
        }
        return upload(b->owned, blkp, dst);
    };
    if (b->fused_window)      // parameter blocks of the window kernel
        for (int br = 0; br < 2; ++br)
            if ((rc = gather_block({{b->ln_gamma[0][br], C}, {b->ln_beta[0][br], C}, {b->qkv.m[br], 3 * C}, {b->qkv.bias[br], 3 * C},
                                    {b->qkv.negcorr[br], 3 * C}}, &b->win_params[br])))
                return bail(rc);
    // Both fused kernels present: the low branch's attention-output codes cross between them packed (two or four
    // per byte, offset-binary); the projection of packed rows then starts at -(zp + offset) * colsum.
    if (b->fused_window && b->fused_token) b->ao_pack = pack_mode(desc->act_bits_low);
    if (b->fused_token) {     // parameter blocks of the token kernel: device-to-device gathers of what was just uploaded
        for (int br = 0; br < 2; ++br) {
            std::vector<float> blkp((size_t)8 * C + 3 * F);
            struct { const void* src; int n; } parts[11] = {
                {b->proj.m[br], C}, {b->proj.bias[br], C}, {b->proj.negcorr[br], C}, {b->ln_gamma[1][br], C},
                {b->ln_beta[1][br], C}, {b->fc2.m[br], C}, {b->fc2.bias[br], C}, {b->fc2.negcorr[br], C},
                {b->fc1.m[br], F}, {b->fc1.bias[br], F}, {b->fc1.negcorr[br], F}};
            size_t off = 0;
            for (auto& pt : parts) {
                if (hipMemcpy(blkp.data() + off, pt.src, (size_t)pt.n * 4, hipMemcpyDeviceToHost) != hipSuccess)
                    return bail(fail(MIXAQ_E_HIP, "copy of a parameter block failed"));
                off += pt.n;
            }
            if (br == 1 && b->ao_pack) {       // packed rows carry u = code + offset: the projection removes zp + offset
                const int shift_by = branch[1].a_proj_in.zero_point + pack_offset(b->ao_pack);
                int* nc = (int*)blkp.data() + 2 * C;
                for (int n = 0; n < C; ++n) nc[n] = -shift_by * b->proj.colsum[n];
            }
            if ((rc = upload(b->owned, blkp, &b->tok_params[br]))) return bail(rc);
        }
    }
    Workspace w;
    b->ws_bytes = carve(b, nullptr, &w);
    b->ws_fused_bytes = carve(b, nullptr, &w, true);
    if (stage_splits(b)) {                  // two chains: each half of the images has its own part of the workspace
        b->ws_bytes = std::max(b->ws_bytes, carve(b, nullptr, &w, false, (desc->B + 1) / 2) + carve(b, nullptr, &w, false, desc->B / 2));
        if (hipStreamCreateWithFlags(&b->side_stream, hipStreamNonBlocking) != hipSuccess ||
            hipEventCreateWithFlags(&b->ev_fork, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&b->ev_join, hipEventDisableTiming) != hipSuccess)
            return bail(fail(MIXAQ_E_HIP, "creating the second stream of the stage failed"));
    }
    owner.b = nullptr;
    *out = b;
    return MIXAQ_OK;
}

int mixaq_block_destroy(mixaq_block* blk)
{
    if (!blk) return MIXAQ_OK;
    for (void* p : blk->owned) (void)hipFree(p);
    if (blk->ev_fork) (void)hipEventDestroy(blk->ev_fork);
    if (blk->ev_join) (void)hipEventDestroy(blk->ev_join);
    if (blk->side_stream) (void)hipStreamDestroy(blk->side_stream);
    delete blk;
    return MIXAQ_OK;
}

int mixaq_block_workspace_bytes(const mixaq_block* blk, size_t* bytes)
{
    if (!blk || !bytes) return fail(MIXAQ_E_NULL, "block or bytes is NULL");
    *bytes = blk->ws_bytes;
    return MIXAQ_OK;
}

int mixaq_score_windows(const mixaq_block* blk, const float* x, double* scores, void* stream)
{
    if (!blk || !x || !scores) return fail(MIXAQ_E_NULL, "block, x or scores is NULL");
    Geom G;
    make_geom(blk, 0, blk->nW, &G);
    launch_score(G, x, blk->d.score_mode, blk->d.ln_eps, blk->score_gamma, blk->score_beta, scores, (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return MIXAQ_OK;
}

int mixaq_select_windows3(const double* scores, int32_t B, int32_t nW, int32_t k_high, int32_t k_low, int32_t reverse,
                          int32_t* perm, void* stream)
{
    if (!scores || !perm) return fail(MIXAQ_E_NULL, "scores or perm is NULL");
    if (B < 1 || nW < 1 || k_high < 0 || k_low < 0 || k_high + k_low > nW)
        return fail(MIXAQ_E_SHAPE, "need B >= 1, nW >= 1, k_high >= 0, k_low >= 0, k_high + k_low <= nW");
    if (nW > 4096) return fail(MIXAQ_E_SHAPE, "at most 4096 windows per image");
    launch_select(scores, B, nW, reverse ? 1 : 0, perm, (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return MIXAQ_OK;
}

int mixaq_select_windows(const double* scores, int32_t B, int32_t nW, int32_t k_high, int32_t reverse, int32_t* perm,
                         void* stream)
{
    if (k_high < 0 || k_high > nW) return fail(MIXAQ_E_SHAPE, "need 0 <= k_high <= nW");
    return mixaq_select_windows3(scores, B, nW, k_high, nW - k_high, reverse, perm, stream);
}

int mixaq_block_forward(const mixaq_block* blk, const float* x, const int32_t* perm, int32_t k_high, float* y,
                        void* workspace, size_t workspace_bytes, void* stream)
{
    return forward_impl(blk, x, perm, nullptr, k_high, -1, y, workspace, workspace_bytes, stream, nullptr);
}

int mixaq_block_forward_scored(const mixaq_block* blk, const float* x, const double* scores, int32_t k_high, int32_t k_low,
                               float* y, int32_t* perm_out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!scores) return fail(MIXAQ_E_NULL, "scores is NULL");
    return forward_impl(blk, x, nullptr, scores, k_high, k_low, y, workspace, workspace_bytes, stream, nullptr, nullptr,
                        perm_out);
}

int mixaq_stage_forward(mixaq_block* const* blocks, int32_t n_blocks, const float* x, const int32_t* k_high,
                        const int32_t* k_low, float* y, float* tmp, double* scores, int32_t* perm, void* workspace,
                        size_t workspace_bytes, void* stream)
{
    if (!blocks || !x || !k_high || !y || !scores || !perm) return fail(MIXAQ_E_NULL, "a required pointer is NULL");
    if (n_blocks < 1) return fail(MIXAQ_E_SHAPE, "n_blocks = %d", n_blocks);
    if (n_blocks > 1 && !tmp) return fail(MIXAQ_E_NULL, "tmp is NULL (needed for more than one block)");
    for (int i = 0; i < n_blocks; ++i) {
        if (!blocks[i]) return fail(MIXAQ_E_NULL, "blocks[%d] is NULL", i);
        const mixaq_block_desc &a = blocks[0]->d, &b = blocks[i]->d;
        if (a.B != b.B || a.H != b.H || a.W != b.W || a.C != b.C)
            return fail(MIXAQ_E_SHAPE, "blocks[%d] was created for another map shape", i);
    }
    {   // the blocks alternate between tmp and y while later blocks (or the other chain) may still read x
        const mixaq_block_desc& d0 = blocks[0]->d;
        const size_t bytes = (size_t)d0.B * d0.H * d0.W * d0.C * 4;
        auto overlap = [&](const float* a, const float* c) {
            return a && c && (const char*)a < (const char*)c + bytes && (const char*)c < (const char*)a + bytes;
        };
        if (overlap(x, y) || overlap(x, tmp) || overlap(y, tmp)) return fail(MIXAQ_E_SHAPE, "x, y and tmp must not overlap");
    }
    const int nW = blocks[0]->nW;
    for (int p = 0; p < (n_blocks + 1) / 2; ++p) {
        const int kh = k_high[p], kl = k_low ? k_low[p] : nW - kh;
        if (kh < 0 || kl < 0 || kh + kl > nW) return fail(MIXAQ_E_SHAPE, "pair %d: k_high %d, k_low %d of %d windows", p, kh, kl, nW);
    }
    int rc = mixaq_score_windows(blocks[0], x, scores, stream);
    if (rc) return rc;
    // A batch of small maps (stage_splits) runs as two chains of blocks, one per half of the images, the second on the
    // first block's side stream: the images are independent through the whole stage, every kernel of such a map leaves
    // CUs idle, and the window kernel of one half runs beside the token kernel of the other.  Not under stream capture.
    hipStream_t st = (hipStream_t)stream;
    const mixaq_block* b0 = blocks[0];
    Part parts[2];
    int n_parts = 1;
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    bool split = n_blocks > 1 && b0->side_stream != nullptr;
    for (int i = 0; split && i < n_blocks; ++i) split = blocks[i]->fused_window && blocks[i]->fused_token;
    if (split) {
        if (hipStreamIsCapturing(st, &capturing) != hipSuccess) {
            (void)hipGetLastError();                                  // not to be mistaken for a launch error later
            split = false;
        } else if (capturing != hipStreamCaptureStatusNone) split = false;
    }
    if (split) {
        Workspace w;
        n_parts = 2;
        parts[0].first = 0; parts[0].images = (b0->d.B + 1) / 2; parts[0].ws_offset = 0;
        parts[1].first = parts[0].images; parts[1].images = b0->d.B / 2;
        parts[1].ws_offset = carve(b0, nullptr, &w, false, parts[0].images);
        HIP_TRY(hipEventRecord(b0->ev_fork, st));                    // both chains start together (the second one window kernel behind
        HIP_TRY(hipStreamWaitEvent(b0->side_stream, b0->ev_fork, 0)); // the first measured slower: 0.377 against 0.361 ms at config 3)
    }
    const float* cur = x;
    for (int i = 0; i < n_blocks && !rc; ++i) {
        float* dst = ((n_blocks - 1 - i) & 1) ? tmp : y;            // the last block writes y
        const int kh = k_high[i / 2], kl = k_low ? k_low[i / 2] : nW - kh;
        for (int p = 0; p < n_parts && !rc; ++p) {
            void* sp = p == 0 ? stream : (void*)b0->side_stream;
            if (i == 0) rc = forward_impl(blocks[0], cur, nullptr, scores, kh, kl, dst, workspace, workspace_bytes, sp, nullptr, nullptr, perm, false, parts[p]);
            else rc = forward_impl(blocks[i], cur, perm, nullptr, kh, kl, dst, workspace, workspace_bytes, sp, nullptr, nullptr, nullptr, false, parts[p]);
        }
        cur = dst;
    }
    if (split) {                                                     // the side chain joins, also after an error in between
        (void)hipEventRecord(b0->ev_join, b0->side_stream);
        (void)hipStreamWaitEvent(st, b0->ev_join, 0);
    }
    return rc;
}

int mixaq_block_forward_pruned(const mixaq_block* blk, const float* x, const int32_t* perm, int32_t k_high, int32_t k_low,
                               float* y, void* workspace, size_t workspace_bytes, void* stream)
{
    if (k_low < 0) return fail(MIXAQ_E_SHAPE, "k_low must not be negative");
    return forward_impl(blk, x, perm, nullptr, k_high, k_low, y, workspace, workspace_bytes, stream, nullptr);
}

int mixaq_block_forward_taps(const mixaq_block* blk, const float* x, const int32_t* perm, int32_t k_high, float* y,
                             void* workspace, size_t workspace_bytes, void* stream, const mixaq_taps* taps)
{
    return forward_impl(blk, x, perm, nullptr, k_high, -1, y, workspace, workspace_bytes, stream, taps);
}

int mixaq_block_forward_static(const mixaq_block* blk, const float* x, const int32_t* perm, int32_t k_high, float* y,
                               void* stream)
{
    if (!blk) return fail(MIXAQ_E_NULL, "block is NULL");
    if (!(blk->fused_window && blk->fused_token))
        return fail(MIXAQ_E_SHAPE, "this call needs the fused kernels (C <= 384, mlp_ratio 4, not switched off)");
    if (blk->ws_fused_bytes > (size_t)MIXAQ_STATIC_SCRATCH_BYTES)
        return fail(MIXAQ_E_WORKSPACE, "the map needs %zu bytes of scratch, the static scratch holds %zu", blk->ws_fused_bytes,
                    (size_t)MIXAQ_STATIC_SCRATCH_BYTES);
    void* ws = nullptr;
    int rc = static_scratch(&ws);
    if (rc) return rc;
    return forward_impl(blk, x, perm, nullptr, k_high, -1, y, ws, (size_t)MIXAQ_STATIC_SCRATCH_BYTES, stream, nullptr, nullptr, nullptr,
                        true);
}

int mixaq_block_set_fused(mixaq_block* blk, int32_t enable)
{
    if (!blk) return fail(MIXAQ_E_NULL, "block is NULL");
    const bool w_ok = fused_window_supported(blk->d.C), t_ok = fused_token_supported(blk->d.C, blk->d.mlp_ratio);
    if (enable && !w_ok && !t_ok)
        return fail(MIXAQ_E_SHAPE, "no fused kernel covers C = %d, mlp_ratio = %d", blk->d.C, blk->d.mlp_ratio);
    blk->fused_window = enable != 0 && w_ok;
    blk->fused_token = enable != 0 && t_ok;
    return MIXAQ_OK;
}

const char* mixaq_kernel_name(int32_t i)
{
    static const char* names[MIXAQ_NUM_KERNELS] = {"score", "select", "gather_ln1_quant", "qkv_gemm", "window_attention",
                                                   "proj_gemm_residual", "ln2_quant", "fc1_gemm_gelu", "fc2_gemm_residual_scatter",
                                                   "window_ln1_qkv_attention", "token_proj_ln2_ffn_scatter"};
    return (i >= 0 && i < MIXAQ_NUM_KERNELS) ? names[i] : "";
}

int mixaq_block_forward_profile(const mixaq_block* blk, const float* x, const int32_t* perm, const double* scores,
                                int32_t k_high, float* y, void* workspace, size_t workspace_bytes, void* stream,
                                int32_t repeats, float* kernel_ms)
{
    if (!kernel_ms) return fail(MIXAQ_E_NULL, "kernel_ms is NULL");
    Prof prof;
    for (int i = 0; i <= MIXAQ_NUM_KERNELS; ++i) HIP_TRY(hipEventCreate(&prof.ev[i]));
    prof.repeats = repeats < 1 ? 1 : repeats;
    int rc = forward_impl(blk, x, perm, scores, k_high, -1, y, workspace, workspace_bytes, stream, nullptr, &prof);
    if (rc == MIXAQ_OK && hipStreamSynchronize((hipStream_t)stream) != hipSuccess) rc = fail(MIXAQ_E_HIP, "stream synchronisation failed");
    for (int i = 0; i < MIXAQ_NUM_KERNELS; ++i) kernel_ms[i] = 0.0f;
    if (rc == MIXAQ_OK)
        for (int i = 0; i + 1 < prof.n; ++i) {
            float ms = 0.0f;
            if (hipEventElapsedTime(&ms, prof.ev[i], prof.ev[i + 1]) == hipSuccess) kernel_ms[prof.idx[i]] = ms / prof.repeats;
        }
    for (int i = 0; i <= MIXAQ_NUM_KERNELS; ++i) (void)hipEventDestroy(prof.ev[i]);
    return rc;
}

}  // extern "C"
