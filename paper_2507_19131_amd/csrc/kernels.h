// Argument blocks and launchers of the gfx950 kernels (host side sees only this).
#pragma once
#include "mixaq_dev.h"

namespace mixaq {

enum { EPI_QKV = 0, EPI_PROJ = 1, EPI_FC1 = 2, EPI_FC2 = 3 };

// the pinned coefficients of 2^r (host side fills kernel arguments with them)
inline PolyCoef pinned_coefficients()
{
    PolyCoef P = {{0x1.000002p+0f, 0x1.62e430p-1f, 0x1.ebf906p-3f, 0x1.c6aeccp-5f, 0x1.3d107cp-7f, 0x1.5f48c8p-10f}};
    return P;
}

// Host side: the GELU_K x 4 coefficient table of gelu_pinned (api.hip uploads it once per block).
void gelu_table(float* tab);

struct LnArgs {
    const int* perm;                 // [B,nW] (gather only)
    const float* src;                // feature map (gather) or h rows [rows,C]
    const float* gamma[2];
    const float* beta[2];
    QDev q[2];
    float eps;
    int8_t* out;                     // [rows,C]
    int* row_pix;                    // [rows] written by the gather, read otherwise
    int* row_canon;                  // [rows]
    int8_t* tap;                     // slot-major copy or NULL
};

struct GemmArgs {
    const int8_t* A;                 // activations [rows,K] row-major
    const v4i* Wp;                   // packed weights [N/32][K/32][64 lanes] x 16 bytes
    int K, N, nb_per_block;
    int kchunk;                      // bytes of K staged in LDS at a time (a divisor of K; set by the launcher)
    const float* m[2];               // s_in * s_w[n] per branch
    const float* bias[2];
    const int* negcorr[2];           // -zp_in * sum_k W[n,k]
    QDev q[2][3];                    // output quantizers (QKV: q,k,v; FC1: [0])
    int8_t* out8;                    // [rows,N] codes (QKV, FC1)
    float* outf;                     // [rows,N] (proj)
    const float* resid;              // [rows,N] (FC2)
    const float* x;                  // feature map, shortcut of the first residual (proj)
    float* y;                        // output map (FC2 scatter)
    const int* row_pix;
    const int* row_canon;
    int32_t* tap_acc;
    int8_t* tap_code;
    float* tap_f;
    const float4* gelu_tab;          // [GELU_K] cubic coefficients (FC1 epilogue)
};

struct AttnArgs {
    const int8_t* qkv;               // [rows,3C]
    const int* perm;
    const float* bias2;              // [4 mask types][heads][49 keys][64 queries], (bias+mask)*log2e
    float m2[2];                     // s_q*s_k/sqrt(d)*log2e
    float m_o[2];                    // s_p*s_v
    QDev qp[2], qo[2];
    int8_t* out;                     // [rows,C]
    int32_t* tap_s;
    int8_t* tap_p;
    int32_t* tap_o;
    int8_t* tap_code;
    PolyCoef poly;
};

struct WinArgs {                     // fused window kernel (gather + LN1 + QKV + attention)
    const float* x;
    const int* perm;                 // selection list, or ...
    const double* scores;            // ... the scores: every workgroup ranks its own window ([B,nW]; NULL = use perm)
    int* perm_out;                   // with scores: receives the selection list
    float* y;                        // with scores: pruned windows are forwarded here
    // per branch one block of 32-bit words, staged in LDS by every workgroup:
    // [LN1 gamma | LN1 beta] (C words each), then [qkv m | qkv bias | qkv negcorr] (3C words each; negcorr integers)
    const float* params[2];
    float eps;
    QDev q_in[2];
    const v4i* Wqkv;                 // packed, natural k order
    QDev q_qkv[2][3];
    const float* bias2;
    float m2[2], m_o[2];
    QDev qp[2], qo[2];
    int8_t* out;                     // attention output codes [rows,C]
    int out_pack;                    // 0: int8 containers; 1, 2: the low region's rows packed (see unpack_codes)
    int* row_pix;
    int* row_canon;
    int8_t* tap_a1; int32_t* tap_acc; int8_t* tap_qkv; int32_t* tap_s; int8_t* tap_p; int32_t* tap_o; int8_t* tap_code;
    PolyCoef poly;
    bool taps;                       // any tap pointer set
};

struct TokArgs {                     // fused token kernel (proj + LN2 + FFN + scatter)
    const int8_t* ao;                // [rows,C]
    int ao_pack;                     // as WinArgs::out_pack
    const float* x;
    float* y;
    const int* row_pix;
    const int* row_canon;
    const v4i* Wproj;                // natural k order
    const v4i* W1;                   // k order of the MFMA result registers
    const v4i* W2;
    // per branch one block of 32-bit words, staged in LDS by every workgroup:
    // [proj m | proj bias | proj negcorr | LN2 gamma | LN2 beta | fc2 m | fc2 bias | fc2 negcorr] (C words each),
    // then [fc1 m | fc1 bias | fc1 negcorr] (4C words each); negcorr words are integers
    const float* params[2];
    float eps;
    QDev q_fc1in[2], q_fc2in[2];
    int32_t* tap_acc_proj; float* tap_h; int8_t* tap_a2; int32_t* tap_acc_fc1; int8_t* tap_g; int32_t* tap_acc_fc2; float* tap_y;
    const float4* gelu_tab;          // [GELU_K] cubic coefficients
    bool taps;
};

bool channels_supported(int C);
bool fused_window_supported(int C);
bool fused_token_supported(int C, int mlp_ratio);
void launch_window(const Geom& G, const WinArgs& A, hipStream_t st);
void launch_token(const Geom& G, const TokArgs& A, hipStream_t st);
bool launch_score(const Geom& G, const float* x, int mode, float eps, const float* gm, const float* bt, double* scores,
                  hipStream_t st);
void launch_select(const double* scores, int B, int nW, int reverse, int* perm, hipStream_t st);
void launch_bypass(const Geom& G, const int* perm, const float* x, float* y, hipStream_t st);
bool launch_ln_quant(const Geom& G, const LnArgs& A, bool gather, hipStream_t st);
void launch_gemm(const Geom& G, const GemmArgs& A, int epi, hipStream_t st);
void launch_attn(const Geom& G, const AttnArgs& A, hipStream_t st);

}  // namespace mixaq
