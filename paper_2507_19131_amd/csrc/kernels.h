// Argument blocks and launchers of the gfx950 kernels (host side sees only this).
#pragma once
#include "mixaq_dev.h"

namespace mixaq {

enum { EPI_QKV = 0, EPI_PROJ = 1, EPI_FC1 = 2, EPI_FC2 = 3 };

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
};

bool channels_supported(int C);
bool launch_score(const Geom& G, const float* x, int mode, float eps, const float* gm, const float* bt, double* scores,
                  hipStream_t st);
void launch_select(const double* scores, int B, int nW, int k_hi, int reverse, int* perm, hipStream_t st);
bool launch_ln_quant(const Geom& G, const LnArgs& A, bool gather, hipStream_t st);
void launch_gemm(const Geom& G, const GemmArgs& A, int epi, hipStream_t st);
void launch_attn(const Geom& G, const AttnArgs& A, hipStream_t st);

}  // namespace mixaq
