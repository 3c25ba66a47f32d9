/*
 * mixaq.h -- C ABI of the MI355X (gfx950) implementation of MixA-Q's
 * Two-Branch Swin Block (paper Sec. 3.2, Fig. 3).
 *
 * The block takes a feature map seen as a sequence of 7x7 activation windows,
 * scores every window by its L2 norm, sends the highest-scoring windows through
 * a high-precision branch and the rest through a low-precision branch, and
 * scatters both results back (Sec. 3.2).  The branches own their LayerNorms and
 * their activation step sizes / zero points; attention and FFN weights and
 * biases are shared "shadow layers" (Sec. 3.2).  One compression ratio is given
 * per pair of blocks, regular + shifted (Sec. 3.3); this API speaks of the keep
 * ratio = 1 - compression ratio and of k_high = windows per image in the high
 * branch.
 *
 * Conventions
 *   - Every function returns 0 (MIXAQ_OK) or a negative mixaq_status; nothing
 *     throws or aborts.  mixaq_last_error() gives the message of the calling
 *     thread's last failure.  Arguments are validated before any launch.
 *   - "device" pointers are HIP device memory owned by the caller; "host"
 *     pointers are ordinary memory.  The library allocates device memory only in
 *     mixaq_block_create (packed weights, tables) and frees it in
 *     mixaq_block_destroy.  All work is enqueued on `stream` (a hipStream_t
 *     passed as void*, NULL = default stream) without synchronising.
 *   - Feature maps are [B,H,W,C] float, channels last, unpadded.  Internally the
 *     map is zero-padded at the bottom/right to multiples of the window and, when
 *     shift > 0, rolled by -shift before partitioning and back afterwards.
 *   - x and y must not overlap.
 *   - Integer codes live in int8 containers whatever the bit width.  A b-bit
 *     quantizer is  q = clamp(rne(v * (1.0f/scale) + zp), -2^(b-1), 2^(b-1)-1):
 *     1.0f/scale is rounded to binary32 once, the product and the sum with the
 *     integer zero point are taken exactly, and the single rounding rne() goes
 *     to the nearest integer, ties to the even code.
 *   - Supported shapes: window 7, head_dim = C/heads = 32, C in {96, 128, 192,
 *     256, 384, 512, 768, 1024}, mlp_ratio in 1..8, shift in {0,..,6} (shift > 0
 *     needs padded height and width >= 14), at most 4096 windows per image.
 */
#ifndef MIXAQ_H
#define MIXAQ_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MIXAQ_OK = 0,
    MIXAQ_E_NULL = -1,        /* a required pointer is NULL */
    MIXAQ_E_SHAPE = -2,       /* unsupported or inconsistent sizes / ratios / scales */
    MIXAQ_E_BITS = -3,        /* a bit width outside 2..8 */
    MIXAQ_E_WORKSPACE = -4,   /* workspace too small or misaligned */
    MIXAQ_E_HIP = -5          /* a HIP runtime call failed */
} mixaq_status;

/* x_hat = scale * (q - zero_point): step size and zero point of one activation
 * quantizer (Sec. 3.2 keeps one set per branch). */
typedef struct { float scale; int32_t zero_point; } mixaq_qparam;

typedef struct {
    int32_t B, H, W, C;                 /* feature map [B,H,W,C]                                  */
    int32_t window, shift;              /* 7; 0 for the regular block, 3 for the shifted one       */
    int32_t heads, mlp_ratio;           /* C/heads must be 32; FFN hidden size = mlp_ratio*C       */
    int32_t act_bits_high, act_bits_low, weight_bits;   /* 2..8                                    */
    int32_t score_mode;                 /* 0: L2 norm of x, 1: L2 norm after the scoring LayerNorm */
    float   ln_eps;
} mixaq_block_desc;

/* Per-branch parameters, index 0 = high precision, 1 = low precision (Sec. 3.2:
 * duplicated LayerNorms, independent step sizes and zero points).  The bias
 * pointers of the two branches may alias (shared in QAT, independent in PTQ,
 * Sec. 4.3, PTQ setup).  All pointers: device, float.  zero_point of a_q, a_k, a_v must be 0. */
typedef struct {
    const float *ln1_gamma, *ln1_beta, *ln2_gamma, *ln2_beta;      /* [C]                 */
    const float *b_qkv, *b_proj, *b_fc1, *b_fc2;                   /* [3C],[C],[4C],[C]   */
    mixaq_qparam a_qkv_in, a_q, a_k, a_v, a_p, a_proj_in, a_fc1_in, a_fc2_in;
} mixaq_branch_params;

/* Parameters shared by the branches (shadow layers).  Weights: device int8 codes,
 * row-major [out,in], symmetric with one float scale per output channel.
 * QKV output channel n = which*C + head*32 + dim, which in {q,k,v}. */
typedef struct {
    const int8_t *w_qkv, *w_proj, *w_fc1, *w_fc2;     /* [3C,C],[C,C],[4C,C],[C,4C]            */
    const float  *s_qkv, *s_proj, *s_fc1, *s_fc2;     /* [3C],[C],[4C],[C]                      */
    const float  *rel_pos_bias;                       /* [heads,49,49], added to the logits     */
    const float  *score_gamma, *score_beta;           /* [C], used when score_mode == 1         */
} mixaq_shared_params;

/* Optional device buffers receiving every intermediate of one forward call, for
 * parity checks.  NULL members are skipped.  All are slot-major: slot
 * g = b*nW + j is position j of image b in perm; S = B*nW. */
typedef struct {
    int8_t  *a_qkv_in;    /* [S,49,C]   codes entering the QKV projection        */
    int32_t *acc_qkv;     /* [S,49,3C]  accumulators, zero-point corrected       */
    int8_t  *qkv;         /* [S,49,3C]  q,k,v codes                              */
    int32_t *acc_s;       /* [S,heads,49,49]  q.k accumulators                   */
    int8_t  *p;           /* [S,heads,49,49]  attention probability codes        */
    int32_t *acc_o;       /* [S,49,C]   p.v accumulators, zero-point corrected   */
    int8_t  *a_proj_in;   /* [S,49,C]                                            */
    int32_t *acc_proj;    /* [S,49,C]                                            */
    float   *h;           /* [S,49,C]   after the first residual                 */
    int8_t  *a_fc1_in;    /* [S,49,C]                                            */
    int32_t *acc_fc1;     /* [S,49,4C]                                           */
    int8_t  *a_fc2_in;    /* [S,49,4C]  codes after GELU                         */
    int32_t *acc_fc2;     /* [S,49,C]                                            */
    float   *y_win;       /* [S,49,C]   block output before the scatter          */
} mixaq_taps;

typedef struct mixaq_block mixaq_block;

int mixaq_version(void);
const char *mixaq_last_error(void);

/* Windows per image of the padded map. */
int mixaq_num_windows(const mixaq_block_desc *desc, int32_t *nW_per_image);
/* k_high = floor(keep_ratio*nW + 1/2) clamped to [0,nW] (Sec. 3.3: the ratio is a
 * share of the windows). */
int mixaq_keep_count(int32_t nW, double keep_ratio, int32_t *k_high);

/* Builds a block: validates, copies the quantizer and LayerNorm parameters and
 * pre-packs the weights into MFMA operand order in library-owned device memory.
 * The caller's parameter buffers may be released afterwards.  Synchronises
 * `stream` once before returning. */
int mixaq_block_create(const mixaq_block_desc *desc, const mixaq_shared_params *shared,
                       const mixaq_branch_params branch[2], void *stream, mixaq_block **out);
int mixaq_block_destroy(mixaq_block *blk);

/* Bytes of device workspace mixaq_block_forward needs (any k_high); 256-aligned. */
int mixaq_block_workspace_bytes(const mixaq_block *blk, size_t *bytes);

/* Importance scores (Sec. 3.2): squared L2 norm of every window of the
 * UN-shifted grid, over in-bounds tokens.  x: device [B,H,W,C]; scores: device
 * double [B,nW].  Computed once per stage and shared by its blocks. */
int mixaq_score_windows(const mixaq_block *blk, const float *x, double *scores, void *stream);

/* Selection (Sec. 3.2): per image, the k_high windows with the highest score
 * form the high group.  perm: device int32 [B,nW] = the windows of each image in
 * order of decreasing score (ties: lower index first); the high group is the
 * first k_high entries, the low group the rest.  reverse != 0 inverts the order
 * of importance (worst-case window selection of the robustness study, Sec. 4.1).
 * A score that is NaN counts as the least important value (in either direction), so perm is
 * always a permutation.  k_high only takes part in validation: the list is the same for every split. */
int mixaq_select_windows(const double *scores, int32_t B, int32_t nW, int32_t k_high,
                         int32_t reverse, int32_t *perm, void *stream);

/* Selection with activation pruning incorporated (Sec. 3.4): the windows with the lowest
 * scores are pruned, the others split into high and low as above.  perm is the same sorted list:
 * high group = first k_high entries, low group = next k_low, pruned group = the rest. */
int mixaq_select_windows3(const double *scores, int32_t B, int32_t nW, int32_t k_high, int32_t k_low,
                          int32_t reverse, int32_t *perm, void *stream);

/* One Two-Branch Swin Block (Fig. 3): gather + per-branch LayerNorm and
 * quantizers -> int8 windowed attention -> FFN -> residuals -> scatter.
 * perm: device [B,nW], per image the high group in its first k_high entries (any
 * order inside a group gives the same y; mixaq_select_windows produces such a
 * list), or NULL to score and select x internally.  y: device [B,H,W,C],
 * fully overwritten. */
int mixaq_block_forward(const mixaq_block *blk, const float *x, const int32_t *perm, int32_t k_high,
                        float *y, void *workspace, size_t workspace_bytes, void *stream);
/* The block with activation pruning (Sec. 3.4): positions k_high+k_low.. of every image's perm
 * row are pruned windows; their computation is skipped and y takes x there.  perm NULL scores
 * and selects internally with the same three-way split. */
int mixaq_block_forward_pruned(const mixaq_block *blk, const float *x, const int32_t *perm, int32_t k_high,
                               int32_t k_low, float *y, void *workspace, size_t workspace_bytes, void *stream);
/* The block given the SCORES instead of a selection list (scores: device double [B,nW] from
 * mixaq_score_windows, shared by the blocks of a stage): the selection of Sec. 3.2 / 3.4 is taken
 * inside the first kernel, where every window finds its own rank.  Same result as
 * mixaq_select_windows3 followed by mixaq_block_forward_pruned; k_low < 0 means no pruning
 * (k_low = nW - k_high).  perm_out (device int32 [B,nW], may be NULL) receives the selection
 * list, for the later blocks of the stage. */
int mixaq_block_forward_scored(const mixaq_block *blk, const float *x, const double *scores, int32_t k_high,
                               int32_t k_low, float *y, int32_t *perm_out, void *workspace, size_t workspace_bytes,
                               void *stream);

/* One stage (Sec. 3.2: the importance scores are computed a single time, on the stage's input,
 * and shared by all of its blocks; Sec. 3.3: blocks 2p and 2p+1 form pair p and share one
 * compression ratio).  blocks: HOST array of n_blocks handles created on the same map shape
 * [B,H,W,C] (normally alternating shift 0 / 3).  k_high, k_low: HOST arrays with one entry per
 * pair (ceil(n_blocks/2)); k_low may be NULL (no pruning).  Runs: scores on x; block 0 takes its
 * selection from the scores and leaves the full list of windows sorted by importance in perm;
 * every later block reads that list with its own pair's counts.  Pruned windows of a block carry
 * their features through that block unchanged (Sec. 3.4).  x is not modified; the result lands
 * in y; tmp is a second map-sized device buffer the blocks alternate with (x, y, tmp must not
 * overlap).  scores (device double [B,nW]) and perm (device int32 [B,nW]) are caller-owned scratch
 * that hold the stage's scores and selection list afterwards.  The workspace must satisfy
 * mixaq_block_workspace_bytes of the stage's blocks (equal shapes give equal sizes).  All work is
 * ordered on `stream`; nothing is allocated.  A batch of small maps (B >= 2, at most 4096 windows in
 * all, fused kernels) runs as two chains of blocks, one per half of the images (they are independent
 * through the whole stage): the second chain is enqueued on a stream of the library's own that
 * starts after the work already on `stream` and that `stream` waits for before the call's work
 * counts as done, so the caller sees the same ordering as without it; under stream capture the
 * stage stays on `stream` alone.  MIXAQ_E_SHAPE if the blocks disagree on the shape or a count is
 * out of range, MIXAQ_E_NULL for missing pointers. */
int mixaq_stage_forward(mixaq_block *const *blocks, int32_t n_blocks, const float *x, const int32_t *k_high,
                        const int32_t *k_low, float *y, float *tmp, double *scores, int32_t *perm, void *workspace,
                        size_t workspace_bytes, void *stream);
/* Same as mixaq_block_forward, and also fills the given taps. */
int mixaq_block_forward_taps(const mixaq_block *blk, const float *x, const int32_t *perm, int32_t k_high,
                             float *y, void *workspace, size_t workspace_bytes, void *stream,
                             const mixaq_taps *taps);

/* For callers that cannot allocate device memory or bring a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same computation and same bits as
 * mixaq_block_forward, with the scratch the two fused kernels exchange (scores, selection list, row
 * bookkeeping, attention-output codes) held in a static device array of MIXAQ_STATIC_SCRATCH_BYTES
 * inside the library: one copy per GPU, kept until the process ends.  The call allocates nothing and
 * frees nothing; on its first use on a device it asks the runtime for the array's address there
 * (the device must be current, as for every call).  Only blocks that run the fused kernels
 * (C <= 384, mlp_ratio 4, not switched off by mixaq_block_set_fused: MIXAQ_E_SHAPE otherwise) and
 * whose scratch fits: about B*nW*49*(C + 8) bytes, e.g. 7.1 MB for the 1392-window stage-1 map at
 * C = 96; MIXAQ_E_WORKSPACE with the two sizes in the message otherwise.  Every call on a GPU uses
 * that GPU's one array, which keeps the last call's contents (nothing in it needs clearing: every
 * call rewrites what it reads): calls that overlap in time on one GPU, on any streams, race. */
#define MIXAQ_STATIC_SCRATCH_BYTES (16u << 20)
int mixaq_block_forward_static(const mixaq_block *blk, const float *x, const int32_t *perm, int32_t k_high,
                               float *y, void *stream);

/* ---- layers between stages ---------------------------------------------------------------- */

/* Patch embedding and patch merging of the Swin backbone the blocks sit in.  The paper keeps them
 * outside MixA-Q (appendix on equivalent activation bits: the constant term of the cost model, the
 * layers whose computation the method cannot save); they are offered so that the stages of a
 * backbone can run as one chain.  Each is ONE uniformly quantized linear layer with the block's
 * arithmetic (codes in int8 containers, int32 sums, f = fma(f32(acc - z*colsum), a_in.scale*s_w[n],
 * bias[n])):
 *   kind 0, patch embedding: token (i,j) takes the patch x patch x C_in values of its patch in the
 *     order (row in patch, column in patch, channel), zero outside the image; quantize; linear
 *     with bias; LayerNorm over the N outputs (ln_gamma, ln_beta: [N]).
 *   kind 1, patch merging: the 2x2 neighbours with (row, column) offsets (0,0), (1,0), (0,1), (1,1)
 *     concatenated along the channels (K = 4*C_in), zero outside the map; LayerNorm over the K
 *     values (ln_gamma, ln_beta: [K]); quantize; linear (bias may be NULL).
 * x: device float [B,H,W,C_in]; y: device float [B,Ho,Wo,N], Ho = ceil(H/P), Wo = ceil(W/P), P =
 * patch (kind 0) or 2 (kind 1).  w: device int8 [N][K] codes, s_w: device float [N].  N must be a
 * multiple of 32, K a multiple of 4 (kind 1: C_in a multiple of 4). */
typedef struct {
    int32_t kind;                    /* 0 = patch embedding, 1 = patch merging                   */
    int32_t B, H, W, C_in;           /* input image / map                                        */
    int32_t patch;                   /* kind 0: patch side (4); ignored for kind 1               */
    int32_t N;                       /* output channels                                          */
    int32_t act_bits, weight_bits;   /* 2..8                                                     */
    float   ln_eps;
} mixaq_downsample_desc;
typedef struct {
    const int8_t *w;
    const float  *s_w;
    const float  *bias;              /* [N] or NULL                                              */
    const float  *ln_gamma, *ln_beta;
    mixaq_qparam  a_in;              /* quantizer of the linear layer's input                    */
} mixaq_downsample_params;
typedef struct mixaq_downsample mixaq_downsample;

/* Output map size and inputs per token of a descriptor (host only). */
int mixaq_downsample_out_shape(const mixaq_downsample_desc *desc, int32_t *Ho, int32_t *Wo, int32_t *K);
/* Copies and pre-packs the parameters into library-owned device memory (synchronous copies).
 * MIXAQ_E_SHAPE / MIXAQ_E_BITS / MIXAQ_E_NULL on a bad descriptor or parameters. */
int mixaq_downsample_create(const mixaq_downsample_desc *desc, const mixaq_downsample_params *params,
                            mixaq_downsample **out);
int mixaq_downsample_destroy(mixaq_downsample *h);
/* One kernel on `stream`; allocates nothing; x and y must not overlap. */
int mixaq_downsample_forward(const mixaq_downsample *h, const float *x, float *y, void *stream);
/* The same, also writing the input codes (device int8 [tokens][K]) and the zero-point corrected
 * int32 sums (device int32 [tokens][N]) for parity checks; either may be NULL. */
int mixaq_downsample_forward_taps(const mixaq_downsample *h, const float *x, float *y, void *stream,
                                  int8_t *tap_codes, int32_t *tap_acc);

/* ---- host-only helpers (no GPU work) ------------------------------------------------------- */

/* Equivalent activation bits (appendix "Calculation of Equivalent Activation Bits"):
 *   act_bits_eq = act_bits_base * (sum_i f_i*gmacs[i] + c_gmacs) / (sum_i gmacs[i] + c_gmacs),
 * f_i = 1 - compress_ratio[i]/2 for MixA-Q (a low-bit window costs half).  prune_ratio (may be
 * NULL) adds activation pruning, f_i = 1 - prune_ratio[i] - compress_ratio[i]/2 (a pruned window
 * costs nothing; ratios are fractions of ALL windows); compress_ratio = 0 with a prune ratio gives
 * the pure-pruning formula f_i = 1 - r.  gmacs: GMACs per pair of blocks, c_gmacs: the layers
 * the method cannot save.  All pointers host. */
int mixaq_equivalent_act_bits(int32_t n_pairs, const double *gmacs, double c_gmacs, const double *compress_ratio,
                              const double *prune_ratio, double act_bits_base, double *act_bits_eq);
/* Bit operations in units of 1e12: GMACs * act_bits * other_operand_bits (the paper's tables hold
 * the other operand at 32, Sec. 4.1). */
int mixaq_bops_tera(double total_gmacs, double act_bits, double other_operand_bits, double *bops_tera);

/* Uniform-sum compression-ratio sampling (Algorithm 1): a target sum S (in tenths) uniform on
 * [10*s_min, 10*s_max], ratios from a flat Dirichlet scaled to S, re-drawn until none exceeds
 * `upper`, rounded to tenths with the largest-remainder method so that they still sum to S/10.
 * The random numbers come from the caller: uniforms[] in (0,1); one is used for S and n per
 * Dirichlet draw (exponential spacings).  n_used (may be NULL) receives how many were consumed;
 * MIXAQ_E_WORKSPACE if they run out.  ratios: host [n]. */
int mixaq_sample_ratios(int32_t n, double s_min, double s_max, double upper, const double *uniforms, size_t n_uniforms,
                        size_t *n_used, double *ratios);

/* Chooses between the two implementations of the forward call: the fused kernels (a window
 * kernel for gather/LN1/QKV/attention, a token kernel per 32- or 64-row tile for
 * proj/LN2/FFN/scatter: C <= 384, the token kernel with mlp_ratio 4; each is the default where it
 * is supported) and the seven-kernel path that handles every supported shape.  Both give the
 * same bits.  enable = 0 selects the seven-kernel path; enabling on a shape no fused kernel
 * covers returns MIXAQ_E_SHAPE. */
int mixaq_block_set_fused(mixaq_block *blk, int32_t enable);

/* Measurement aid for benchmarks (not part of the paper's method): one forward
 * call in which every kernel is launched `repeats` times in a row (each launch
 * recomputes the same result) between two HIP events on `stream`; synchronises
 * the stream and writes the mean duration of each kernel in milliseconds to the
 * HOST array kernel_ms[MIXAQ_NUM_KERNELS] (0 for kernels that did not run, e.g.
 * score and select when perm is given).  perm / scores as in mixaq_block_forward /
 * mixaq_block_forward_scored (at most one non-NULL).  mixaq_kernel_name(i) names entry i. */
#define MIXAQ_NUM_KERNELS 11
int mixaq_block_forward_profile(const mixaq_block *blk, const float *x, const int32_t *perm, const double *scores,
                                int32_t k_high, float *y, void *workspace, size_t workspace_bytes, void *stream,
                                int32_t repeats, float *kernel_ms);
const char *mixaq_kernel_name(int32_t i);

#ifdef __cplusplus
}
#endif
#endif
