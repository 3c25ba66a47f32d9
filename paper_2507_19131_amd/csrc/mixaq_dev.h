// Device-side building blocks shared by the gfx950 kernels of the Two-Branch
// Swin Block: the pinned binary32 arithmetic that decides integer codes, the
// int8 MFMA wrappers with their lane layouts, and the row-space bookkeeping.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mixaq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int WS = 7;            // window side
constexpr int TOK = 49;          // tokens per window
constexpr int HD = 32;           // head dimension = one 32-wide MFMA block
constexpr int ROW_TILE = 64;     // rows per GEMM tile
constexpr int REGION_ALIGN = 128; // the branch regions of the row space are padded to this (the largest row tile of any kernel)
constexpr float LOG2E_F = 0x1.715476p+0f;
constexpr float MASK_VALUE = -100.0f;
constexpr float RND_MAGIC = 12582912.0f;          // 1.5 * 2^23: adding it rounds to an integer, ties to even

// One activation quantizer prepared for the device.  code = clamp(round-half-even(v*inv_s + zp)):
// u = fma(v, inv_s, MAGIC + zp) rounds the exact sum to an integer in one operation (ties to the
// even code), the clamp is taken on u, and the code is the low mantissa byte of u.
struct QDev {
    float inv_s;      // 1.0f / scale
    float magic;      // MAGIC + zp
    float lo, hi;     // MAGIC + qmin, MAGIC + qmax
    float scale;
    int   zp;
};

// returns the bit pattern of u; its low byte is the int8 code
__device__ __forceinline__ int quant_code(float v, const QDev& q)
{
    float u = fmaf(v, q.inv_s, q.magic);
    u = __builtin_amdgcn_fmed3f(u, q.lo, q.hi);
    return __float_as_int(u);
}
// the code as a sign-extended integer
__device__ __forceinline__ int code_value(int ubits) { return (int)(int8_t)(ubits & 0xff); }

// low bytes of four words -> one dword of int8 (byte k = code k)
__device__ __forceinline__ int pack4(int c0, int c1, int c2, int c3)
{
    int lo = __builtin_amdgcn_perm(c1, c0, 0x0c0c0400);
    int hi = __builtin_amdgcn_perm(c3, c2, 0x04000c0c);
    return lo | hi;
}

// Coefficients of the pinned exponential.  They travel as kernel arguments so that they sit
// in scalar registers and every Horner step is one v_fma with a scalar addend.
struct PolyCoef {
    float e[6];       // 2^r on [-1/2, 1/2], degree 5, e[0] = constant term
};

// 2^y for y <= 0 (clamped at -100): split, degree-5 polynomial, exact scaling.
__device__ __forceinline__ float exp2_pinned(float y, const PolyCoef& P)
{
    y = fmaxf(y, -100.0f);
    float n = rintf(y);
    float r = y - n;
    float p = P.e[5];
    p = fmaf(p, r, P.e[4]);
    p = fmaf(p, r, P.e[3]);
    p = fmaf(p, r, P.e[2]);
    p = fmaf(p, r, P.e[1]);
    p = fmaf(p, r, P.e[0]);
    return ldexpf(p, (int)n);
}

// GELU(x) = max(x,0) - H(|x|), H(a) = a*Phi(-a) as a piecewise cubic: interval i of width
// 2^-GELU_LOG2K on [0,6) holds the cubic in d = fract(a * 2^GELU_LOG2K); beyond the last
// interval the argument is held at its end.  The coefficient table (one float4 per interval)
// lives in LDS; replicating it per lane group to spread the banks was measured and is no faster.
//
// The kernels evaluate it on SCALED values: xs = x * 2^GELU_LOG2K goes in, GELU(x) * 2^GELU_LOG2K
// comes out, with the table's coefficients scaled by the same power of two.  A power-of-two
// factor commutes with every binary32 rounding (no overflow or underflow is near), so each
// step is exactly 2^GELU_LOG2K times the unscaled step and the codes are the same bit for bit,
// provided the caller folds the factor into what surrounds the call: the dequantization that
// produces xs uses (2^GELU_LOG2K * m, 2^GELU_LOG2K * bias), the quantizer that consumes the
// result uses inv_s / 2^GELU_LOG2K.  This saves the multiply that would form the table index.
constexpr int GELU_LOG2K = 4;
constexpr int GELU_K = 6 << GELU_LOG2K;                       // intervals on [0,6)
constexpr float GELU_SCALE = (float)(1 << GELU_LOG2K);
__device__ __forceinline__ void gelu_stage_table(float4* lds, const float4* tab, int tid, int nthreads)
{
    for (int e = tid; e < GELU_K; e += nthreads) lds[e] = tab[e];
}
__device__ __forceinline__ float gelu_scaled(float xs, const float4* lds)
{
    const float u = fminf(fabsf(xs), (float)GELU_K * 0x1.fffffep-1f);
    const float d = __builtin_amdgcn_fractf(u);
    const float4 c = lds[(int)u];
    float h = fmaf(c.w, d, c.z);
    h = fmaf(h, d, c.y);
    h = fmaf(h, d, c.x);
    return fmaxf(xs, 0.0f) - h;
}

// ---- packed sub-byte codes (tensors that cross a kernel boundary) ---------------------------------
// The attention-output codes of the LOW branch travel packed when its bit width allows: two codes per byte
// (widths 3 and 4) or four per byte (width 2), stored offset-binary (u = code + PACK_OFFSET, never negative) so
// that unpacking is a shift and a mask; the consumer removes the offset together with the zero point
// (sum_k u_k w_k - (zp + offset) * sum_k w_k).  The layout is chosen so that the producer (a lane of the window
// kernel holds, per query and head, the dims qd*8 + g*4 + e, qd = 0..3, e = 0..3, of its half g) packs without
// leaving the lane, and the consumer (a lane needs 16 consecutive channels) reads 8 contiguous bytes:
//   pack 1 (nibbles), row stride C/2, per head 16 bytes: dword p*2 + g (p = 0,1), byte e:
//       low nibble = u(dim p*16 + g*4 + e), high nibble = u(dim p*16 + 8 + g*4 + e)
//   pack 2 (two-bit fields), row stride C/4, per head 8 bytes: dword g, byte e, bits 2qd..2qd+1 = u(dim qd*8 + g*4 + e)
__host__ __device__ constexpr int pack_mode(int bits) { return bits <= 2 ? 2 : bits <= 4 ? 1 : 0; }
__host__ __device__ constexpr int pack_offset(int mode) { return mode == 2 ? 2 : mode == 1 ? 8 : 0; }

// the 16 codes (offset-binary, one per byte, in channel order) of channels 32*ks + 16*half .. +15 of one packed row
__device__ __forceinline__ v4i unpack_codes(const int8_t* packed_row, int mode, int ks, int half)
{
    if (mode == 1) {
        const int2 w = *(const int2*)(packed_row + ks * 16 + half * 8);
        return (v4i){w.x & 0x0f0f0f0f, w.y & 0x0f0f0f0f, (w.x >> 4) & 0x0f0f0f0f, (w.y >> 4) & 0x0f0f0f0f};
    }
    const int2 w = *(const int2*)(packed_row + ks * 8);
    const int s = half * 4;
    return (v4i){(w.x >> s) & 0x03030303, (w.y >> s) & 0x03030303, (w.x >> (s + 2)) & 0x03030303, (w.y >> (s + 2)) & 0x03030303};
}

// D[32x32] += A[32 x 32k] * B[32k x 32]; lane l supplies row (A) / column (B) l%32 and
// the 16 k-values of half l/32; D register r of lane l is row (r/4)*8 + (l/32)*4 + r%4,
// column l%32.
__device__ __forceinline__ v16i mfma32(v4i a, v4i b, v16i c)
{
    return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
}
// row of the 32x32 result held in register r by a lane of half g
__device__ __forceinline__ int mfma_row(int r, int g) { return (r >> 2) * 8 + g * 4 + (r & 3); }

// Geometry of one forward call.  Rows of the gathered activation matrices: the
// high group of all images first (slot = b*k_hi + j), padded to a multiple of
// REGION_ALIGN, then the low group (slot = b*k_lo + j - k_hi).
struct Geom {
    int B, H, W, C, shift, heads;
    int Hp, Wp, nWc, nW;
    int k_hi, k_lo;              // windows per image in the high / low branch (the rest is pruned)
    int n_slots;                 // B*(k_hi+k_lo) windows that are computed
    int rows_hi, rows_lo;        // valid rows per region (B*k*49)
    int base_lo;                 // first row of the low region (multiple of REGION_ALIGN)
    int rows_total;              // multiple of REGION_ALIGN
};

// row -> branch, canonical slot-major row (g*49+t) and source pixel index (or -1)
struct RowInfo { int branch; int canon; int pix; int win; };

__device__ __forceinline__ RowInfo row_info(const Geom& G, const int* __restrict__ perm, int row)
{
    RowInfo ri;
    int r = row, k = G.k_hi, jbase = 0, valid_rows = G.rows_hi;
    ri.branch = 0;
    if (row >= G.base_lo) { r = row - G.base_lo; k = G.k_lo; jbase = G.k_hi; valid_rows = G.rows_lo; ri.branch = 1; }
    if (r >= valid_rows) { ri.canon = -1; ri.pix = -1; ri.win = -1; return ri; }
    int s = r / TOK, t = r - s * TOK;
    int b = s / k, j = jbase + (s - b * k);
    int w = perm[b * G.nW + j];
    int wr = w / G.nWc, wc = w - wr * G.nWc, tr = t / WS, tc = t - tr * WS;
    int pr = wr * WS + tr + G.shift; if (pr >= G.Hp) pr -= G.Hp;
    int pc = wc * WS + tc + G.shift; if (pc >= G.Wp) pc -= G.Wp;
    ri.canon = (b * G.nW + j) * TOK + t;
    ri.win = w;
    ri.pix = (pr < G.H && pc < G.W) ? (b * G.H + pr) * G.W + pc : -1;
    return ri;
}

}  // namespace mixaq
