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
constexpr int ROW_TILE = 64;     // rows per GEMM tile; branch regions are padded to this
constexpr float LOG2E_F = 0x1.715476p+0f;
constexpr float MASK_VALUE = -100.0f;
constexpr float RND_MAGIC = 12582912.0f;          // 1.5 * 2^23: adding it rounds to an integer, ties to even
constexpr int RND_MAGIC_BITS = 0x4B400000;

// One activation quantizer prepared for the device.  code = clamp(rne(v*inv_s) + zp):
// u = fma(v, inv_s, MAGIC) rounds the exact product half-to-even, the clamp is taken
// on u, and the integer is the low mantissa of u.
struct QDev {
    float inv_s;      // 1.0f / scale
    float lo, hi;     // MAGIC + (qmin - zp), MAGIC + (qmax - zp)
    int   off;        // zp - RND_MAGIC_BITS
    float scale;
    int   zp;
};

__device__ __forceinline__ int quant_code(float v, const QDev& q)
{
    float u = fmaf(v, q.inv_s, RND_MAGIC);
    u = __builtin_amdgcn_fmed3f(u, q.lo, q.hi);
    return __float_as_int(u) + q.off;
}

// four int codes -> one dword of int8 (byte k = code k)
__device__ __forceinline__ int pack4(int c0, int c1, int c2, int c3)
{
    int lo = __builtin_amdgcn_perm(c1, c0, 0x0c0c0400);
    int hi = __builtin_amdgcn_perm(c3, c2, 0x04000c0c);
    return lo | hi;
}

// 2^y for y <= 0 (clamped at -100): split, degree-5 polynomial, exact scaling.
__device__ __forceinline__ float exp2_pinned(float y)
{
    y = fmaxf(y, -100.0f);
    float n = rintf(y);
    float r = y - n;
    float p = 0x1.5f48c8p-10f;
    p = fmaf(p, r, 0x1.3d107cp-7f);
    p = fmaf(p, r, 0x1.c6aeccp-5f);
    p = fmaf(p, r, 0x1.ebf906p-3f);
    p = fmaf(p, r, 0x1.62e430p-1f);
    p = fmaf(p, r, 0x1.000002p+0f);
    return ldexpf(p, (int)n);
}

// GELU(x) = max(x,0) - a*Phi(-a), a = |x|; the remainder is a degree-14 polynomial
// in t = 2a/5.5 - 1 for a <= 5.5 and constant beyond.
__device__ __forceinline__ float gelu_pinned(float x)
{
    float a = fminf(fabsf(x), 5.5f);
    float t = fmaf(a, 0x1.745d18p-2f, -1.0f);
    float h = 0x1.280820p-5f;
    h = fmaf(h, t, -0x1.42e9b8p-5f);
    h = fmaf(h, t, -0x1.3d2fc0p-3f);
    h = fmaf(h, t, 0x1.e1f934p-3f);
    h = fmaf(h, t, 0x1.7cae60p-3f);
    h = fmaf(h, t, -0x1.18547cp-1f);
    h = fmaf(h, t, 0x1.88e9f6p-3f);
    h = fmaf(h, t, 0x1.d7ab76p-2f);
    h = fmaf(h, t, -0x1.46f9bap-1f);
    h = fmaf(h, t, 0x1.0a7892p-2f);
    h = fmaf(h, t, 0x1.711f2ap-3f);
    h = fmaf(h, t, -0x1.3c122ap-2f);
    h = fmaf(h, t, 0x1.8794f2p-3f);
    h = fmaf(h, t, -0x1.f0423cp-5f);
    h = fmaf(h, t, 0x1.0c8760p-7f);
    return fmaxf(x, 0.0f) - h;
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
// ROW_TILE, then the low group (slot = b*k_lo + j - k_hi).
struct Geom {
    int B, H, W, C, shift, heads;
    int Hp, Wp, nWc, nW;
    int k_hi, k_lo;
    int rows_hi, rows_lo;        // valid rows per region (B*k*49)
    int base_lo;                 // first row of the low region (multiple of ROW_TILE)
    int rows_total;              // multiple of ROW_TILE
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
