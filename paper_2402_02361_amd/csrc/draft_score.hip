// Draft model: Symbol-based Analyzer over a population of candidate schedules (Alg. 2, C_SA and the loop over S_x).
//
// One thread scores VEC neighbouring candidates.  Tile factors arrive structure-of-arrays (one uint16 row per
// split level), so a wavefront reads 64*VEC consecutive uint16 of every row; everything else stays in registers.
// Per-subgraph constants (device abstraction, loop-nest class, division magics) sit in a small table that all
// lanes of a block read through the scalar cache; a block never straddles two subgraphs.
//
// Arithmetic contract (this file is compiled with -ffp-contract=off and correctly rounded division):
//   symbols are exact integers (Table 2);
//   penalties, utilisation and latency (Sec. 4.1 "Hardware-aware Penalty", Eq. 1) are binary32, in one of two forms.
//   analyze_fused(): the penalties of a statement group, all of them ratios, multiplied out and divided once (within
//   2^-20 relative of Eq. 1's value); used by the per-class launches of populations of 2^20 candidates and more, or
//   everywhere under PRUNER_FUSED_ARITHMETIC.  analyze(): one IEEE operation per step (used by single-launch calls, or
//   everywhere under PRUNER_REFERENCE_ROUNDING), in this order:
//     P0m = min(m_l0 / S1, 1)          P0c = 1 + S2 / S1            P1m = min(m_l1 / S3, 1)
//     sch = ceil(S4 / n_l1)            P1c = sch / (ceil(sch / pu_l1) * pu_l1)
//     alpha = S4 / (sch * n_l1)        P2c = S6 / (ceil(S6 / pu_l2) * pu_l2)
//     Up  = (((T_p * P0c) * P1c) * alpha) * P2c   [ * Ptc in fragment mode ]
//     L   = S8 / Up
//     for each memory statement In_0, In_1, store:
//         P2m = S7 / (ceil(S7 / n_l2) * n_l2);  Um = ((T_m * P0m) * P1m) * P2m;  L = L + S5 / Um
//     score = -L
//   integer-to-float conversions round to nearest even.  Quotients are correctly rounded (see div_rn).
#include "lse_child.h"
#include "select_common.h"

#include <string.h>

#include <algorithm>
#include <vector>

namespace pruner {
namespace {

constexpr int kBlock = 256;

enum NestClass : int32_t { kGeneric = 0, kGemm = 1, kBatchedGemm = 2, kConv2d = 3, kDepthwiseConv2d = 4 };

// Unsigned division by a run-time constant.  Powers of two (warp size, schedulers, transaction length and
// fragment size nearly always are) shift; other divisors use one multiply-high (Granlund & Montgomery,
// "Division by invariant integers using multiplication", PLDI 1994, Fig. 4.1): for 2 <= d < 2^31,
// L = ceil(log2 d), m = floor(2^32 (2^L - d) / d) + 1, sh = L - 1:
//   floor(x / d) = (((x - mulhi(m, x)) >> 1) + mulhi(m, x)) >> sh      for every 32-bit x.
// The divisor is the same for all lanes, so the choice is a scalar branch.
struct UDiv {
    uint32_t d, m, sh, pow2;  // pow2: d = 2^sh (then m is unused); d = 1 is 2^0
};

UDiv make_udiv(uint32_t d)
{
    UDiv u{d, 0, 0, 0};
    uint32_t L = 0;
    while ((1ull << L) < d) ++L;
    if ((1ull << L) == d) {
        u.pow2 = 1;
        u.sh = L;
    } else {
        u.m = (uint32_t)((((1ull << L) - d) << 32) / d + 1);
        u.sh = L - 1;
    }
    return u;
}

__device__ __forceinline__ uint32_t cdiv(uint32_t x, const UDiv& u)
{
    const uint32_t y = x + u.d - 1;
    if (u.pow2) return y >> u.sh;
    const uint32_t q = __umulhi(u.m, y);
    return (((y - q) >> 1) + q) >> u.sh;
}

// Correctly rounded binary32 quotient for operands whose quotient and residuals stay well inside the normal
// range (here: counts below 2^53 against peaks and products between 2^-100 and 2^100; checked on the host).
// This is the Newton-Raphson / fused-residual sequence that compilers emit for IEEE division (reciprocal
// estimate, one refinement of the reciprocal, two corrections of the quotient with exact fma residuals, cf.
// Markstein, "IA-64 and Elementary Functions", ch. 8) without the exponent pre-scaling and special-value fix-up,
// which only matter outside that range.  recip() exposes the refined reciprocal so that two quotients with the
// same divisor share it.
__device__ __forceinline__ float recip(float b)
{
    const float y0 = __builtin_amdgcn_rcpf(b);
    const float e = __builtin_fmaf(-b, y0, 1.0f);
    return __builtin_fmaf(e, y0, y0);
}
__device__ __forceinline__ float div_by(float a, float b, float y)  // a / b with y = recip(b)
{
    const float q0 = a * y;
    const float r0 = __builtin_fmaf(-b, q0, a);
    const float q1 = __builtin_fmaf(r0, y, q0);
    const float r1 = __builtin_fmaf(-b, q1, a);
    return __builtin_fmaf(r1, y, q1);
}
__device__ __forceinline__ float div_rn(float a, float b) { return div_by(a, b, recip(b)); }

// Per-subgraph constants, read by all lanes of a block at the same address.
struct alignas(16) SgDesc {
    int32_t cls, n_sp, n_rd, rd_levels;
    int32_t n_in, frag_mode;
    uint32_t dtype_bytes, n_l1;
    float T_p, T_m, m_l0f, m_l1f;
    float S8f, S5out_f;
    int32_t stride_h, stride_w;  // conv classes: coefficient of the output row / column in the image index
    int64_t S8, S5out;
    double cA, cB;       // GEMM classes: bytes * elements of In_0 / In_1
    double bytes_f64;    // dtype_bytes as binary64
    int32_t run_max;     // upper bound of S7 over the three memory statements
    int32_t f32_s2;      // prod R and prod q stay below 2^24: S2 may be formed in binary32
    int32_t f32_traffic; // GEMM classes: f32_s2, and cA, cB are binary32 numbers: S5 may be formed in binary32
    int32_t f32_frag;    // the fragment products (two inner spatial tiles, rounded up; inner reduction tile) are exact
    float cAf, cBf;
    int32_t small;       // every operand of an integer multiply in the symbol code stays below 2^24
    float k_c;           // S8 / T_p: the compute statement's latency before penalties       } constants of the
    float inv_m0, inv_m1, inv_Tm;  // 1 / m_l0, 1 / m_l1, 1 / T_m                          } fused evaluation
    float lanes_f;       // lanes one scheduling unit stands for: n_l1, or 1 in fragment mode
    UDiv div_n_l1, div_pu_l1, div_pu_l2, div_n_l2, div_frag[3];
    // generic class only: access tables of in0, in1, out
    int32_t ndim[3];
    int32_t pad0;
    int8_t axis[3][PRUNER_MAX_DIMS][PRUNER_MAX_TERMS];
    int32_t coef[3][PRUNER_MAX_DIMS][PRUNER_MAX_TERMS];
};

struct alignas(8) SegEnt {
    int64_t begin, end;
    int32_t first_block, desc;
    int32_t blocks;    // workgroups that share the segment; workgroup j takes chunks j, j + blocks, j + 2 blocks, ...
    int32_t iters;     // chunks of kBlock * VEC candidates each of them walks through (the last may fall off the end)
    int32_t use_tab;   // the block tabulates P_l2,m over the possible run lengths first
    int32_t seg;       // the segment's place in the caller's order
};

constexpr int kTabMax = 4096;   // longest run length the P_l2,m table covers
constexpr int64_t kPerClassMin = 1 << 20;   // candidates from which a call launches one kernel per loop-nest class

// ---- symbols (Table 2) ---------------------------------------------------------------------------------------------

// Tile sizes of one candidate.  Spatial axis a: G grid, T threads, R = V*I thread tile, B = R*T block tile, In the
// inner factor.  Reduction axis r: O outer steps, D shared-tile depth, q register step.
template <int NSP, int NRD> struct Tiling {
    uint32_t G[NSP], V[NSP], T[NSP], R[NSP], B[NSP], In[NSP];
    uint32_t O[NRD > 0 ? NRD : 1], Mid[NRD > 0 ? NRD : 1], D[NRD > 0 ? NRD : 1], q[NRD > 0 ? NRD : 1];
};

struct Symbols {
    uint32_t S1;      // L0MemAlloc before the per-lane split of fragment mode
    uint32_t S3, S6;
    uint32_t prod_T;  // L1ParaInfo is prod_T, or n_l1 * prod_T in fragment mode
    double S2;        // exact: can pass 2^32            } only the symbol dump reads the binary64 values;
    double S5[2];     // exact: products below 2^53      } the scores use the binary32 roundings below
    float S3f, S6f;      // S3, S6 as binary32 (rounded to nearest even where they pass 2^24)
    float S2f, S5f[2];   // S2, S5 rounded to nearest even.  A binary32 product of two exactly represented integers
                         // IS that rounding of the exact product, so where both factors are exact (checked on the
                         // host, d.f32_*) one v_mul_f32 replaces the binary64 detour.
    uint32_t S7[3];
};

// 32-bit integer multiplies run at a quarter of the rate of 24-bit ones on this part.  Tile factors are uint16 and
// the factors of an axis multiply to its extent (< 2^16), so products of two per-axis quantities always qualify;
// SMALL says that the host has bounded every other operand below 2^24 as well (d.small).
__device__ __forceinline__ uint32_t mul24(uint32_t a, uint32_t b) { return __umul24(a, b); }
template <bool SMALL> __device__ __forceinline__ uint32_t mul(uint32_t a, uint32_t b) { return SMALL ? __umul24(a, b) : a * b; }

// Loop-nest classes.  Every symbol is an exact integer, so a class may use any algebraically equal form of the
// definitions (S1 = prod R + sum of operand register tiles, S3 = bytes of the operand block tiles,
// S5 = bytes * blocks * outer steps * block tile, S7 = innermost run of the block tile); equality of the closed
// forms relies on the factors of an axis multiplying to its extent, which the boundary requires.
// cA, cB: bytes * (elements of In_0 / In_1) as binary64.

struct NestGemm {  // C[i,j] += A[i,k] B[k,j]; axes i j | k
    static constexpr int NSP = 2, NRD = 1;
    static constexpr bool FIXED = true;
    template <bool DUMP, bool SMALL> __device__ static void symbols(const SgDesc& d, const Tiling<2, 1>& t, Symbols& y);
};
struct NestBatchedGemm {  // C[b,i,j] += A[b,i,k] B[b,k,j]; axes b i j | k
    static constexpr int NSP = 3, NRD = 1;
    static constexpr bool FIXED = true;
    template <bool DUMP, bool SMALL> __device__ static void symbols(const SgDesc& d, const Tiling<3, 1>& t, Symbols& y);
};
struct NestConv2d {  // O[n,k,h,w] += I[n,c,h*sh+r,w*sw+s] W[k,c,r,s]; axes n k h w | c r s
    static constexpr int NSP = 4, NRD = 3;
    static constexpr bool FIXED = true;
    template <bool DUMP, bool SMALL> __device__ static void symbols(const SgDesc& d, const Tiling<4, 3>& t, Symbols& y);
};
struct NestDepthwiseConv2d {  // O[n,c,h,w] += I[n,c,h*sh+r,w*sw+s] W[c,r,s]; axes n c h w | r s
    static constexpr int NSP = 4, NRD = 2;
    static constexpr bool FIXED = true;
    template <bool DUMP, bool SMALL> __device__ static void symbols(const SgDesc& d, const Tiling<4, 2>& t, Symbols& y);
};
struct NestGeneric {  // any affine nest, from the access tables; absent axes carry factors of 1 and drop out
    static constexpr int NSP = PRUNER_MAX_SP, NRD = PRUNER_MAX_RD;
    static constexpr bool FIXED = false;
    template <bool DUMP, bool SMALL> __device__ static void symbols(const SgDesc& d, const Tiling<4, 3>& t, Symbols& y);
};

template <bool DUMP, bool SMALL> __device__ __forceinline__ void NestGemm::symbols(const SgDesc& d, const Tiling<2, 1>& t, Symbols& y)
{
    // every operand below is a per-axis quantity (< 2^16), a sum of two, or dtype_bytes times such a sum (< 2^21)
    const uint32_t RR = mul24(t.R[0], t.R[1]);
    y.S1 = RR + mul24(t.q[0], t.R[0] + t.R[1]);                   // accumulators + a column of A + a row of B
    y.S3 = mul24(t.D[0], mul24(d.dtype_bytes, t.B[0] + t.B[1]));
    y.prod_T = mul24(t.T[0], t.T[1]);
    y.S6 = mul24(t.G[0], t.G[1]);
    if (DUMP || !d.f32_traffic) {
        y.S2 = 2.0 * ((double)RR * (double)t.q[0]);
        y.S5[0] = d.cA * (double)t.G[1];                          // A is read once per column of blocks
        y.S5[1] = d.cB * (double)t.G[0];                          // B once per row of blocks
    }
    if (d.f32_traffic) {
        y.S2f = 2.0f * ((float)RR * (float)t.q[0]);
        y.S5f[0] = d.cAf * (float)t.G[1];
        y.S5f[1] = d.cBf * (float)t.G[0];
    } else {
        y.S2f = (float)y.S2;
        y.S5f[0] = (float)y.S5[0];
        y.S5f[1] = (float)y.S5[1];
    }
    y.S3f = (float)y.S3;
    y.S6f = (float)y.S6;
    y.S7[0] = t.D[0];
    y.S7[1] = t.B[1];
    y.S7[2] = t.B[1];
}

template <bool DUMP, bool SMALL> __device__ __forceinline__ void NestBatchedGemm::symbols(const SgDesc& d, const Tiling<3, 1>& t, Symbols& y)
{
    const uint32_t RR = mul24(t.R[1], t.R[2]);
    const uint32_t RRR = mul<SMALL>(t.R[0], RR);
    y.S1 = mul<SMALL>(t.R[0], RR + mul24(t.q[0], t.R[1] + t.R[2]));
    y.S3 = mul<SMALL>(mul24(t.B[0], t.D[0]), mul24(d.dtype_bytes, t.B[1] + t.B[2]));
    y.prod_T = mul<SMALL>(mul24(t.T[0], t.T[1]), t.T[2]);
    y.S6 = mul<SMALL>(mul24(t.G[0], t.G[1]), t.G[2]);
    if (DUMP || !d.f32_traffic) {
        y.S2 = 2.0 * ((double)RRR * (double)t.q[0]);
        y.S5[0] = d.cA * (double)t.G[2];
        y.S5[1] = d.cB * (double)t.G[1];
    }
    if (d.f32_traffic) {
        y.S2f = 2.0f * ((float)RRR * (float)t.q[0]);
        y.S5f[0] = d.cAf * (float)t.G[2];
        y.S5f[1] = d.cBf * (float)t.G[1];
    } else {
        y.S2f = (float)y.S2;
        y.S5f[0] = (float)y.S5[0];
        y.S5f[1] = (float)y.S5[1];
    }
    y.S7[0] = t.D[0];
    y.S7[1] = t.B[2];
    y.S7[2] = t.B[2];
    y.S3f = (float)y.S3;
    y.S6f = (float)y.S6;
}

template <bool DUMP, bool SMALL> __device__ __forceinline__ void NestConv2d::symbols(const SgDesc& d, const Tiling<4, 3>& t, Symbols& y)
{
    const uint32_t sh = (uint32_t)d.stride_h, sw = (uint32_t)d.stride_w;   // < 2^16
    const uint32_t rows_b = mul24(t.B[2] - 1, sh) + t.D[1], cols_b = mul24(t.B[3] - 1, sw) + t.D[2];
    const uint32_t rows_r = mul24(t.R[2] - 1, sh) + t.q[1], cols_r = mul24(t.R[3] - 1, sw) + t.q[2];
    const uint32_t img_b = mul<SMALL>(mul<SMALL>(t.B[0], rows_b), cols_b);                   // per input channel
    const uint32_t wgt_b = mul<SMALL>(mul24(t.B[1], t.D[1]), t.D[2]);
    const uint32_t prod_R = mul<SMALL>(mul24(t.R[0], t.R[1]), mul24(t.R[2], t.R[3]));
    const uint32_t prod_q = mul<SMALL>(mul24(t.q[0], t.q[1]), t.q[2]);
    y.S1 = prod_R + mul<SMALL>(t.q[0], mul<SMALL>(mul<SMALL>(t.R[0], rows_r), cols_r) + mul<SMALL>(mul24(t.R[1], t.q[1]), t.q[2]));
    y.S2 = 2.0 * ((double)prod_R * (double)prod_q);
    y.S3 = mul<SMALL>(d.dtype_bytes, mul<SMALL>(t.D[0], img_b + wgt_b));
    y.prod_T = mul<SMALL>(mul24(t.T[0], t.T[1]), mul24(t.T[2], t.T[3]));
    y.S6 = mul<SMALL>(mul24(t.G[0], t.G[1]), mul24(t.G[2], t.G[3]));
    const double reads = d.bytes_f64 * ((double)y.S6 * (double)mul<SMALL>(mul24(t.O[0], t.O[1]), t.O[2])) * (double)t.D[0];
    y.S5[0] = reads * (double)img_b;
    y.S5[1] = reads * (double)wgt_b;
    y.S2f = d.f32_s2 ? 2.0f * ((float)prod_R * (float)prod_q) : (float)y.S2;
    y.S5f[0] = (float)y.S5[0];
    y.S5f[1] = (float)y.S5[1];
    y.S7[0] = cols_b;
    y.S7[1] = t.D[2];
    y.S7[2] = t.B[3];
    y.S3f = (float)y.S3;
    y.S6f = (float)y.S6;
}

template <bool DUMP, bool SMALL> __device__ __forceinline__ void NestDepthwiseConv2d::symbols(const SgDesc& d, const Tiling<4, 2>& t, Symbols& y)
{
    const uint32_t sh = (uint32_t)d.stride_h, sw = (uint32_t)d.stride_w;   // < 2^16
    const uint32_t rows_b = mul24(t.B[2] - 1, sh) + t.D[0], cols_b = mul24(t.B[3] - 1, sw) + t.D[1];
    const uint32_t rows_r = mul24(t.R[2] - 1, sh) + t.q[0], cols_r = mul24(t.R[3] - 1, sw) + t.q[1];
    const uint32_t img_b = mul<SMALL>(mul<SMALL>(t.B[0], rows_b), cols_b), wgt_b = mul24(t.D[0], t.D[1]);   // per channel
    const uint32_t prod_R = mul<SMALL>(mul24(t.R[0], t.R[1]), mul24(t.R[2], t.R[3])), prod_q = mul24(t.q[0], t.q[1]);
    y.S1 = prod_R + mul<SMALL>(t.R[1], mul<SMALL>(mul<SMALL>(t.R[0], rows_r), cols_r) + prod_q);
    y.S2 = 2.0 * ((double)prod_R * (double)prod_q);
    y.S3 = mul<SMALL>(d.dtype_bytes, mul<SMALL>(t.B[1], img_b + wgt_b));
    y.prod_T = mul<SMALL>(mul24(t.T[0], t.T[1]), mul24(t.T[2], t.T[3]));
    y.S6 = mul<SMALL>(mul24(t.G[0], t.G[1]), mul24(t.G[2], t.G[3]));
    const double reads = d.bytes_f64 * ((double)y.S6 * (double)mul24(t.O[0], t.O[1])) * (double)t.B[1];
    y.S5[0] = reads * (double)img_b;
    y.S5[1] = reads * (double)wgt_b;
    y.S2f = d.f32_s2 ? 2.0f * ((float)prod_R * (float)prod_q) : (float)y.S2;
    y.S5f[0] = (float)y.S5[0];
    y.S5f[1] = (float)y.S5[1];
    y.S7[0] = cols_b;
    y.S7[1] = t.D[1];
    y.S7[2] = t.B[3];
    y.S3f = (float)y.S3;
    y.S6f = (float)y.S6;
}

namespace generic {
__device__ __forceinline__ uint32_t pick(const uint32_t* e, int axis)
{
    uint32_t v = e[0];
#pragma unroll
    for (int a = 1; a < PRUNER_MAX_AXES; ++a) v = axis == a ? e[a] : v;
    return v;
}
// extent of one buffer dimension over a tile with per-axis extents e[]: 1 + sum coef * (e - 1)
__device__ __forceinline__ uint32_t ext(const uint32_t* e, const SgDesc& d, int b, int dim)
{
    uint32_t x = 1;
#pragma unroll
    for (int t = 0; t < PRUNER_MAX_TERMS; ++t) {
        const int axis = d.axis[b][dim][t];
        if (axis >= 0) x += (uint32_t)d.coef[b][dim][t] * (pick(e, axis) - 1);
    }
    return x;
}
__device__ __forceinline__ uint32_t footprint(const uint32_t* e, const SgDesc& d, int b)
{
    uint32_t p = 1;
#pragma unroll
    for (int dim = 0; dim < PRUNER_MAX_DIMS; ++dim)
        if (dim < d.ndim[b]) p *= ext(e, d, b, dim);
    return p;
}
__device__ __forceinline__ uint32_t run(const uint32_t* e, const SgDesc& d, int b)
{
    uint32_t r = 1;
#pragma unroll
    for (int dim = 0; dim < PRUNER_MAX_DIMS; ++dim)
        if (dim == d.ndim[b] - 1) r = ext(e, d, b, dim);
    return r;
}
}  // namespace generic

template <bool DUMP, bool SMALL> __device__ __forceinline__ void NestGeneric::symbols(const SgDesc& d, const Tiling<4, 3>& t, Symbols& y)
{
    uint32_t e_blk[PRUNER_MAX_AXES], e_reg[PRUNER_MAX_AXES];
    uint32_t prod_R = 1, prod_T = 1, prod_G = 1, prod_q = 1, prod_O = 1;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        e_blk[a] = t.B[a];
        e_reg[a] = t.R[a];
        prod_R *= t.R[a];
        prod_T *= t.T[a];
        prod_G *= t.G[a];
    }
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        e_blk[4 + r] = t.D[r];
        e_reg[4 + r] = t.q[r];
        prod_q *= t.q[r];
        prod_O *= t.O[r];
    }
    const bool two = d.n_in > 1;
    const uint32_t fpb0 = generic::footprint(e_blk, d, 0), fpb1 = two ? generic::footprint(e_blk, d, 1) : 0u;
    y.S1 = prod_R + generic::footprint(e_reg, d, 0) + (two ? generic::footprint(e_reg, d, 1) : 0u);
    y.S2 = 2.0 * ((double)prod_R * (double)prod_q);
    y.S3 = d.dtype_bytes * (fpb0 + fpb1);
    y.prod_T = prod_T;
    y.S6 = prod_G;
    const double reads = d.bytes_f64 * ((double)prod_G * (double)prod_O);
    y.S5[0] = reads * (double)fpb0;
    y.S5[1] = reads * (double)fpb1;
    y.S2f = d.f32_s2 ? 2.0f * ((float)prod_R * (float)prod_q) : (float)y.S2;
    y.S5f[0] = (float)y.S5[0];
    y.S5f[1] = (float)y.S5[1];
    y.S7[0] = generic::run(e_blk, d, 0);
    y.S7[1] = two ? generic::run(e_blk, d, 1) : 1u;
    y.S7[2] = generic::run(e_blk, d, 2);
    y.S3f = (float)y.S3;
    y.S6f = (float)y.S6;
}

// VEC consecutive uint16 tile factors of one slot, as loaded: kept packed while a later chunk's loads are in flight.
// Every tile byte is read exactly once, so the loads carry the streaming (non-temporal) hint and leave the caches
// to the scores, which the selection stage reads back right away.
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
template <int VEC> struct Packed;
template <> struct Packed<1> {
    typedef uint32_t type;
    __device__ static type load(const uint16_t* p) { return __builtin_nontemporal_load(p); }
    __device__ static void unpack(type w, uint32_t* out) { out[0] = w; }
};
template <> struct Packed<2> {
    typedef uint32_t type;
    __device__ static type load(const uint16_t* p) { return __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(p)); }
    __device__ static void unpack(type w, uint32_t* out)
    {
        out[0] = w & 0xFFFFu;
        out[1] = w >> 16;
    }
};
template <> struct Packed<4> {
    typedef u32x2 type;
    __device__ static type load(const uint16_t* p) { return __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p)); }
    __device__ static void unpack(type w, uint32_t* out)
    {
        out[0] = w.x & 0xFFFFu;
        out[1] = w.x >> 16;
        out[2] = w.y & 0xFFFFu;
        out[3] = w.y >> 16;
    }
};

// The tile slots of a thread's VEC candidates, straight from memory.
template <class Nest, int VEC> struct RawTiles {
    typename Packed<VEC>::type sp[Nest::NSP][4];
    typename Packed<VEC>::type rd[Nest::NRD][3];
};

template <class Nest, int VEC>
__device__ __forceinline__ void load_tiles(const SgDesc& d, const uint16_t* __restrict__ tiles, int64_t pitch, int64_t c0, RawTiles<Nest, VEC>& raw)
{
    constexpr int NSP = Nest::NSP, NRD = Nest::NRD;
    const uint16_t* col = tiles + c0;
#pragma unroll
    for (int a = 0; a < NSP; ++a) {
#pragma unroll
        for (int l = 0; l < 4; ++l)
            if (Nest::FIXED || a < d.n_sp) raw.sp[a][l] = Packed<VEC>::load(col + (int64_t)(a * 4 + l) * pitch);
    }
    const int rdl = d.rd_levels;
#pragma unroll
    for (int r = 0; r < NRD; ++r) {
#pragma unroll
        for (int l = 0; l < 3; ++l)
            if ((Nest::FIXED || r < d.n_rd) && l < rdl)
                raw.rd[r][l] = Packed<VEC>::load(col + (int64_t)((Nest::FIXED ? NSP : d.n_sp) * 4 + r * rdl + l) * pitch);
    }
}

// SchMutation of Alg. 2 in place of the loads (the explorer loop from its second step on): the thread's four
// candidates are made from parents in S_spec, stored as the population's new columns, and handed on in the layout the
// loads would have produced; the population is written once and not read back.  NP: 16-byte pieces of a record that
// the subgraph's slots reach.
struct MutSeg {
    LseSeg seg;
    int32_t sub, count;   // count < 1: the subgraph has no S_spec, its population stays as it is
};

template <class Nest, int NP>
__device__ __forceinline__ void make_children_np(const SgDesc& d, const MutSeg& ms, const MutArgs& mut, uint16_t* __restrict__ tiles,
                                                 int64_t pitch, int64_t c0, int64_t c_end, RawTiles<Nest, 4>& raw)
{
    constexpr int NSP = Nest::NSP, NRD = Nest::NRD;
    constexpr int kRows = 8 * NP < PRUNER_MAX_SLOTS ? 8 * NP : PRUNER_MAX_SLOTS;
    const int live = c_end - c0 < 4 ? (int)(c_end - c0) : 4;
    const uint64_t z0 = lse_child_state(mut.seed, mut.step, c0);
    uint32_t f[4][kAosWords];
    lse_child<NP>(ms.seg, ms.sub, ms.count, mut.k, z0, mut.spec_aos, mut.mutate_q16, f[0]);
#pragma unroll
    for (int e = 1; e < 4; ++e) {
        if (e < live) {
            lse_child<NP>(ms.seg, ms.sub, ms.count, mut.k, z0 + (uint64_t)(2 * e) * kGamma, mut.spec_aos, mut.mutate_q16, f[e]);
        } else {
            // past the segment's end: a valid schedule that is neither stored nor scored
#pragma unroll
            for (int w = 0; w < kAosWords; ++w) f[e][w] = f[0][w];
        }
    }
    // row by row: the factor of each of the four children, as a column load would deliver it
    u32x2 T[kAosSlots];
#pragma unroll
    for (int row = 0; row < kAosSlots; ++row) {
        if (row < kRows) {
            const uint32_t half = row & 1 ? 0x07060302u : 0x05040100u;
            T[row].x = __builtin_amdgcn_perm(f[1][row >> 1], f[0][row >> 1], half);
            T[row].y = __builtin_amdgcn_perm(f[3][row >> 1], f[2][row >> 1], half);
            if (row < ms.seg.n_slots) {
                uint16_t* dst = tiles + (int64_t)row * pitch + c0;
                if (live == 4) {
                    *reinterpret_cast<u32x2*>(dst) = T[row];
                } else {
#pragma unroll
                    for (int e = 0; e < 3; ++e)
                        if (e < live) dst[e] = (uint16_t)(f[e][row >> 1] >> (16 * (row & 1)));
                }
            }
        } else {
            T[row] = u32x2{0u, 0u};
        }
    }
#pragma unroll
    for (int a = 0; a < NSP; ++a) {
#pragma unroll
        for (int l = 0; l < 4; ++l)
            if (Nest::FIXED || a < d.n_sp) raw.sp[a][l] = T[a * 4 + l];
    }
    // the reduction slots follow the spatial ones: at a row that depends on the number of spatial axes and of levels
    u32x2 U[NRD * 3];
#pragma unroll
    for (int i = 0; i < NRD * 3; ++i) {
        if constexpr (Nest::FIXED) {
            U[i] = T[NSP * 4 + i];
        } else {
            U[i] = T[4 + i];
#pragma unroll
            for (int n = 2; n <= NSP; ++n)
                if (d.n_sp == n) U[i] = T[n * 4 + i];
        }
    }
    const int rdl = d.rd_levels;
#pragma unroll
    for (int r = 0; r < NRD; ++r) {
#pragma unroll
        for (int l = 0; l < 3; ++l)
            if ((Nest::FIXED || r < d.n_rd) && l < rdl) raw.rd[r][l] = rdl == 3 ? U[r * 3 + l] : U[(r * 2 + l) % (NRD * 3)];
    }
}

template <class Nest>
__device__ __forceinline__ void make_children(const SgDesc& d, const MutSeg& ms, const MutArgs& mut, uint16_t* __restrict__ tiles, int64_t pitch,
                                              int64_t c0, int64_t c_end, RawTiles<Nest, 4>& raw)
{
    switch ((ms.seg.n_slots + 7) >> 3) {   // the same for the whole workgroup
        case 0:
        case 1: make_children_np<Nest, 1>(d, ms, mut, tiles, pitch, c0, c_end, raw); break;
        case 2: make_children_np<Nest, 2>(d, ms, mut, tiles, pitch, c0, c_end, raw); break;
        case 3: make_children_np<Nest, 3>(d, ms, mut, tiles, pitch, c0, c_end, raw); break;
        default: make_children_np<Nest, 4>(d, ms, mut, tiles, pitch, c0, c_end, raw); break;
    }
}

// ---- penalties, utilisation, latency: the binary32 sequence of the header comment -----------------------------------
// Written stage by stage over the VEC candidates of a thread, so that the candidates' dependent chains interleave;
// branches depend on per-subgraph constants only and are taken by the whole wavefront.

template <int VEC> __device__ __forceinline__ void cdiv_vec(const uint32_t (&x)[VEC], const UDiv& u, uint32_t (&out)[VEC])
{
    if (u.pow2) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) out[v] = (x[v] + u.d - 1) >> u.sh;
    } else {
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            const uint32_t y = x[v] + u.d - 1, q = __umulhi(u.m, y);
            out[v] = (((y - q) >> 1) + q) >> u.sh;
        }
    }
}
template <int VEC> __device__ __forceinline__ void round_up_vec(const uint32_t (&x)[VEC], const UDiv& u, uint32_t (&out)[VEC])
{
    if (u.pow2) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) out[v] = (x[v] + u.d - 1) & ~(u.d - 1);
    } else {
        cdiv_vec<VEC>(x, u, out);
#pragma unroll
        for (int v = 0; v < VEC; ++v) out[v] *= u.d;
    }
}
// q[v] = a[v] / b[v], correctly rounded
template <int VEC> __device__ __forceinline__ void div_vec(const float (&a)[VEC], const float (&b)[VEC], float (&q)[VEC])
{
    float y[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) y[v] = recip(b[v]);
#pragma unroll
    for (int v = 0; v < VEC; ++v) q[v] = div_by(a[v], b[v], y[v]);
}
template <int VEC> __device__ __forceinline__ void ratio_vec(const uint32_t (&a)[VEC], const uint32_t (&b)[VEC], float (&q)[VEC])
{
    float fa[VEC], fb[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        fa[v] = (float)a[v];
        fb[v] = (float)b[v];
    }
    div_vec<VEC>(fa, fb, q);
}

template <int VEC>
__device__ __forceinline__ void analyze(const SgDesc& d, const Symbols (&y)[VEC], const uint32_t (&S1)[VEC], const uint32_t (&S4)[VEC],
                                        const float (&frag_num)[VEC], const float (&frag_den)[VEC], bool whole_fragments, int32_t flags,
                                        const float* p2m_tab /* LDS table of P_l2,m by run length, or null */, float (&score)[VEC])
{
    float L[VEC], Tm0[VEC];
    {   // compute statement: L = S8 / Up
        float Up[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) Up[v] = d.T_p;
        if (!(flags & PRUNER_NO_COMPUTE_PENALTY)) {
            float S1f[VEC], rS1[VEC], S2f[VEC], P0c[VEC], P1c[VEC], alpha[VEC], P2c[VEC];
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                S1f[v] = (float)S1[v];
                rS1[v] = recip(S1f[v]);
                S2f[v] = y[v].S2f;
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v) P0c[v] = 1.0f + div_by(S2f[v], S1f[v], rS1[v]);
            uint32_t sch[VEC], sch_up[VEC], lanes[VEC], S6[VEC], S6_up[VEC];
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                alpha[v] = 1.0f;
                S6[v] = y[v].S6;
            }
            if (d.frag_mode) {
                // S4 = n_l1 * prod T: the block is prod T whole warps, so sch = prod T and alpha = S4 / S4 = 1 exactly
#pragma unroll
                for (int v = 0; v < VEC; ++v) sch[v] = y[v].prod_T;
            } else {
                cdiv_vec<VEC>(S4, d.div_n_l1, sch);
#pragma unroll
                for (int v = 0; v < VEC; ++v) lanes[v] = sch[v] * d.n_l1;
                ratio_vec<VEC>(S4, lanes, alpha);
            }
            round_up_vec<VEC>(sch, d.div_pu_l1, sch_up);
            ratio_vec<VEC>(sch, sch_up, P1c);
            round_up_vec<VEC>(S6, d.div_pu_l2, S6_up);
            {
                float num[VEC], den[VEC];
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    num[v] = y[v].S6f;
                    den[v] = (float)S6_up[v];
                }
                div_vec<VEC>(num, den, P2c);
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v) Up[v] = (((Up[v] * P0c[v]) * P1c[v]) * alpha[v]) * P2c[v];
            if (d.frag_mode && !whole_fragments) {   // otherwise the factor is x / x = 1 in every lane
                float Ptc[VEC];
                div_vec<VEC>(frag_num, frag_den, Ptc);
#pragma unroll
                for (int v = 0; v < VEC; ++v) Up[v] = Up[v] * Ptc[v];
            }
        }
        float S8f[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) S8f[v] = d.S8f;
        div_vec<VEC>(S8f, Up, L);
    }
    if (!(flags & PRUNER_NO_MEMORY_PENALTY)) {
        float S1f[VEC], S3f[VEC], m0[VEC], m1[VEC], P0m[VEC], P1m[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            S1f[v] = (float)S1[v];
            S3f[v] = y[v].S3f;
            m0[v] = d.m_l0f;
            m1[v] = d.m_l1f;
        }
        div_vec<VEC>(m0, S1f, P0m);
        div_vec<VEC>(m1, S3f, P1m);
#pragma unroll
        for (int v = 0; v < VEC; ++v) Tm0[v] = (d.T_m * fminf(P0m[v], 1.0f)) * fminf(P1m[v], 1.0f);
    }
#pragma unroll
    for (int s = 0; s < 3; ++s) {   // memory statements In_0, In_1, store: L += S5 / Um
        if (s == 1 && d.n_in < 2) continue;
        float S5f[VEC], Um[VEC], Lm[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            S5f[v] = s < 2 ? y[v].S5f[s] : d.S5out_f;
            Um[v] = d.T_m;
        }
        if (!(flags & PRUNER_NO_MEMORY_PENALTY)) {
            uint32_t S7[VEC], S7_up[VEC];
            float P2m[VEC];
#pragma unroll
            for (int v = 0; v < VEC; ++v) S7[v] = y[v].S7[s];
            if (p2m_tab) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) P2m[v] = p2m_tab[S7[v] < (uint32_t)kTabMax ? S7[v] : (uint32_t)kTabMax];   // clamp: factors that break the contract stay in bounds
            } else {
                round_up_vec<VEC>(S7, d.div_n_l2, S7_up);
                ratio_vec<VEC>(S7, S7_up, P2m);
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v) Um[v] = Tm0[v] * P2m[v];
        }
        div_vec<VEC>(S5f, Um, Lm);
#pragma unroll
        for (int v = 0; v < VEC; ++v) L[v] = L[v] + Lm[v];
    }
#pragma unroll
    for (int v = 0; v < VEC; ++v) score[v] = -L[v];
}

// Eq. 1 with the penalties of one statement group multiplied out before dividing.  Every penalty is a ratio, so
//   L_c = S8 / (T_p * P_l0,c * P_l1,c * alpha_l1 * P_l2,c [* fragment ratio])
//       = (S8 / T_p) * [S1 * sch_up * lanes * S6_up (* frag_den)] / [(S1 + S2) * S4' * S6 (* frag_num)]
// (P_l1,c * alpha_l1 = S4' / (sch_up * lanes) with S4' = prod T: lanes = n_l1, or 1 in fragment mode where alpha = 1),
// and min(m / S, 1) = 1 / max(S / m, 1), so
//   sum_s L_m,s = [sum_s S5_s / P_l2,m(S7_s)] * max(S1 / m_l0, 1) * max(S3 / m_l1, 1) / T_m.
// One reciprocal estimate (1 ulp) and about a dozen roundings per statement group; every term is positive, so the
// relative error of the score stays below 2^-20 (the parity bound is 1e-5).  Operands are the same exact symbols as in
// analyze(); the products stay inside binary32's range under the bounds the host checks.
template <int VEC>
__device__ __forceinline__ void analyze_fused(const SgDesc& d, const Symbols (&y)[VEC], const uint32_t (&S1)[VEC],
                                              const float (&frag_num)[VEC], const float (&frag_den)[VEC], bool whole_fragments,
                                              int32_t flags, const float* inv_p2m_tab /* LDS table of 1 / P_l2,m, or null */,
                                              float (&score)[VEC])
{
    float L[VEC], S1f[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        S1f[v] = (float)S1[v];
        L[v] = d.k_c;
    }
    if (!(flags & PRUNER_NO_COMPUTE_PENALTY)) {
        uint32_t sch[VEC], sch_up[VEC], S6[VEC], S6_up[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            sch[v] = y[v].prod_T;
            S6[v] = y[v].S6;
        }
        if (!d.frag_mode) cdiv_vec<VEC>(sch, d.div_n_l1, sch);
        round_up_vec<VEC>(sch, d.div_pu_l1, sch_up);
        round_up_vec<VEC>(S6, d.div_pu_l2, S6_up);
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            float num = ((S1f[v] + y[v].S2f) * y[v].S6f) * (float)y[v].prod_T;
            float den = (S1f[v] * (float)S6_up[v]) * ((float)sch_up[v] * d.lanes_f);
            if (d.frag_mode && !whole_fragments) {
                num = num * frag_num[v];
                den = den * frag_den[v];
            }
            L[v] = (den * __builtin_amdgcn_rcpf(num)) * d.k_c;
        }
    }
    float w[VEC], sum[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        w[v] = d.inv_Tm;
        sum[v] = 0.0f;
    }
    if (!(flags & PRUNER_NO_MEMORY_PENALTY)) {
#pragma unroll
        for (int v = 0; v < VEC; ++v)
            w[v] = (fmaxf(S1f[v] * d.inv_m0, 1.0f) * fmaxf(y[v].S3f * d.inv_m1, 1.0f)) * d.inv_Tm;
    }
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        if (s == 1 && d.n_in < 2) continue;
        float inv[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) inv[v] = 1.0f;
        if (!(flags & PRUNER_NO_MEMORY_PENALTY)) {
            uint32_t S7[VEC], S7_up[VEC];
#pragma unroll
            for (int v = 0; v < VEC; ++v) S7[v] = y[v].S7[s];
            if (inv_p2m_tab) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) inv[v] = inv_p2m_tab[S7[v] < (uint32_t)kTabMax ? S7[v] : (uint32_t)kTabMax];
            } else {
                // the table's entries are correctly rounded quotients: the same here, so that a score does not depend
                // on whether its workgroup tabulated (which follows from the launch shape, not from the candidate)
                round_up_vec<VEC>(S7, d.div_n_l2, S7_up);
                ratio_vec<VEC>(S7_up, S7, inv);
            }
        }
#pragma unroll
        for (int v = 0; v < VEC; ++v) sum[v] = __builtin_fmaf(s < 2 ? y[v].S5f[s] : d.S5out_f, inv[v], sum[v]);
    }
#pragma unroll
    for (int v = 0; v < VEC; ++v) score[v] = -__builtin_fmaf(sum[v], w[v], L[v]);
}

template <class Nest, int VEC, bool DUMP, bool EXACT, bool HIST>
__device__ __forceinline__ void score_candidates(const SgDesc& d, const RawTiles<Nest, VEC>& raw, int64_t c0, int64_t c_end,
                                                 int32_t flags, const float* p2m_tab, float* __restrict__ score,
                                                 int64_t* __restrict__ symbols, int64_t n_total, uint32_t* digit_hist,
                                                 uint32_t* __restrict__ block_max, int seg_index)
{
    constexpr int NSP = Nest::NSP, NRD = Nest::NRD;
    uint32_t sp[NSP][4][VEC];   // grid, virtual thread, thread, inner
    uint32_t rd[NRD][3][VEC];   // outer steps, middle, inner (inner = 1 with two levels)
#pragma unroll
    for (int a = 0; a < NSP; ++a) {
#pragma unroll
        for (int l = 0; l < 4; ++l) {
            if (Nest::FIXED || a < d.n_sp) {
                Packed<VEC>::unpack(raw.sp[a][l], sp[a][l]);
            } else {
#pragma unroll
                for (int v = 0; v < VEC; ++v) sp[a][l][v] = 1;
            }
        }
    }
    const int rdl = d.rd_levels;
#pragma unroll
    for (int r = 0; r < NRD; ++r) {
#pragma unroll
        for (int l = 0; l < 3; ++l) {
            if ((Nest::FIXED || r < d.n_rd) && l < rdl) {
                Packed<VEC>::unpack(raw.rd[r][l], rd[r][l]);
            } else {
#pragma unroll
                for (int v = 0; v < VEC; ++v) rd[r][l][v] = 1;
            }
        }
    }

    Symbols y[VEC];
    uint32_t S1[VEC], S4[VEC];
    float frag_num[VEC], frag_den[VEC];
    bool whole_fragments = false;
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        Tiling<NSP, NRD> t;
#pragma unroll
        for (int a = 0; a < NSP; ++a) {
            t.G[a] = sp[a][0][v];
            t.V[a] = sp[a][1][v];
            t.T[a] = sp[a][2][v];
            t.In[a] = sp[a][3][v];
            t.R[a] = mul24(sp[a][1][v], sp[a][3][v]);
            t.B[a] = mul24(t.R[a], t.T[a]);     // the factors of an axis multiply to its extent, which is below 2^16
        }
#pragma unroll
        for (int r = 0; r < NRD; ++r) {
            t.O[r] = rd[r][0][v];
            t.Mid[r] = rd[r][1][v];
            t.q[r] = rd[r][2][v];
            t.D[r] = rdl == 3 ? mul24(rd[r][1][v], rd[r][2][v]) : rd[r][1][v];
        }
        if (d.small) Nest::template symbols<DUMP, true>(d, t, y[v]);
        else Nest::template symbols<DUMP, false>(d, t, y[v]);
        S1[v] = y[v].S1;
        S4[v] = y[v].prod_T;
        frag_num[v] = 1.0f;
        frag_den[v] = 1.0f;
    }
    if (d.frag_mode) {
        // thread-level factors count warps: n_l1 lanes each, the register tile shared out over them; the inner tiles
        // of the last two spatial axes and of the last reduction axis are rounded up to whole fragments
        cdiv_vec<VEC>(S1, d.div_n_l1, S1);
        uint32_t fi[VEC], fj[VEC], fk[VEC], ui[VEC], uj[VEC], uk[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            S4[v] = d.n_l1 * S4[v];
            if constexpr (Nest::FIXED) {
                fi[v] = sp[NSP >= 2 ? NSP - 2 : 0][3][v];
                fj[v] = sp[NSP - 1][3][v];
                fk[v] = rd[NRD - 1][2][v];
            } else {
                fi[v] = fj[v] = fk[v] = 1;
#pragma unroll
                for (int a = 0; a < NSP; ++a) {
                    if (a == d.n_sp - 2) fi[v] = sp[a][3][v];
                    if (a == d.n_sp - 1) fj[v] = sp[a][3][v];
                }
#pragma unroll
                for (int r = 0; r < NRD; ++r)
                    if (r == d.n_rd - 1) fk[v] = rd[r][2][v];
            }
        }
        round_up_vec<VEC>(fi, d.div_frag[0], ui);
        round_up_vec<VEC>(fj, d.div_frag[1], uj);
        round_up_vec<VEC>(fk, d.div_frag[2], uk);
        bool whole = true;
#pragma unroll
        for (int v = 0; v < VEC; ++v) whole = whole && fi[v] == ui[v] && fj[v] == uj[v] && fk[v] == uk[v];
        whole_fragments = __all(whole);   // same for the whole wavefront
        if (!whole_fragments) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                // a candidate of whole fragments keeps the factors 1 (exact products): its score is then the same
                // whether or not its wavefront takes this branch
                if (!EXACT && fi[v] == ui[v] && fj[v] == uj[v] && fk[v] == uk[v]) continue;
                if (d.f32_frag) {
                    frag_num[v] = (float)(fi[v] * fj[v]) * (float)fk[v];
                    frag_den[v] = (float)(ui[v] * uj[v]) * (float)uk[v];
                } else {
                    frag_num[v] = (float)(((double)fi[v] * (double)fj[v]) * (double)fk[v]);
                    frag_den[v] = (float)(((double)ui[v] * (double)uj[v]) * (double)uk[v]);
                }
            }
        }
    }

    float out[VEC];
    if constexpr (EXACT) analyze<VEC>(d, y, S1, S4, frag_num, frag_den, whole_fragments, flags, p2m_tab, out);
    else analyze_fused<VEC>(d, y, S1, frag_num, frag_den, whole_fragments, flags, p2m_tab, out);

    if constexpr (DUMP) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            const int64_t c = c0 + v;
            if (c < c_end) {
                symbols[PRUNER_SYM_S1 * n_total + c] = S1[v];
                symbols[PRUNER_SYM_S2 * n_total + c] = (int64_t)y[v].S2;
                symbols[PRUNER_SYM_S3 * n_total + c] = y[v].S3;
                symbols[PRUNER_SYM_S4 * n_total + c] = S4[v];
                symbols[PRUNER_SYM_S6 * n_total + c] = y[v].S6;
                symbols[PRUNER_SYM_S8 * n_total + c] = d.S8;
                symbols[PRUNER_SYM_S5_IN0 * n_total + c] = (int64_t)y[v].S5[0];
                symbols[PRUNER_SYM_S7_IN0 * n_total + c] = y[v].S7[0];
                symbols[PRUNER_SYM_S5_IN1 * n_total + c] = d.n_in > 1 ? (int64_t)y[v].S5[1] : 0;
                symbols[PRUNER_SYM_S7_IN1 * n_total + c] = d.n_in > 1 ? y[v].S7[1] : 0;
                symbols[PRUNER_SYM_S5_OUT * n_total + c] = d.S5out;
                symbols[PRUNER_SYM_S7_OUT * n_total + c] = y[v].S7[2];
            }
        }
    }

    if constexpr (HIST) {
        // the selection stage's first pass, done here while the scores are in registers.  Plain LDS atomics: even
        // when all lanes hit one bin (equal scores) their serialisation stays hidden under this kernel's loads.
        uint32_t top = 0;   // below the key of every number
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            if (c0 + v < c_end) {
                const uint32_t key = key_of(out[v]);
                atomicAdd(&digit_hist[key >> 21], 1u);
                top = key > top ? key : top;
            }
        }
        // and the largest key of the wavefront's 256 neighbouring candidates, by which the selection's second pass steps
        // over the block.  The lanes at work here are lanes 0..m (a thread is here when its first candidate lies inside
        // the segment): lane m ends up with the maximum.
        if constexpr (VEC == 4) {
            if (block_max) {
                top = wave_inclusive_max(top);
                const int last = 63 - __clzll(__ballot(true));
                if (lane_id() == last) block_max[block_max_slot(c0 - 4 * last, seg_index)] = top;
            }
        }
    }

    if (c0 + VEC <= c_end) {
        if constexpr (VEC == 4) {
            *reinterpret_cast<float4*>(score + c0) = make_float4(out[0], out[1], out[2], out[3]);
        } else if constexpr (VEC == 2) {
            *reinterpret_cast<float2*>(score + c0) = make_float2(out[0], out[1]);
        } else {
            score[c0] = out[0];
        }
    } else {
#pragma unroll
        for (int v = 0; v < VEC; ++v)
            if (c0 + v < c_end) score[c0 + v] = out[v];
    }
}

// The chunks of one workgroup: the workgroups of a segment take its chunks round robin, so that at any moment the
// resident workgroups read one contiguous window of every slot row.  The tile slots of the next chunk are
// requested before the current one is scored: every wavefront keeps loads in flight while it computes.
template <class Nest, int VEC, bool DUMP, bool EXACT, bool HIST, bool MUT>
__device__ __forceinline__ void walk_segment(const SgDesc& d, const SegEnt& seg, int32_t b, const uint16_t* __restrict__ tiles,
                                             int64_t pitch, int32_t flags, const float* p2m_tab, float* __restrict__ score,
                                             int64_t* __restrict__ symbols, int64_t n_total, uint32_t* digit_hist, uint32_t* __restrict__ block_max,
                                             const MutArgs& mut)
{
    const int64_t step = (int64_t)seg.blocks * kBlock * VEC;
    RawTiles<Nest, VEC> cur{}, nxt{};
    int64_t c0 = seg.begin + ((int64_t)(b - seg.first_block) * kBlock + threadIdx.x) * VEC;
    if constexpr (MUT) {
        static_assert(VEC == 4, "children are made four at a time");
        MutSeg ms;
        ms.seg = mut.segs[seg.seg];
        ms.sub = seg.seg;
        ms.count = mut.spec_count[seg.seg];
        if (ms.count >= 1) {
            // (the population is this call's to write: the explorer loop hands its own buffer in)
            uint16_t* out = const_cast<uint16_t*>(tiles);
            for (int it = 0; it < seg.iters; ++it) {
                if (c0 < seg.end) {
                    make_children<Nest>(d, ms, mut, out, pitch, c0, seg.end, cur);
                    score_candidates<Nest, VEC, DUMP, EXACT, HIST>(d, cur, c0, seg.end, flags, p2m_tab, score, symbols, n_total, digit_hist, block_max, seg.seg);
                }
                c0 += step;
            }
            return;
        }
    }
    if constexpr (MUT || Nest::NSP * 4 + Nest::NRD * 3 > 16) {
        // many slots: a second set of them in flight costs more in occupancy than it gains
        // (and in the kernels that make their candidates this path only serves a subgraph without S_spec)
        for (int it = 0; it < seg.iters; ++it) {
            if (c0 < seg.end) {
                load_tiles<Nest, VEC>(d, tiles, pitch, c0, cur);
                score_candidates<Nest, VEC, DUMP, EXACT, HIST>(d, cur, c0, seg.end, flags, p2m_tab, score, symbols, n_total, digit_hist, block_max, seg.seg);
            }
            c0 += step;
        }
        return;
    }
    if (c0 < seg.end) load_tiles<Nest, VEC>(d, tiles, pitch, c0, cur);
    for (int it = 0; it < seg.iters; ++it) {
        const int64_t c1 = c0 + step;
        if (it + 1 < seg.iters && c1 < seg.end) load_tiles<Nest, VEC>(d, tiles, pitch, c1, nxt);
        if (c0 < seg.end) score_candidates<Nest, VEC, DUMP, EXACT, HIST>(d, cur, c0, seg.end, flags, p2m_tab, score, symbols, n_total, digit_hist, block_max, seg.seg);
        cur = nxt;
        c0 = c1;
    }
}

constexpr int kAnyClass = -1;

// One launch scores the segments of one loop-nest class (CLS), so that each class gets the register budget, and with
// it the occupancy, of its own symbol code; CLS = kAnyClass branches on the class at run time instead and serves
// small populations, where one launch for everything beats several, and the narrow load widths.
// HIST: the workgroup also counts the first selection digit (top 11 bits of the order-preserving key) of its scores
// in LDS and merges the counts into one of `copies` global histograms of its segment.
// MUT: the candidates are not read but made (SchMutation from S_spec, `mut`), stored and scored in one pass.
template <int CLS, int VEC, bool DUMP, bool EXACT, bool HIST, bool MUT>
__global__ void __launch_bounds__(kBlock) draft_kernel(const SegEnt* __restrict__ segs, int32_t n_seg,
                                                       const SgDesc* __restrict__ descs, const uint16_t* __restrict__ tiles,
                                                       int64_t pitch, int32_t flags, float* __restrict__ score,
                                                       int64_t* __restrict__ symbols, int64_t n_total,
                                                       uint32_t* __restrict__ first_digit, uint32_t* __restrict__ block_max, int copies,
                                                       int n_sg_all, MutArgs mut)
{
    const int32_t b = blockIdx.x;
    const SegEnt seg = segs[segment_of_block(segs, n_seg, b)];
    const SgDesc& d = descs[seg.desc];

    // P_l2,m = S7 / (ceil(S7 / n_l2) * n_l2) depends on the run length alone: when a block scores enough candidates,
    // the quotients for all possible run lengths (their inverses for the fused evaluation) are formed once and the
    // three memory statements look them up.
    __shared__ float tab[kTabMax + 1];
    __shared__ uint32_t digit_hist[HIST ? kBins : 1];
    if constexpr (HIST) {
        for (int i = threadIdx.x; i < kBins; i += kBlock) digit_hist[i] = 0;
        if (!seg.use_tab) __syncthreads();
    }
    if (seg.use_tab) {
        for (int r = threadIdx.x; r <= d.run_max; r += kBlock) {
            const uint32_t run[1] = {r > 0 ? (uint32_t)r : 1u};
            uint32_t up[1];
            round_up_vec<1>(run, d.div_n_l2, up);
            tab[r] = EXACT ? div_rn((float)run[0], (float)up[0]) : div_rn((float)up[0], (float)run[0]);
        }
        __syncthreads();
    }
    const float* p2m_tab = seg.use_tab ? tab : nullptr;

#define PRUNER_WALK(NEST) walk_segment<NEST, VEC, DUMP, EXACT, HIST, MUT>(d, seg, b, tiles, pitch, flags, p2m_tab, score, symbols, n_total, digit_hist, block_max, mut)
    if constexpr (CLS == kGemm) PRUNER_WALK(NestGemm);
    else if constexpr (CLS == kBatchedGemm) PRUNER_WALK(NestBatchedGemm);
    else if constexpr (CLS == kConv2d) PRUNER_WALK(NestConv2d);
    else if constexpr (CLS == kDepthwiseConv2d) PRUNER_WALK(NestDepthwiseConv2d);
    else if constexpr (CLS == kGeneric) PRUNER_WALK(NestGeneric);
    else {
        switch (d.cls) {
            case kGemm: PRUNER_WALK(NestGemm); break;
            case kBatchedGemm: PRUNER_WALK(NestBatchedGemm); break;
            case kConv2d: PRUNER_WALK(NestConv2d); break;
            case kDepthwiseConv2d: PRUNER_WALK(NestDepthwiseConv2d); break;
            default: PRUNER_WALK(NestGeneric); break;
        }
    }
#undef PRUNER_WALK
    if constexpr (HIST) {
        __syncthreads();
        flush_hist<kBlock>(digit_hist, first_digit, copies, n_sg_all, seg.seg);
    }
}

using DraftFn = void (*)(const SegEnt*, int32_t, const SgDesc*, const uint16_t*, int64_t, int32_t, float*, int64_t*, int64_t, uint32_t*, uint32_t*, int, int, MutArgs);

// The digit-counting variant exists for the full load width without the symbol dump (the shape large populations run in).
template <int CLS, bool DUMP, bool EXACT> DraftFn pick_vec(int vec, bool hist, bool mut)
{
    if constexpr (CLS == kAnyClass) {
        if (vec == 2) return draft_kernel<CLS, 2, DUMP, EXACT, false, false>;
        if (vec == 1) return draft_kernel<CLS, 1, DUMP, EXACT, false, false>;
    }
    if constexpr (!DUMP) {
        if constexpr (CLS != kAnyClass) {
            if (hist && mut) return draft_kernel<CLS, 4, false, EXACT, true, true>;
        }
        if (hist) return draft_kernel<CLS, 4, false, EXACT, true, false>;
    }
    return draft_kernel<CLS, 4, DUMP, EXACT, false, false>;
}
template <bool DUMP, bool EXACT> DraftFn pick_class(int cls, int vec, bool hist, bool mut)
{
    switch (cls) {
        case kGemm: return pick_vec<kGemm, DUMP, EXACT>(vec, hist, mut);
        case kBatchedGemm: return pick_vec<kBatchedGemm, DUMP, EXACT>(vec, hist, mut);
        case kConv2d: return pick_vec<kConv2d, DUMP, EXACT>(vec, hist, mut);
        case kDepthwiseConv2d: return pick_vec<kDepthwiseConv2d, DUMP, EXACT>(vec, hist, mut);
        case kGeneric: return pick_vec<kGeneric, DUMP, EXACT>(vec, hist, mut);
        default: return pick_vec<kAnyClass, DUMP, EXACT>(vec, hist, mut);
    }
}
// mut is honoured for the per-class kernels at the full load width that also count the first selection digit
DraftFn pick_kernel(int cls, int vec, bool dump, bool exact, bool hist, bool mut)
{
    if (dump) return exact ? pick_class<true, true>(cls, vec, hist, mut) : pick_class<true, false>(cls, vec, hist, mut);
    return exact ? pick_class<false, true>(cls, vec, hist, mut) : pick_class<false, false>(cls, vec, hist, mut);
}

// Workgroups of a kernel instance that the device holds at once (its register budget decides).  Asked of the runtime
// once per kernel instance and device and remembered (the answer does not change, and the two queries cost a call of a
// few thousand candidates a tenth of its time); two host threads that ask at once write the same values.
int64_t resident_blocks(DraftFn fn)
{
    struct Known { DraftFn fn; int dev; int64_t blocks; };
    static Known known[64];
    static int n_known = 0;
    int cus = 0;
    const int dev = current_device(&cus);
    if (dev < 0) {
        (void)hipGetLastError();
        return 256;   // (the launch that follows reports what is wrong with the device)
    }
    const int have = n_known;
    for (int i = 0; i < have; ++i)
        if (known[i].fn == fn && known[i].dev == dev) return known[i].blocks;
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kBlock, 0) != hipSuccess || per_cu < 1) per_cu = 1;
    (void)hipGetLastError();
    const int64_t blocks = (int64_t)per_cu * cus;
    if (have < 64) {
        known[have] = Known{fn, dev, blocks};
        n_known = have + 1;
    }
    return blocks;
}

// ---- host side: validation, classification, tables -------------------------------------------------------------

bool dim_is(const pruner_dim& d, int a0, int c0, int a1 = -1, int c1 = 0)
{
    // a dimension's terms may be listed in either order
    auto same = [&](int x0, int y0, int x1, int y1) {
        const bool t0 = d.axis[0] == x0 && (x0 < 0 || d.coef[0] == y0);
        const bool t1 = d.axis[1] == x1 && (x1 < 0 || d.coef[1] == y1);
        return t0 && t1;
    };
    return same(a0, c0, a1, c1) || (a1 >= 0 && same(a1, c1, a0, c0));
}

int32_t classify(const pruner_subgraph& s, int32_t* stride_h, int32_t* stride_w)
{
    *stride_h = *stride_w = 1;
    const pruner_buffer &A = s.in[0], &B = s.in[1], &O = s.out;
    if (s.n_in != 2) return kGeneric;
    if (s.n_sp == 2 && s.n_rd == 1 && A.ndim == 2 && B.ndim == 2 && O.ndim == 2 && dim_is(A.dim[0], 0, 1) &&
        dim_is(A.dim[1], 2, 1) && dim_is(B.dim[0], 2, 1) && dim_is(B.dim[1], 1, 1) && dim_is(O.dim[0], 0, 1) && dim_is(O.dim[1], 1, 1))
        return kGemm;
    if (s.n_sp == 3 && s.n_rd == 1 && A.ndim == 3 && B.ndim == 3 && O.ndim == 3 && dim_is(A.dim[0], 0, 1) &&
        dim_is(A.dim[1], 1, 1) && dim_is(A.dim[2], 3, 1) && dim_is(B.dim[0], 0, 1) && dim_is(B.dim[1], 3, 1) &&
        dim_is(B.dim[2], 2, 1) && dim_is(O.dim[0], 0, 1) && dim_is(O.dim[1], 1, 1) && dim_is(O.dim[2], 2, 1))
        return kBatchedGemm;
    const bool out4 = O.ndim == 4 && dim_is(O.dim[0], 0, 1) && dim_is(O.dim[1], 1, 1) && dim_is(O.dim[2], 2, 1) && dim_is(O.dim[3], 3, 1);
    auto strided = [](const pruner_dim& d, int sp_axis, int rd_axis, int32_t* stride) {
        for (int t = 0; t < 2; ++t)
            if (d.axis[t] == sp_axis && d.axis[1 - t] == rd_axis && d.coef[1 - t] == 1 && d.coef[t] >= 1) {
                *stride = d.coef[t];
                return true;
            }
        return false;
    };
    if (s.n_sp == 4 && s.n_rd == 3 && out4 && A.ndim == 4 && B.ndim == 4 && dim_is(A.dim[0], 0, 1) && dim_is(A.dim[1], 4, 1) &&
        strided(A.dim[2], 2, 5, stride_h) && strided(A.dim[3], 3, 6, stride_w) && dim_is(B.dim[0], 1, 1) && dim_is(B.dim[1], 4, 1) &&
        dim_is(B.dim[2], 5, 1) && dim_is(B.dim[3], 6, 1))
        return kConv2d;
    if (s.n_sp == 4 && s.n_rd == 2 && out4 && A.ndim == 4 && B.ndim == 3 && dim_is(A.dim[0], 0, 1) && dim_is(A.dim[1], 1, 1) &&
        strided(A.dim[2], 2, 4, stride_h) && strided(A.dim[3], 3, 5, stride_w) && dim_is(B.dim[0], 1, 1) && dim_is(B.dim[1], 4, 1) &&
        dim_is(B.dim[2], 5, 1))
        return kDepthwiseConv2d;
    *stride_h = *stride_w = 1;
    return kGeneric;
}

// Upper bound of the footprint of buffer b over any tile: every index expression at its largest.
double footprint_bound(const pruner_subgraph& s, const pruner_buffer& b)
{
    double p = 1;
    for (int d = 0; d < b.ndim; ++d) {
        double e = 1;
        for (int t = 0; t < PRUNER_MAX_TERMS; ++t)
            if (b.dim[d].axis[t] >= 0) e += (double)b.dim[d].coef[t] * (s.extent[b.dim[d].axis[t]] - 1);
        p *= e;
    }
    return p;
}

// Upper bound of blocks * outer steps * block-tile footprint of buffer b over all tilings: an axis the buffer
// does not index contributes its extent (grid or step count); a dimension contributes its terms' extents
// times the sum of its coefficients (G * tile <= extent along every axis).
double traffic_bound(const pruner_subgraph& s, const pruner_buffer& b)
{
    bool used[PRUNER_MAX_AXES] = {false};
    double p = 1;
    for (int d = 0; d < b.ndim; ++d) {
        double csum = 0, e = 1;
        for (int t = 0; t < PRUNER_MAX_TERMS; ++t)
            if (b.dim[d].axis[t] >= 0) {
                csum += b.dim[d].coef[t];
                e *= s.extent[b.dim[d].axis[t]];
                used[b.dim[d].axis[t]] = true;
            }
        p *= (csum > 1 ? csum : 1) * e;
    }
    for (int a = 0; a < s.n_sp + s.n_rd; ++a)
        if (!used[a]) p *= s.extent[a];
    return p;
}

int make_desc(const pruner_subgraph& s, SgDesc* out)
{
    SgDesc d;
    memset(&d, 0, sizeof d);
    if (s.n_sp < 1 || s.n_sp > PRUNER_MAX_SP || s.n_rd < 0 || s.n_rd > PRUNER_MAX_RD) return PRUNER_EINVAL;
    if (s.sp_levels != 4 || (s.rd_levels != 2 && s.rd_levels != 3)) return PRUNER_EINVAL;
    if (s.n_in < 1 || s.n_in > 2 || s.dtype_bytes < 1 || s.dtype_bytes > 16) return PRUNER_EINVAL;
    const pruner_device& h = s.hw;
    if (!(h.T_p > 0) || !(h.T_m > 0) || h.m_l0 < 1 || h.m_l1 < 1 || h.pu_l1 < 1 || h.n_l1 < 1 || h.pu_l2 < 1 || h.n_l2 < 1)
        return PRUNER_EINVAL;
    if (h.pu_l1 > (1 << 20) || h.n_l1 > (1 << 20) || h.pu_l2 > (1 << 20) || h.n_l2 > (1 << 20)) return PRUNER_EINVAL;
    const int n_axes = s.n_sp + s.n_rd;
    for (int a = 0; a < n_axes; ++a)
        if (s.extent[a] < 1 || s.extent[a] > 65535) return PRUNER_EINVAL;
    const bool frag = s.frag[0] != 0 || s.frag[1] != 0 || s.frag[2] != 0;
    if (frag && (s.frag[0] < 1 || s.frag[1] < 1 || s.frag[2] < 1 || s.n_sp < 2 || s.n_rd < 1)) return PRUNER_EINVAL;
    const pruner_buffer* bufs[3] = {&s.in[0], &s.in[1], &s.out};
    for (int b = 0; b < 3; ++b) {
        if (b == 1 && s.n_in < 2) continue;
        if (bufs[b]->ndim < 1 || bufs[b]->ndim > PRUNER_MAX_DIMS) return PRUNER_EINVAL;
        for (int dm = 0; dm < bufs[b]->ndim; ++dm)
            for (int t = 0; t < PRUNER_MAX_TERMS; ++t) {
                const int ax = bufs[b]->dim[dm].axis[t];
                if (ax >= n_axes || ax < -1) return PRUNER_EINVAL;
                if (ax >= 0 && (bufs[b]->dim[dm].coef[t] < 0 || bufs[b]->dim[dm].coef[t] > 65535)) return PRUNER_EINVAL;
            }
    }

    // integer ranges of the kernel: 32-bit symbols, 2^53 for the exact double products
    double prod_sp = 1, prod_all = 1;
    for (int a = 0; a < n_axes; ++a) {
        prod_all *= s.extent[a];
        if (a < s.n_sp) prod_sp *= s.extent[a];
    }
    const double two31 = 2147483648.0, two53 = 9007199254740992.0;
    double fp_sum = 0, traffic_max = 0;
    for (int b = 0; b < s.n_in; ++b) {
        fp_sum += footprint_bound(s, *bufs[b]);
        const double t = traffic_bound(s, *bufs[b]);
        traffic_max = t > traffic_max ? t : traffic_max;
    }
    if (prod_sp * (frag ? h.n_l1 : 1) + h.n_l1 + h.pu_l2 >= two31) return PRUNER_ERANGE;  // S4, S6 and their round-ups
    if (prod_sp + fp_sum + h.n_l1 >= two31) return PRUNER_ERANGE;                          // S1
    if (s.dtype_bytes * fp_sum >= two31) return PRUNER_ERANGE;                             // S3
    if (footprint_bound(s, s.out) + h.n_l2 >= two31) return PRUNER_ERANGE;                 // S7
    if (2.0 * prod_all >= two53 || (double)s.dtype_bytes * traffic_max >= two53) return PRUNER_ERANGE;  // S2, S8, S5

    // magnitudes of the binary32 stage: every divisor, quotient and product must stay between 2^-100 and 2^100,
    // the range in which div_rn is the correctly rounded quotient
    {
        const double lo = 7.888609052210118e-31, hi = 1.2676506002282294e30;  // 2^-100, 2^100
        const double S1max = prod_sp + fp_sum, S3max = (double)s.dtype_bytes * fp_sum;
        const double P0m_min = h.m_l0 < S1max ? h.m_l0 / S1max : 1.0, P1m_min = h.m_l1 < S3max ? h.m_l1 / S3max : 1.0;
        const double frag_min = frag ? 1.0 / ((double)s.frag[0] * s.frag[1] * s.frag[2]) : 1.0;
        const double Up_min = (double)h.T_p / ((double)h.pu_l1 * h.n_l1 * h.pu_l2) * frag_min;
        const double Up_max = (double)h.T_p * (1.0 + 2.0 * prod_all);
        const double Um_min = (double)h.T_m * P0m_min * P1m_min / h.n_l2;
        const double S8 = 2.0 * prod_all, S5max = (double)s.dtype_bytes * traffic_max;
        const double probe[] = {Up_min, Up_max, Um_min, (double)h.T_m, S8 / Up_min, S8 / Up_max, S5max / Um_min,
                                1.0 / (double)h.T_m, S8 / Up_min + 3.0 * S5max / Um_min};
        for (double v : probe)
            if (!(v > lo && v < hi)) return PRUNER_ERANGE;
        // the fused evaluation multiplies numerators and denominators out before it divides: G * T <= extent along
        // every axis bounds S6 * prod T by prod_sp and S2 * S6 * prod T by S8; round-ups add at most their unit
        const double fn = frag ? (double)s.extent[s.n_sp - 2] * s.extent[s.n_sp - 1] * s.extent[n_axes - 1] : 1.0;
        const double fd = frag ? fn * s.frag[0] * s.frag[1] * s.frag[2] : 1.0;
        const double c1 = frag ? (double)h.pu_l1 : (double)h.n_l1 * (h.pu_l1 + 1.0);
        const double num_max = (S1max * prod_sp + S8) * fn, den_max = S1max * (prod_sp + h.pu_l2) * (1.0 + c1) * fd;
        const double w_max = (S1max / h.m_l0 + 1.0) * (S3max / h.m_l1 + 1.0) / (double)h.T_m;
        if (!(num_max < hi) || !(den_max < hi * 1048576.0) || !(3.0 * S5max * h.n_l2 < hi) || !(w_max > lo && w_max < hi))
            return PRUNER_ERANGE;
        if (frag && (s.frag[0] > 4096 || s.frag[1] > 4096 || s.frag[2] > 4096)) return PRUNER_EINVAL;
    }

    d.cls = classify(s, &d.stride_h, &d.stride_w);
    d.n_sp = s.n_sp;
    d.n_rd = s.n_rd;
    d.rd_levels = s.rd_levels;
    d.n_in = s.n_in;
    d.frag_mode = frag ? 1 : 0;
    d.dtype_bytes = (uint32_t)s.dtype_bytes;
    d.n_l1 = (uint32_t)h.n_l1;
    d.T_p = h.T_p;
    d.T_m = h.T_m;
    d.m_l0f = (float)h.m_l0;
    d.m_l1f = (float)h.m_l1;
    d.S8 = 2 * (int64_t)prod_all;
    d.S5out = (int64_t)s.dtype_bytes * (int64_t)prod_sp;
    d.S8f = (float)d.S8;
    d.S5out_f = (float)d.S5out;
    d.bytes_f64 = (double)s.dtype_bytes;
    d.k_c = (float)((double)d.S8 / h.T_p);
    d.inv_m0 = (float)(1.0 / (double)h.m_l0);
    d.inv_m1 = (float)(1.0 / (double)h.m_l1);
    d.inv_Tm = (float)(1.0 / h.T_m);
    d.lanes_f = frag ? 1.0f : (float)h.n_l1;
    if (d.cls == kGemm) {
        d.cA = (double)s.dtype_bytes * s.extent[0] * s.extent[2];
        d.cB = (double)s.dtype_bytes * s.extent[2] * s.extent[1];
    } else if (d.cls == kBatchedGemm) {
        d.cA = (double)s.dtype_bytes * s.extent[0] * s.extent[1] * s.extent[3];
        d.cB = (double)s.dtype_bytes * s.extent[0] * s.extent[3] * s.extent[2];
    }
    {
        double rm = 1;
        for (int b = 0; b < 3; ++b) {
            if (b == 1 && s.n_in < 2) continue;
            const pruner_dim& last = bufs[b]->dim[bufs[b]->ndim - 1];
            double e = 1;
            for (int t = 0; t < PRUNER_MAX_TERMS; ++t)
                if (last.axis[t] >= 0) e += (double)last.coef[t] * (s.extent[last.axis[t]] - 1);
            rm = e > rm ? e : rm;
        }
        d.run_max = rm < 2147483647.0 ? (int32_t)rm : 2147483647;
    }
    {
        const double two24 = 16777216.0;
        d.f32_s2 = prod_sp <= two24 && prod_all / prod_sp <= two24;
        d.cAf = (float)d.cA;
        d.cBf = (float)d.cB;
        d.f32_traffic = d.f32_s2 && (d.cls == kGemm || d.cls == kBatchedGemm) && (double)d.cAf == d.cA && (double)d.cBf == d.cB;
        // S1, S3, grid, thread and reduction products bound every operand the symbol code multiplies
        d.small = prod_sp + fp_sum < two24 && (double)s.dtype_bytes * fp_sum < two24 && prod_all / prod_sp < two24 &&
                  (double)(s.hw.n_l1) * prod_sp < two24;
        d.f32_frag = 0;
        if (frag) {
            auto up = [](double e, double f) { return (double)(int64_t)((e + f - 1) / f) * f; };
            const double ei = up(s.extent[s.n_sp - 2], s.frag[0]), ej = up(s.extent[s.n_sp - 1], s.frag[1]);
            const double ek = up(s.extent[s.n_sp + s.n_rd - 1], s.frag[2]);
            d.f32_frag = ei * ej <= two24 && ek <= two24;
        }
    }
    d.div_n_l1 = make_udiv((uint32_t)h.n_l1);
    d.div_pu_l1 = make_udiv((uint32_t)h.pu_l1);
    d.div_pu_l2 = make_udiv((uint32_t)h.pu_l2);
    d.div_n_l2 = make_udiv((uint32_t)h.n_l2);
    for (int i = 0; i < 3; ++i) d.div_frag[i] = make_udiv(frag ? (uint32_t)s.frag[i] : 1u);
    for (int b = 0; b < 3; ++b) {
        if (b == 1 && s.n_in < 2) continue;
        d.ndim[b] = bufs[b]->ndim;
        for (int dm = 0; dm < PRUNER_MAX_DIMS; ++dm)
            for (int t = 0; t < PRUNER_MAX_TERMS; ++t) {
                const bool used = dm < bufs[b]->ndim && bufs[b]->dim[dm].axis[t] >= 0;
                // the generic kernel keeps spatial extents in e[0..3] and reduction extents in e[4..6]
                const int ax = used ? bufs[b]->dim[dm].axis[t] : -1;
                d.axis[b][dm][t] = (int8_t)(ax < s.n_sp ? ax : PRUNER_MAX_SP + (ax - s.n_sp));
                d.coef[b][dm][t] = used ? bufs[b]->dim[dm].coef[t] : 0;
            }
    }
    *out = d;
    return PRUNER_OK;
}

size_t table_bytes(int32_t n_sg) { return round_up((size_t)n_sg * sizeof(SegEnt), 256) + round_up((size_t)n_sg * sizeof(SgDesc), 256); }

}  // namespace
}  // namespace pruner

namespace pruner {

// Everything pruner_draft_score refuses, without enqueuing anything.
int draft_check(const pruner_subgraph* sg, int32_t n_sg, const int64_t* seg_off, const uint16_t* tiles, int64_t tiles_pitch,
                int32_t flags, const float* score, const int64_t* symbols, const void* workspace, size_t workspace_bytes)
{
    if (!sg || !seg_off || n_sg < 1 || n_sg > PRUNER_MAX_SUBGRAPHS) return PRUNER_EINVAL;
    if (flags & ~(PRUNER_NO_COMPUTE_PENALTY | PRUNER_NO_MEMORY_PENALTY | PRUNER_REFERENCE_ROUNDING | PRUNER_FUSED_ARITHMETIC)) return PRUNER_EINVAL;
    if ((flags & PRUNER_REFERENCE_ROUNDING) && (flags & PRUNER_FUSED_ARITHMETIC)) return PRUNER_EINVAL;
    if (seg_off[0] != 0) return PRUNER_EINVAL;
    for (int32_t s = 0; s < n_sg; ++s)
        if (seg_off[s + 1] < seg_off[s]) return PRUNER_EINVAL;
    const int64_t n = seg_off[n_sg];
    if (tiles_pitch < n || n > ((int64_t)1 << 40)) return PRUNER_EINVAL;
    if (!tiles || !score || !aligned(tiles, 2) || !aligned(score, 4) || (symbols && !aligned(symbols, 8))) return PRUNER_EINVAL;
    if (!workspace || !aligned(workspace, 256)) return PRUNER_EWORKSPACE;
    if (workspace_bytes < table_bytes(n_sg)) return PRUNER_EWORKSPACE;
    for (int32_t s = 0; s < n_sg; ++s) {
        SgDesc d;
        const int rc = make_desc(sg[s], &d);
        if (rc) return rc;
    }
    return PRUNER_OK;
}

// measurement hook (pruner_time_dominant_draft_launch): two events and a host counter, or nulls
void* g_time_start = nullptr;
void* g_time_stop = nullptr;
int64_t* g_time_bytes = nullptr;

int draft_launch(const pruner_subgraph* sg, int32_t n_sg, const int64_t* seg_off, const uint16_t* tiles, int64_t tiles_pitch,
                 int32_t flags, float* score, int64_t* symbols, void* workspace, size_t workspace_bytes, hipStream_t st,
                 uint32_t* first_digit, uint32_t* block_max, int copies, bool* counted, const Upload* also, const MutArgs* mut, bool* mutated)
{
    if (counted) *counted = false;
    if (mutated) *mutated = false;
    if (!sg || !seg_off || n_sg < 1 || n_sg > PRUNER_MAX_SUBGRAPHS) return PRUNER_EINVAL;
    if (flags & ~(PRUNER_NO_COMPUTE_PENALTY | PRUNER_NO_MEMORY_PENALTY | PRUNER_REFERENCE_ROUNDING | PRUNER_FUSED_ARITHMETIC)) return PRUNER_EINVAL;
    if ((flags & PRUNER_REFERENCE_ROUNDING) && (flags & PRUNER_FUSED_ARITHMETIC)) return PRUNER_EINVAL;
    if (seg_off[0] != 0) return PRUNER_EINVAL;
    for (int32_t s = 0; s < n_sg; ++s)
        if (seg_off[s + 1] < seg_off[s]) return PRUNER_EINVAL;
    const int64_t n = seg_off[n_sg];
    if (tiles_pitch < n || n > ((int64_t)1 << 40)) return PRUNER_EINVAL;
    if (!tiles || !score || !aligned(tiles, 2) || !aligned(score, 4) || (symbols && !aligned(symbols, 8))) return PRUNER_EINVAL;
    if (!workspace || !aligned(workspace, 256)) return PRUNER_EWORKSPACE;
    if (workspace_bytes < table_bytes(n_sg)) return PRUNER_EWORKSPACE;

    // descriptors, shared between subgraphs that are byte-for-byte equal
    std::vector<SgDesc> descs;
    std::vector<int> desc_of(n_sg);
    for (int32_t s = 0; s < n_sg; ++s) {
        int found = -1;
        for (int32_t t = 0; t < s && found < 0; ++t)
            if (memcmp(&sg[t], &sg[s], sizeof(pruner_subgraph)) == 0) found = desc_of[t];
        if (found < 0) {
            SgDesc d;
            const int rc = make_desc(sg[s], &d);
            if (rc) return rc;
            found = (int)descs.size();
            descs.push_back(d);
        }
        desc_of[s] = found;
    }
    if (n == 0) {
        if (counted) *counted = first_digit != nullptr;   // nothing to count
        if (also && also->dst) return put_table(also->dst, also->bytes.data(), also->bytes.size(), st, also->zero, also->zero_bytes);
        return PRUNER_OK;
    }

    // widest vector load that keeps every thread's first candidate aligned
    int vec = 4;
    auto fits = [&](int v) {
        if (tiles_pitch % v || !aligned(tiles, 2 * (size_t)v) || !aligned(score, 4 * (size_t)v)) return false;
        for (int32_t s = 0; s < n_sg; ++s)
            if (seg_off[s] % v) return false;
        return true;
    };
    while (vec > 1 && !fits(vec)) vec >>= 1;

    // Launch plan.  Large populations at the full load width: one launch per loop-nest class present, the table
    // grouped by class; otherwise a single launch of the kernel that branches on the class.  A launch has at most
    // as many workgroups as the device holds at once; they walk through the chunks of their segment.
    struct Launch { int cls; int32_t first_seg, n_seg; int64_t blocks, chunks; DraftFn fn; };
    std::vector<Launch> plan;
    std::vector<int32_t> order(n_sg);
    for (int32_t s = 0; s < n_sg; ++s) order[s] = s;
    const bool by_class = vec == 4 && n >= kPerClassMin;
    if (by_class)
        std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return descs[desc_of[a]].cls < descs[desc_of[b]].cls; });
    // Arithmetic of Eq. 1: one rounded operation per step of the definitions wherever the call is a single launch (below
    // 2^20 candidates a call is bound by launch latency, and the dozen divisions per candidate cost nothing measurable),
    // the multiplied-out form in the per-class launches of large populations, unless a flag asks for one of them.
    const bool exact = (flags & PRUNER_REFERENCE_ROUNDING) != 0 || (!(flags & PRUNER_FUSED_ARITHMETIC) && !by_class);
    const bool hist = first_digit != nullptr && vec == 4 && symbols == nullptr && copies >= 1;
    const bool fused = mut != nullptr && by_class && hist;   // every launch of the plan then makes its candidates itself
    const int64_t chunk = (int64_t)kBlock * vec;
    for (int32_t i = 0; i < n_sg; ++i) {
        const int cls = by_class ? descs[desc_of[order[i]]].cls : kAnyClass;
        if (plan.empty() || plan.back().cls != cls) plan.push_back(Launch{cls, i, 0, 0, 0, pick_kernel(cls, vec, symbols != nullptr, exact, hist, fused)});
        const int64_t len = seg_off[order[i] + 1] - seg_off[order[i]];
        plan.back().chunks += (len + chunk - 1) / chunk;
        plan.back().n_seg += 1;
    }
    std::vector<SegEnt> segs(n_sg);
    for (Launch& L : plan) {
        const int64_t room = resident_blocks(L.fn);
        const int64_t depth = (L.chunks + room - 1) / room;   // chunks per workgroup when the launch fills the device once
        for (int32_t i = L.first_seg; i < L.first_seg + L.n_seg; ++i) {
            const int32_t s = order[i];
            const SgDesc& dd = descs[desc_of[s]];
            const int64_t chunks = (seg_off[s + 1] - seg_off[s] + chunk - 1) / chunk;
            const int64_t iters = depth < 1 ? 1 : depth;
            const int64_t blocks = (chunks + iters - 1) / iters;
            if (blocks > 0x7FFFFFFF || iters > 0x7FFFFFFF || L.blocks + blocks > 0x7FFFFFFF) return PRUNER_EINVAL;
            const bool tab = dd.run_max <= kTabMax && 2 * ((int64_t)dd.run_max + 1) <= 3 * chunk * iters && !(flags & PRUNER_NO_MEMORY_PENALTY);
            segs[i] = SegEnt{seg_off[s], seg_off[s + 1], (int32_t)L.blocks, desc_of[s], (int32_t)blocks, (int32_t)iters, tab ? 1 : 0, s};
            L.blocks += blocks;
        }
    }

    char* ws = static_cast<char*>(workspace);
    SegEnt* d_segs = reinterpret_cast<SegEnt*>(ws);
    SgDesc* d_descs = reinterpret_cast<SgDesc*>(ws + round_up((size_t)n_sg * sizeof(SegEnt), 256));
    // both tables travel in one launch: the workspace image is assembled on the host
    const size_t descs_at = round_up((size_t)n_sg * sizeof(SegEnt), 256);
    std::vector<char> image(descs_at + descs.size() * sizeof(SgDesc), 0);
    memcpy(image.data(), segs.data(), segs.size() * sizeof(SegEnt));
    memcpy(image.data() + descs_at, descs.data(), descs.size() * sizeof(SgDesc));
    void* zero = nullptr;
    size_t zero_bytes = 0;
    bool apart = false;
    if (also && also->dst) {
        // the other table rides along in the same launch if it starts shortly behind this call's tables (with many
        // subgraphs that share descriptors the reserved room is much larger than the tables: then it travels by itself)
        const ptrdiff_t at = static_cast<const char*>(also->dst) - ws;
        if (at < (ptrdiff_t)image.size()) return PRUNER_EINVAL;
        if (at <= (ptrdiff_t)image.size() + 4096) {
            image.resize((size_t)at, 0);
            image.insert(image.end(), also->bytes.begin(), also->bytes.end());
            zero = also->zero;
            zero_bytes = also->zero_bytes;
        } else {
            apart = true;
        }
    }
    int rc = put_table(ws, image.data(), image.size(), st, zero, zero_bytes);
    if (rc) return rc;
    if (apart) {
        rc = put_table(also->dst, also->bytes.data(), also->bytes.size(), st, also->zero, also->zero_bytes);
        if (rc) return rc;
    }

    // measurement hook: events around the launch that covers the most candidates
    const Launch* timed = nullptr;
    int64_t timed_candidates = -1, timed_bytes = 0;
    if (g_time_start && g_time_stop) {
        for (const Launch& L : plan) {
            if (L.blocks == 0) continue;
            int64_t cands = 0, bytes = 0;
            for (int32_t i = L.first_seg; i < L.first_seg + L.n_seg; ++i) {
                const int32_t sub = order[i];
                const int64_t len = seg_off[sub + 1] - seg_off[sub];
                cands += len;
                bytes += len * (2 * (int64_t)(sg[sub].n_sp * 4 + sg[sub].n_rd * sg[sub].rd_levels) + 4);
            }
            if (cands > timed_candidates) timed = &L, timed_candidates = cands, timed_bytes = bytes;
        }
        if (g_time_bytes) *g_time_bytes = timed ? timed_bytes : 0;
    }
    for (const Launch& L : plan) {
        if (L.blocks == 0) continue;
        if (&L == timed && hipEventRecord(static_cast<hipEvent_t>(g_time_start), st) != hipSuccess) return PRUNER_EHIP;
        hipLaunchKernelGGL(L.fn, dim3((unsigned)L.blocks), dim3(kBlock), 0, st, d_segs + L.first_seg, L.n_seg, d_descs, tiles, tiles_pitch,
                           flags, score, symbols, n, first_digit, block_max, copies, n_sg, fused ? *mut : MutArgs{});
        if (&L == timed && hipEventRecord(static_cast<hipEvent_t>(g_time_stop), st) != hipSuccess) return PRUNER_EHIP;
        PRUNER_LAUNCH_CHECK();
    }
    if (counted) *counted = hist;
    if (mutated) *mutated = fused;
    return PRUNER_OK;
}

bool draft_launches_by_class(int64_t n) { return n >= kPerClassMin; }

}  // namespace pruner

using namespace pruner;

extern "C" int pruner_draft_score(const pruner_subgraph* sg, int32_t n_sg, const int64_t* seg_off, const uint16_t* tiles,
                                  int64_t tiles_pitch, int32_t flags, float* score, int64_t* symbols, void* workspace,
                                  size_t workspace_bytes, void* stream)
{
    return draft_launch(sg, n_sg, seg_off, tiles, tiles_pitch, flags, score, symbols, workspace, workspace_bytes,
                        static_cast<hipStream_t>(stream), nullptr, nullptr, 0, nullptr);
}

extern "C" int pruner_time_dominant_draft_launch(void* start_event, void* stop_event, int64_t* algorithmic_bytes)
{
    if ((start_event == nullptr) != (stop_event == nullptr)) return PRUNER_EINVAL;
    g_time_start = start_event;
    g_time_stop = stop_event;
    g_time_bytes = start_event ? algorithmic_bytes : nullptr;
    return PRUNER_OK;
}

namespace pruner {
size_t draft_workspace_bytes(int32_t n_sg) { return table_bytes(n_sg < 1 ? 1 : n_sg); }
}
