// Draft model: Symbol-based Analyzer over a population of candidate schedules (Alg. 2, C_SA and the loop over S_x).
//
// One thread scores VEC neighbouring candidates.  Tile factors arrive structure-of-arrays (one uint16 row per
// split level), so a wavefront reads 64*VEC consecutive uint16 of every row; everything else stays in registers.
// Per-subgraph constants (device abstraction, loop-nest class, division magics) sit in a small table that all
// lanes of a block read through the scalar cache; a block never straddles two subgraphs.
//
// Arithmetic contract (this file is compiled with -ffp-contract=off and correctly rounded division):
//   symbols are exact integers (Table 2);
//   penalties, utilisation and latency (Sec. 4.1 "Hardware-aware Penalty", Eq. 1) are binary32, one IEEE
//   operation per step, in this order:
//     P0m = min(m_l0 / S1, 1)          P0c = 1 + S2 / S1            P1m = min(m_l1 / S3, 1)
//     sch = ceil(S4 / n_l1)            P1c = sch / (ceil(sch / pu_l1) * pu_l1)
//     alpha = S4 / (sch * n_l1)        P2c = S6 / (ceil(S6 / pu_l2) * pu_l2)
//     Up  = (((T_p * P0c) * P1c) * alpha) * P2c   [ * Ptc in fragment mode ]
//     L   = S8 / Up
//     for each memory statement In_0, In_1, store:
//         P2m = S7 / (ceil(S7 / n_l2) * n_l2);  Um = ((T_m * P0m) * P1m) * P2m;  L = L + S5 / Um
//     score = -L
//   integer-to-float conversions round to nearest even.
#include "common.h"

#include <string.h>

#include <vector>

namespace pruner {
namespace {

constexpr int kBlock = 256;

enum NestClass : int32_t { kGeneric = 0, kGemm = 1, kBatchedGemm = 2, kConv2d = 3, kDepthwiseConv2d = 4 };

// Unsigned division by a run-time constant with one multiply-high (Granlund & Montgomery, "Division by invariant
// integers using multiplication", PLDI 1994, Fig. 4.1): for 2 <= d < 2^31, L = ceil(log2 d),
// m = floor(2^32 (2^L - d) / d) + 1, sh = L - 1:  floor(x / d) = (((x - mulhi(m, x)) >> 1) + mulhi(m, x)) >> sh
// for every 32-bit x.  d = 1 is flagged.
struct UDiv {
    uint32_t d, m, sh, one;
};

UDiv make_udiv(uint32_t d)
{
    UDiv u{d, 0, 0, d == 1 ? 1u : 0u};
    if (d >= 2) {
        uint32_t L = 0;
        while ((1ull << L) < d) ++L;
        u.m = (uint32_t)((((1ull << L) - d) << 32) / d + 1);
        u.sh = L - 1;
    }
    return u;
}

__device__ __forceinline__ uint32_t udiv(uint32_t x, const UDiv& u)
{
    const uint32_t q = __umulhi(u.m, x);
    const uint32_t t = (((x - q) >> 1) + q) >> u.sh;
    return u.one ? x : t;
}
__device__ __forceinline__ uint32_t cdiv(uint32_t x, const UDiv& u) { return udiv(x + u.d - 1, u); }

// Per-subgraph constants, read by all lanes of a block at the same address.
struct alignas(16) SgDesc {
    int32_t cls, n_sp, n_rd, rd_levels;
    int32_t n_in, frag_mode;
    uint32_t dtype_bytes, n_l1;
    float T_p, T_m, m_l0f, m_l1f;
    float S8f, S5out_f;
    int32_t stride_h, stride_w;  // conv classes: coefficient of the output row / column in the image index
    int64_t S8, S5out;
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
};

// ---- loop-nest classes: footprints of the operand tiles over per-axis tile extents e[] --------------------------
// e[a] is the tile extent of axis a (spatial axes first).  fp0/fp1: elements of In_0 / In_1 touched; run0/run1/
// runo: extent of the innermost (contiguous) dimension of the In_0 / In_1 / output tile.

struct NestGemm {  // C[i,j] += A[i,k] B[k,j]; axes i j | k
    static constexpr int NSP = 2, NRD = 1;
    static constexpr bool FIXED = true;
    __device__ static uint32_t fp0(const uint32_t* e, const SgDesc&) { return e[0] * e[2]; }
    __device__ static uint32_t fp1(const uint32_t* e, const SgDesc&) { return e[2] * e[1]; }
    __device__ static uint32_t run0(const uint32_t* e, const SgDesc&) { return e[2]; }
    __device__ static uint32_t run1(const uint32_t* e, const SgDesc&) { return e[1]; }
    __device__ static uint32_t runo(const uint32_t* e, const SgDesc&) { return e[1]; }
};

struct NestBatchedGemm {  // C[b,i,j] += A[b,i,k] B[b,k,j]; axes b i j | k
    static constexpr int NSP = 3, NRD = 1;
    static constexpr bool FIXED = true;
    __device__ static uint32_t fp0(const uint32_t* e, const SgDesc&) { return e[0] * e[1] * e[3]; }
    __device__ static uint32_t fp1(const uint32_t* e, const SgDesc&) { return e[0] * e[3] * e[2]; }
    __device__ static uint32_t run0(const uint32_t* e, const SgDesc&) { return e[3]; }
    __device__ static uint32_t run1(const uint32_t* e, const SgDesc&) { return e[2]; }
    __device__ static uint32_t runo(const uint32_t* e, const SgDesc&) { return e[2]; }
};

struct NestConv2d {  // O[n,k,h,w] += I[n,c,h*sh+r,w*sw+s] W[k,c,r,s]; axes n k h w | c r s
    static constexpr int NSP = 4, NRD = 3;
    static constexpr bool FIXED = true;
    __device__ static uint32_t rows(const uint32_t* e, const SgDesc& d) { return (e[2] - 1) * (uint32_t)d.stride_h + e[5]; }
    __device__ static uint32_t cols(const uint32_t* e, const SgDesc& d) { return (e[3] - 1) * (uint32_t)d.stride_w + e[6]; }
    __device__ static uint32_t fp0(const uint32_t* e, const SgDesc& d) { return e[0] * e[4] * rows(e, d) * cols(e, d); }
    __device__ static uint32_t fp1(const uint32_t* e, const SgDesc&) { return e[1] * e[4] * e[5] * e[6]; }
    __device__ static uint32_t run0(const uint32_t* e, const SgDesc& d) { return cols(e, d); }
    __device__ static uint32_t run1(const uint32_t* e, const SgDesc&) { return e[6]; }
    __device__ static uint32_t runo(const uint32_t* e, const SgDesc&) { return e[3]; }
};

struct NestDepthwiseConv2d {  // O[n,c,h,w] += I[n,c,h*sh+r,w*sw+s] W[c,r,s]; axes n c h w | r s
    static constexpr int NSP = 4, NRD = 2;
    static constexpr bool FIXED = true;
    __device__ static uint32_t rows(const uint32_t* e, const SgDesc& d) { return (e[2] - 1) * (uint32_t)d.stride_h + e[4]; }
    __device__ static uint32_t cols(const uint32_t* e, const SgDesc& d) { return (e[3] - 1) * (uint32_t)d.stride_w + e[5]; }
    __device__ static uint32_t fp0(const uint32_t* e, const SgDesc& d) { return e[0] * e[1] * rows(e, d) * cols(e, d); }
    __device__ static uint32_t fp1(const uint32_t* e, const SgDesc&) { return e[1] * e[4] * e[5]; }
    __device__ static uint32_t run0(const uint32_t* e, const SgDesc& d) { return cols(e, d); }
    __device__ static uint32_t run1(const uint32_t* e, const SgDesc&) { return e[5]; }
    __device__ static uint32_t runo(const uint32_t* e, const SgDesc&) { return e[3]; }
};

// Any affine nest, from the access tables.  Axes beyond n_sp / n_rd carry extent 1, so they drop out.
struct NestGeneric {
    static constexpr int NSP = PRUNER_MAX_SP, NRD = PRUNER_MAX_RD;
    static constexpr bool FIXED = false;
    __device__ static uint32_t pick(const uint32_t* e, int axis)
    {
        uint32_t v = e[0];
#pragma unroll
        for (int a = 1; a < PRUNER_MAX_AXES; ++a) v = axis == a ? e[a] : v;
        return v;
    }
    __device__ static uint32_t ext(const uint32_t* e, const SgDesc& d, int b, int dim)
    {
        uint32_t x = 1;
#pragma unroll
        for (int t = 0; t < PRUNER_MAX_TERMS; ++t) {
            const int axis = d.axis[b][dim][t];
            if (axis >= 0) x += (uint32_t)d.coef[b][dim][t] * (pick(e, axis) - 1);
        }
        return x;
    }
    __device__ static uint32_t fp(const uint32_t* e, const SgDesc& d, int b)
    {
        uint32_t p = 1;
#pragma unroll
        for (int dim = 0; dim < PRUNER_MAX_DIMS; ++dim)
            if (dim < d.ndim[b]) p *= ext(e, d, b, dim);
        return p;
    }
    __device__ static uint32_t run(const uint32_t* e, const SgDesc& d, int b)
    {
        uint32_t r = 1;
#pragma unroll
        for (int dim = 0; dim < PRUNER_MAX_DIMS; ++dim)
            if (dim == d.ndim[b] - 1) r = ext(e, d, b, dim);
        return r;
    }
    __device__ static uint32_t fp0(const uint32_t* e, const SgDesc& d) { return fp(e, d, 0); }
    __device__ static uint32_t fp1(const uint32_t* e, const SgDesc& d) { return d.n_in > 1 ? fp(e, d, 1) : 0u; }
    __device__ static uint32_t run0(const uint32_t* e, const SgDesc& d) { return run(e, d, 0); }
    __device__ static uint32_t run1(const uint32_t* e, const SgDesc& d) { return d.n_in > 1 ? run(e, d, 1) : 1u; }
    __device__ static uint32_t runo(const uint32_t* e, const SgDesc& d) { return run(e, d, 2); }
};

template <int VEC> struct VecLoad;
template <> struct VecLoad<1> {
    __device__ static void load(const uint16_t* p, uint32_t* out) { out[0] = *p; }
};
template <> struct VecLoad<2> {
    __device__ static void load(const uint16_t* p, uint32_t* out)
    {
        const uint32_t w = *reinterpret_cast<const uint32_t*>(p);
        out[0] = w & 0xFFFFu;
        out[1] = w >> 16;
    }
};
template <> struct VecLoad<4> {
    __device__ static void load(const uint16_t* p, uint32_t* out)
    {
        const uint2 w = *reinterpret_cast<const uint2*>(p);
        out[0] = w.x & 0xFFFFu;
        out[1] = w.x >> 16;
        out[2] = w.y & 0xFFFFu;
        out[3] = w.y >> 16;
    }
};

struct Symbols {
    uint32_t S1, S3, S4, S6;
    double S2;        // exact: can pass 2^32
    double S5[2];     // exact: products below 2^53 (checked on the host)
    uint32_t S7[3];
    double frag_num, frag_den;
};

// Penalties, utilisation, latency: the binary32 sequence of the header comment.
__device__ __forceinline__ float analyze(const SgDesc& d, const Symbols& y, int32_t flags)
{
    const float S1f = (float)y.S1;
    const float P0m = fminf(d.m_l0f / S1f, 1.0f);
    const float P0c = 1.0f + (float)y.S2 / S1f;
    const float P1m = fminf(d.m_l1f / (float)y.S3, 1.0f);
    const uint32_t sch = cdiv(y.S4, d.div_n_l1);
    const float P1c = (float)sch / (float)(cdiv(sch, d.div_pu_l1) * d.div_pu_l1.d);
    const float alpha = (float)y.S4 / (float)(sch * d.n_l1);
    const float P2c = (float)y.S6 / (float)(cdiv(y.S6, d.div_pu_l2) * d.div_pu_l2.d);

    float Up = d.T_p;
    if (!(flags & PRUNER_NO_COMPUTE_PENALTY)) {
        Up = (((Up * P0c) * P1c) * alpha) * P2c;
        if (d.frag_mode) Up = Up * ((float)y.frag_num / (float)y.frag_den);
    }
    float L = d.S8f / Up;

    const float Tm0 = (d.T_m * P0m) * P1m;
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        if (s == 1 && d.n_in < 2) continue;
        const float S5f = s < 2 ? (float)y.S5[s] : d.S5out_f;
        float Um = d.T_m;
        if (!(flags & PRUNER_NO_MEMORY_PENALTY)) {
            const float P2m = (float)y.S7[s] / (float)(cdiv(y.S7[s], d.div_n_l2) * d.div_n_l2.d);
            Um = Tm0 * P2m;
        }
        L = L + S5f / Um;
    }
    return -L;
}

template <class Nest, int VEC, bool DUMP>
__device__ __forceinline__ void score_candidates(const SgDesc& d, const uint16_t* __restrict__ tiles, int64_t pitch,
                                                 int64_t c0, int64_t c_end, int32_t flags, float* __restrict__ score,
                                                 int64_t* __restrict__ symbols, int64_t n_total)
{
    constexpr int NSP = Nest::NSP, NRD = Nest::NRD;
    uint32_t sp[NSP][4][VEC];   // grid, virtual thread, thread, inner
    uint32_t rd[NRD][3][VEC];   // outer steps, middle, inner (inner = 1 with two levels)

    const uint16_t* col = tiles + c0;
#pragma unroll
    for (int a = 0; a < NSP; ++a) {
#pragma unroll
        for (int l = 0; l < 4; ++l) {
            if (Nest::FIXED || a < d.n_sp) {
                VecLoad<VEC>::load(col + (int64_t)(a * 4 + l) * pitch, sp[a][l]);
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
                VecLoad<VEC>::load(col + (int64_t)((Nest::FIXED ? NSP : d.n_sp) * 4 + r * rdl + l) * pitch, rd[r][l]);
            } else {
#pragma unroll
                for (int v = 0; v < VEC; ++v) rd[r][l][v] = 1;
            }
        }
    }

    float out[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        uint32_t e_blk[NSP + NRD], e_reg[NSP + NRD];
        uint32_t prod_R = 1, prod_T = 1, prod_G = 1, prod_q = 1, prod_O = 1;
#pragma unroll
        for (int a = 0; a < NSP; ++a) {
            const uint32_t G = sp[a][0][v], V = sp[a][1][v], T = sp[a][2][v], I = sp[a][3][v];
            e_reg[a] = V * I;          // thread tile R_a
            e_blk[a] = e_reg[a] * T;   // block tile  B_a
            prod_R *= e_reg[a];
            prod_T *= T;
            prod_G *= G;
        }
#pragma unroll
        for (int r = 0; r < NRD; ++r) {
            const uint32_t O = rd[r][0][v], mid = rd[r][1][v], q = rd[r][2][v];
            e_reg[NSP + r] = q;          // register step q_r
            e_blk[NSP + r] = mid * q;    // shared-tile depth D_r
            prod_q *= q;
            prod_O *= O;
        }

        Symbols y;
        const uint32_t fpb0 = Nest::fp0(e_blk, d), fpb1 = Nest::fp1(e_blk, d);
        y.S1 = prod_R + Nest::fp0(e_reg, d) + Nest::fp1(e_reg, d);
        y.S2 = 2.0 * ((double)prod_R * (double)prod_q);
        y.S3 = d.dtype_bytes * (fpb0 + fpb1);
        y.S4 = prod_T;
        y.S6 = prod_G;
        if (d.frag_mode) {
            y.S4 = d.n_l1 * prod_T;
            y.S1 = cdiv(y.S1, d.div_n_l1);
            const uint32_t Ii = sp[NSP >= 2 ? NSP - 2 : 0][3][v], Ij = sp[NSP - 1][3][v], qk = rd[NRD - 1][2][v];
            // NestGeneric carries absent axes as trailing 1s, so pick by the real axis counts there
            uint32_t fi = Ii, fj = Ij, fk = qk;
            if constexpr (!Nest::FIXED) {
                fi = 1, fj = 1, fk = 1;
#pragma unroll
                for (int a = 0; a < NSP; ++a) {
                    if (a == d.n_sp - 2) fi = sp[a][3][v];
                    if (a == d.n_sp - 1) fj = sp[a][3][v];
                }
#pragma unroll
                for (int r = 0; r < NRD; ++r)
                    if (r == d.n_rd - 1) fk = rd[r][2][v];
            }
            y.frag_num = ((double)fi * (double)fj) * (double)fk;
            y.frag_den = ((double)(cdiv(fi, d.div_frag[0]) * d.div_frag[0].d) * (double)(cdiv(fj, d.div_frag[1]) * d.div_frag[1].d)) *
                         (double)(cdiv(fk, d.div_frag[2]) * d.div_frag[2].d);
        } else {
            y.frag_num = 1.0;
            y.frag_den = 1.0;
        }
        // S5 of a load: dtype_bytes * blocks * outer reduction steps * block-tile footprint
        const double reads = (double)d.dtype_bytes * ((double)prod_G * (double)prod_O);
        y.S5[0] = reads * (double)fpb0;
        y.S5[1] = reads * (double)fpb1;
        y.S7[0] = Nest::run0(e_blk, d);
        y.S7[1] = Nest::run1(e_blk, d);
        y.S7[2] = Nest::runo(e_blk, d);

        out[v] = analyze(d, y, flags);

        if constexpr (DUMP) {
            const int64_t c = c0 + v;
            if (c < c_end) {
                symbols[PRUNER_SYM_S1 * n_total + c] = y.S1;
                symbols[PRUNER_SYM_S2 * n_total + c] = (int64_t)y.S2;
                symbols[PRUNER_SYM_S3 * n_total + c] = y.S3;
                symbols[PRUNER_SYM_S4 * n_total + c] = y.S4;
                symbols[PRUNER_SYM_S6 * n_total + c] = y.S6;
                symbols[PRUNER_SYM_S8 * n_total + c] = d.S8;
                symbols[PRUNER_SYM_S5_IN0 * n_total + c] = (int64_t)y.S5[0];
                symbols[PRUNER_SYM_S7_IN0 * n_total + c] = y.S7[0];
                symbols[PRUNER_SYM_S5_IN1 * n_total + c] = d.n_in > 1 ? (int64_t)y.S5[1] : 0;
                symbols[PRUNER_SYM_S7_IN1 * n_total + c] = d.n_in > 1 ? y.S7[1] : 0;
                symbols[PRUNER_SYM_S5_OUT * n_total + c] = d.S5out;
                symbols[PRUNER_SYM_S7_OUT * n_total + c] = y.S7[2];
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

template <int VEC, bool DUMP>
__global__ void __launch_bounds__(kBlock) draft_kernel(const SegEnt* __restrict__ segs, int32_t n_seg,
                                                       const SgDesc* __restrict__ descs, const uint16_t* __restrict__ tiles,
                                                       int64_t pitch, int32_t flags, float* __restrict__ score,
                                                       int64_t* __restrict__ symbols, int64_t n_total)
{
    // the segment of this block: last entry whose first block is not after this one (empty segments share a
    // first block with their successor and are never picked)
    const int32_t b = blockIdx.x;
    int lo = 0, hi = n_seg - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (segs[mid].first_block <= b) lo = mid; else hi = mid - 1;
    }
    const SegEnt seg = segs[lo];
    const SgDesc& d = descs[seg.desc];
    const int64_t c0 = seg.begin + ((int64_t)(b - seg.first_block) * kBlock + threadIdx.x) * VEC;
    if (c0 >= seg.end) return;

    switch (d.cls) {
        case kGemm: score_candidates<NestGemm, VEC, DUMP>(d, tiles, pitch, c0, seg.end, flags, score, symbols, n_total); break;
        case kBatchedGemm: score_candidates<NestBatchedGemm, VEC, DUMP>(d, tiles, pitch, c0, seg.end, flags, score, symbols, n_total); break;
        case kConv2d: score_candidates<NestConv2d, VEC, DUMP>(d, tiles, pitch, c0, seg.end, flags, score, symbols, n_total); break;
        case kDepthwiseConv2d: score_candidates<NestDepthwiseConv2d, VEC, DUMP>(d, tiles, pitch, c0, seg.end, flags, score, symbols, n_total); break;
        default: score_candidates<NestGeneric, VEC, DUMP>(d, tiles, pitch, c0, seg.end, flags, score, symbols, n_total); break;
    }
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

using namespace pruner;

extern "C" int pruner_draft_score(const pruner_subgraph* sg, int32_t n_sg, const int64_t* seg_off, const uint16_t* tiles,
                                  int64_t tiles_pitch, int32_t flags, float* score, int64_t* symbols, void* workspace,
                                  size_t workspace_bytes, void* stream)
{
    if (!sg || !seg_off || n_sg < 1 || n_sg > PRUNER_MAX_SUBGRAPHS) return PRUNER_EINVAL;
    if (flags & ~(PRUNER_NO_COMPUTE_PENALTY | PRUNER_NO_MEMORY_PENALTY)) return PRUNER_EINVAL;
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
    if (n == 0) return PRUNER_OK;

    // widest vector load that keeps every thread's first candidate aligned
    int vec = 4;
    auto fits = [&](int v) {
        if (tiles_pitch % v || !aligned(tiles, 2 * (size_t)v) || !aligned(score, 4 * (size_t)v)) return false;
        for (int32_t s = 0; s < n_sg; ++s)
            if (seg_off[s] % v) return false;
        return true;
    };
    while (vec > 1 && !fits(vec)) vec >>= 1;

    std::vector<SegEnt> segs(n_sg);
    int64_t blocks = 0;
    for (int32_t s = 0; s < n_sg; ++s) {
        segs[s] = SegEnt{seg_off[s], seg_off[s + 1], (int32_t)blocks, desc_of[s]};
        blocks += (seg_off[s + 1] - seg_off[s] + (int64_t)kBlock * vec - 1) / ((int64_t)kBlock * vec);
        if (blocks > 0x7FFFFFFF) return PRUNER_EINVAL;
    }

    hipStream_t st = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    SegEnt* d_segs = reinterpret_cast<SegEnt*>(ws);
    SgDesc* d_descs = reinterpret_cast<SgDesc*>(ws + round_up((size_t)n_sg * sizeof(SegEnt), 256));
    int rc = put_table(d_segs, segs.data(), segs.size() * sizeof(SegEnt), st);
    if (rc) return rc;
    rc = put_table(d_descs, descs.data(), descs.size() * sizeof(SgDesc), st);
    if (rc) return rc;

    const dim3 grid((unsigned)blocks), block(kBlock);
#define PRUNER_DRAFT_LAUNCH(V, D) \
    hipLaunchKernelGGL((draft_kernel<V, D>), grid, block, 0, st, d_segs, n_sg, d_descs, tiles, tiles_pitch, flags, score, symbols, n)
    if (symbols) {
        if (vec == 4) PRUNER_DRAFT_LAUNCH(4, true); else if (vec == 2) PRUNER_DRAFT_LAUNCH(2, true); else PRUNER_DRAFT_LAUNCH(1, true);
    } else {
        if (vec == 4) PRUNER_DRAFT_LAUNCH(4, false); else if (vec == 2) PRUNER_DRAFT_LAUNCH(2, false); else PRUNER_DRAFT_LAUNCH(1, false);
    }
#undef PRUNER_DRAFT_LAUNCH
    PRUNER_LAUNCH_CHECK();
    return PRUNER_OK;
}

namespace pruner {
size_t draft_workspace_bytes(int32_t n_sg) { return table_bytes(n_sg < 1 ? 1 : n_sg); }
}
