// Verify stage: statement-feature branch of the learned cost model on the drafted candidates
// (Sec. 4.2, "Pattern-aware Transformer": statement features -> linear layers -> summation over statements).
//
//   y(c,s)   = w3 . relu(W2 relu(W1 x(c,s) + b1) + b2) + b3          164 -> 256 -> 256 -> 1
//   vscore_c = sum over s < n_stmt[c] of y(c,s)
//
// The valid statement rows of all candidates get consecutive row numbers (exclusive scan of n_stmt), so the matrix
// cores never see padding rows.  Up to 16383 candidates (drafted sets are a few thousand) the scan is done by every
// workgroup of mlp_kernel itself, in LDS, while its weights arrive: one launch, no workspace traffic, and tiles that
// begin and end on candidate boundaries, so every candidate is summed and stored by exactly one thread.  Beyond that:
//   rows kernels   the scan as two launches of their own (chunk totals, then one workgroup per chunk of 8192
//                  candidates), writing a table of source rows; clears vscore.
//   mlp_kernel     persistent workgroups (one per CU, 4 wavefronts).  Wavefront w owns hidden units
//                  [64w, 64w+64) of both layers and keeps its slices of W1 and W2 in registers for the whole
//                  launch (they pass through LDS once, so that HBM/L2 sees contiguous reads); feature rows stream
//                  through LDS 64 at a time as bfloat16, the next tile's rows being fetched while the current tile
//                  is computed.  Layers are computed transposed (H^T = W X^T) with v_mfma_f32_32x32x16_bf16, so
//                  that one lane holds 16 hidden units of ONE row: bias is the accumulator's initial value, ReLU
//                  and the bfloat16 rounding are lane-local, and the last layer's dot product with w3 is a
//                  lane-local sum plus one cross-lane add.  Hidden activations never leave the CU.  The rows of a
//                  candidate are added pairwise inside a tile; with the row table a candidate whose rows
//                  straddle two tiles receives two atomic adds onto zero, which commute.
#include "common.h"

namespace pruner {
namespace {

constexpr int kF = PRUNER_FEAT_DIM;   // 164
constexpr int kS = PRUNER_MAX_STMT;   // 8
constexpr int kH = PRUNER_HIDDEN;     // 256
constexpr int kTM = 64;               // rows per tile
constexpr int kK1 = 176;              // 164 padded to a multiple of the MFMA depth 16
constexpr int kXs = kK1 + 8;          // LDS row strides in bfloat16 elements (rows stay 16-byte aligned)
constexpr int kHs = kH + 8;
constexpr int kThreads = 256;
constexpr int kF4 = kF / 4;           // float4 per feature row (41)
constexpr int kXLoads = (kTM * kF4 + kThreads - 1) / kThreads;   // float4 a thread fetches per tile (11)
constexpr int kNominal = kTM - (kS - 1);   // in-kernel scan: tile t begins at the first candidate whose rows start at or after 57 t,
                                           // and therefore holds at most 57 + 7 = 64 rows
constexpr int kFusedMax = 16383;           // candidates whose row numbers fit in LDS next to the tile buffers

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct Head {
    int32_t n_rows;   // valid statement rows in total
    int32_t pad[3];
};

// ---- rows kernels: compact numbering of the valid rows (sets too large for the in-kernel numbering) --------------
// One workgroup per chunk of 8192 candidates.  rows_total_kernel leaves every chunk's row count; rows_kernel adds up
// the counts of the chunks before its own, scans its chunk (counts read coalesced; thread t owns candidates
// [8t, 8t+8) of the chunk and leaves each candidate's first row number in LDS) and writes the row table by
// (candidate, statement) pairs, so that neighbouring threads write neighbouring rows.

constexpr int kRowsChunk = 8192;
constexpr int kRowsPer = kRowsChunk / 1024;

__device__ __forceinline__ int32_t clamp_stmt(int32_t v) { return v < 0 ? 0 : v > kS ? kS : v; }

// sum over the workgroup (1024 threads); wave_tot: 16 LDS words; all threads call and receive the sum
__device__ __forceinline__ int32_t block_sum_1024(int32_t v, int32_t* wave_tot)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    __syncthreads();   // wave_tot may still be read from an earlier call
    if ((threadIdx.x & 63) == 0) wave_tot[threadIdx.x >> 6] = v;
    __syncthreads();
    int32_t all = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) all += wave_tot[w];
    return all;
}

__global__ void __launch_bounds__(1024) rows_total_kernel(const int32_t* __restrict__ n_stmt, int64_t n_d, int32_t* __restrict__ chunk_rows)
{
    __shared__ int32_t wave_tot[16];
    const int64_t base = (int64_t)blockIdx.x * kRowsChunk;
    int32_t mine = 0;
#pragma unroll
    for (int j = 0; j < kRowsPer; ++j) {
        const int64_t c = base + j * 1024 + threadIdx.x;
        mine += c < n_d ? clamp_stmt(n_stmt[c]) : 0;
    }
    const int32_t all = block_sum_1024(mine, wave_tot);
    if (threadIdx.x == 0) chunk_rows[blockIdx.x] = all;
}

__global__ void __launch_bounds__(1024) rows_kernel(const int32_t* __restrict__ n_stmt, int64_t n_d, const int32_t* __restrict__ chunk_rows,
                                                    int32_t* __restrict__ row_src /* [n_d*8] */, Head* __restrict__ head,
                                                    float* __restrict__ vscore)
{
    __shared__ uint8_t cnt[kRowsChunk];
    __shared__ int32_t first[kRowsChunk];
    __shared__ int32_t wave_tot[16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t base = (int64_t)blockIdx.x * kRowsChunk;
    int32_t v[kRowsPer];
#pragma unroll
    for (int j = 0; j < kRowsPer; ++j) {
        const int64_t c = base + j * 1024 + threadIdx.x;
        v[j] = c < n_d ? n_stmt[c] : 0;
    }
    // rows of the chunks before this one
    int32_t before = 0;
    for (int b = threadIdx.x; b < (int)blockIdx.x; b += 1024) before += chunk_rows[b];
    const int32_t carry = block_sum_1024(before, wave_tot);
#pragma unroll
    for (int j = 0; j < kRowsPer; ++j) {
        const int64_t c = base + j * 1024 + threadIdx.x;
        cnt[j * 1024 + threadIdx.x] = (uint8_t)clamp_stmt(v[j]);
        if (c < n_d) vscore[c] = 0.f;
    }
    __syncthreads();
    int32_t m[kRowsPer], mine = 0;
#pragma unroll
    for (int j = 0; j < kRowsPer; ++j) {
        m[j] = cnt[threadIdx.x * kRowsPer + j];
        mine += m[j];
    }
    int32_t incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int32_t up = __shfl_up(incl, off, 64);
        if (lane >= off) incl += up;
    }
    __syncthreads();   // wave_tot is free again
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int32_t ahead = 0, all = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        const int32_t t = wave_tot[w];
        ahead += w < wave ? t : 0;
        all += t;
    }
    int32_t row = carry + ahead + incl - mine;
#pragma unroll
    for (int j = 0; j < kRowsPer; ++j) {
        first[threadIdx.x * kRowsPer + j] = row;
        row += m[j];
    }
    __syncthreads();
#pragma unroll 8
    for (int p = threadIdx.x; p < kRowsChunk * kS; p += 1024) {
        const int c = p >> 3, s2 = p & 7;
        if (s2 < cnt[c]) row_src[first[c] + s2] = (int32_t)((base + c) * kS + s2);
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) head->n_rows = carry + all;
}

// ---- mlp_kernel ----------------------------------------------------------------------------------------------------

__device__ __forceinline__ float bf16_round(float x) { return (float)(__bf16)x; }

// FUSED: row numbering in LDS from n_stmt (n_d <= kFusedMax); else the row table of rows_kernel.
template <bool FUSED>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
mlp_kernel(const float* __restrict__ feat, const int32_t* __restrict__ row_src, const Head* __restrict__ head,
           const int32_t* __restrict__ n_stmt, int32_t n_d, const uint16_t* __restrict__ W1, const float* __restrict__ b1, const uint16_t* __restrict__ W2, const float* __restrict__ b2,
           const uint16_t* __restrict__ w3, float b3, float* __restrict__ vscore)
{
    // One LDS arena: first the staging area of the weights, then the tile buffers.
    __shared__ __attribute__((aligned(16))) __bf16 arena[kTM * kXs + kTM * kHs];
    __shared__ float red[4][kTM];        // last-layer partial sums per wavefront, then the row outputs in red[0]
    __shared__ __attribute__((aligned(16))) float cst[3][kH];   // b1, b2, w3 as binary32
    __shared__ int32_t src[2][kTM];      // source row (candidate * 8 + statement) of the tile's rows, double-buffered
    __bf16* X = arena;                   // feature tile, bfloat16 [kTM][kXs]
    __bf16* H1 = arena + kTM * kXs;      // first hidden layer of the tile [kTM][kHs]

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int step = gridDim.x;

    // Row numbering.  before[c] = valid rows of candidates 0..c-1; tile_first[t] = first candidate of tile t.
    extern __shared__ uint32_t dyn[];
    uint32_t* before = dyn;                                                     // [n_d + 1]
    uint16_t* tile_first = reinterpret_cast<uint16_t*>(dyn + (FUSED ? n_d + 1 : 0));   // [tiles + 1]
    __shared__ uint32_t scan_tot[4];
    int n_rows, n_tiles;
    if constexpr (FUSED) {
        const int max_tiles = (n_d * kS + kNominal - 1) / kNominal;
        if ((reinterpret_cast<uintptr_t>(n_stmt) & 15) == 0) {
            // four counts per load, eight loads in flight per thread
            typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
            const int n4 = n_d >> 2;
            for (int base = 0; base < n4; base += 8 * kThreads) {
                i32x4 v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int q = base + j * kThreads + threadIdx.x;
                    v[j] = *reinterpret_cast<const i32x4*>(n_stmt + 4 * (q < n4 ? q : 0));
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int q = base + j * kThreads + threadIdx.x;
                    if (q < n4) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) before[4 * q + e] = (uint32_t)(v[j][e] < 0 ? 0 : v[j][e] > kS ? kS : v[j][e]);
                    }
                }
            }
            for (int c = 4 * n4 + threadIdx.x; c < n_d; c += kThreads) {
                const int v = n_stmt[c];
                before[c] = (uint32_t)(v < 0 ? 0 : v > kS ? kS : v);
            }
        } else {
            for (int base = 0; base < n_d; base += 8 * kThreads) {   // eight loads in flight per thread
                int v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int c = base + j * kThreads + threadIdx.x;
                    v[j] = c < n_d ? n_stmt[c] : 0;
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int c = base + j * kThreads + threadIdx.x;
                    if (c < n_d) before[c] = (uint32_t)(v[j] < 0 ? 0 : v[j] > kS ? kS : v[j]);
                }
            }
        }
        for (int t = threadIdx.x; t <= max_tiles; t += kThreads) tile_first[t] = (uint16_t)n_d;
        __syncthreads();
        // candidates without rows score 0; the workgroups share them out
        for (int c = blockIdx.x * kThreads + threadIdx.x; c < n_d; c += step * kThreads)
            if (before[c] == 0) vscore[c] = 0.f;
        // thread t owns a run of `per` candidates (odd: neighbouring threads then start in different banks)
        const int per = ((n_d + kThreads - 1) / kThreads) | 1;
        const int c_lo = threadIdx.x * per < n_d ? threadIdx.x * per : n_d;
        const int c_hi = c_lo + per < n_d ? c_lo + per : n_d;
        uint32_t mine = 0;
        for (int c0 = c_lo; c0 < c_hi; c0 += 8) {
            uint32_t v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = c0 + j < c_hi ? before[c0 + j] : 0u;
#pragma unroll
            for (int j = 0; j < 8; ++j) mine += v[j];
        }
        uint32_t incl = mine;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t up = __shfl_up(incl, off, 64);
            if (lane >= off) incl += up;
        }
        if (lane == 63) scan_tot[wave] = incl;
        __syncthreads();
        uint32_t run = incl - mine, total = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            run += w < wave ? scan_tot[w] : 0u;
            total += scan_tot[w];
        }
        // candidate c + 1 is the first one at or after a multiple of 57 when the running count reaches it (a candidate
        // has at most 8 rows, so it reaches at most one multiple)
        uint32_t tq = run / kNominal + 1, reach = tq * kNominal;
        for (int c0 = c_lo; c0 < c_hi; c0 += 8) {
            uint32_t v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = c0 + j < c_hi ? before[c0 + j] : 0u;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int c = c0 + j;
                if (c < c_hi) {
                    before[c] = run;
                    run += v[j];
                    if (run >= reach) {
                        tile_first[tq] = (uint16_t)(c + 1);
                        ++tq;
                        reach += kNominal;
                    }
                }
            }
        }
        if (threadIdx.x == 0) {
            before[n_d] = total;
            tile_first[0] = 0;
        }
        n_rows = (int)total;
        n_tiles = (n_rows + kNominal - 1) / kNominal;
        __syncthreads();
    } else {
        n_rows = head->n_rows;
        n_tiles = (n_rows + kTM - 1) / kTM;
    }
    // source row (candidate * 8 + statement) of row r of tile t, or -1
    auto source_of = [&](int t, int r) -> int {
        if constexpr (FUSED) {
            if (t >= n_tiles) return -1;
            int lo = tile_first[t], hi = tile_first[t + 1];
            const uint32_t R = before[lo] + (uint32_t)r;
            if (R >= before[hi]) return -1;
            while (hi - lo > 1) {   // before[lo] <= R < before[hi]
                const int mid = (lo + hi) >> 1;
                if (before[mid] <= R) lo = mid; else hi = mid;
            }
            return lo * kS + (int)(R - before[lo]);
        } else {
            const int g = t * kTM + r;
            return g < n_rows ? row_src[g] : -1;
        }
    };

    // prologue: source rows of the first two tiles, features of the first
    int tile = blockIdx.x;
    if (threadIdx.x < kTM) {
        src[0][threadIdx.x] = source_of(tile, threadIdx.x);
        src[1][threadIdx.x] = source_of(tile + step, threadIdx.x);
    }
    __syncthreads();
    f32x4 xr[kXLoads];
    // FETCH(buf): features of the tile whose source rows sit in src[buf] -> registers.  Rows past the end read row 0
    // (their outputs are never used), pieces past the end repeat the last piece: nothing between the loads waits.
#define PRUNER_FETCH(buf)                                                                                             \
    _Pragma("unroll") for (int i = 0; i < kXLoads; ++i) {                                                             \
        int q = threadIdx.x + i * kThreads;                                                                           \
        q = q < kTM * kF4 ? q : kTM * kF4 - 1;                                                                        \
        const int sr = src[buf][q / kF4];                                                                             \
        xr[i] = *reinterpret_cast<const f32x4*>(feat + (size_t)(sr < 0 ? 0 : sr) * kF + 4 * (q % kF4));               \
    }
    // PARK: registers -> X as bfloat16
#define PRUNER_PARK()                                                                                                 \
    _Pragma("unroll") for (int i = 0; i < kXLoads; ++i) {                                                             \
        int q = threadIdx.x + i * kThreads;                                                                           \
        q = q < kTM * kF4 ? q : kTM * kF4 - 1;                                                                        \
        bf16x4 o;                                                                                                     \
        o[0] = (__bf16)xr[i][0];                                                                                       \
        o[1] = (__bf16)xr[i][1];                                                                                       \
        o[2] = (__bf16)xr[i][2];                                                                                       \
        o[3] = (__bf16)xr[i][3];                                                                                       \
        *reinterpret_cast<bf16x4*>(&X[(q / kF4) * kXs + 4 * (q % kF4)]) = o;                                          \
    }
    if (tile < n_tiles) {
        PRUNER_FETCH(0)   // in flight while the weights are staged
    }

    // This wavefront's weights.  As the A operand of a 32x32x16 MFMA, lane (l32, half) supplies hidden unit
    // n = base + l32 and the eight depth entries 8*half .. 8*half+7 of the 16-deep step.  The 64 rows of a
    // wavefront's slice are read from memory by the whole workgroup, contiguously, into LDS (W1 rows padded
    // with zeros to 176), from where the owning wavefront picks its fragments.
    bf16x8 w1r[2][kK1 / 16], w2r[2][kH / 16];
    {
        __bf16* S1 = arena;                 // [64][kXs]: row strides as for the tiles, which spread the banks
        __bf16* S2 = arena + 64 * kXs;      // [64][kHs]
        constexpr int kW1Loads = (64 * kF4 + kThreads - 1) / kThreads;   // 8-byte pieces per thread (11)
        constexpr int kW2Loads = 64 * (kH / 8) / kThreads;               // 16-byte pieces per thread (8)
        // depth 164..175 of the staged W1 rows is zero and stays zero
        for (int q = threadIdx.x; q < 64 * ((kK1 - kF) / 4); q += kThreads)
            *reinterpret_cast<uint2*>(&S1[(q / ((kK1 - kF) / 4)) * kXs + kF + 4 * (q % ((kK1 - kF) / 4))]) = make_uint2(0, 0);
        u32x2 p1[kW1Loads];
        u32x4 p2[kW2Loads];
        // LOAD(w): every piece of slice w in flight together; pieces past the end repeat the last one
#define PRUNER_LOAD_SLICE(w)                                                                                         \
    _Pragma("unroll") for (int i = 0; i < kW1Loads; ++i) {                                                           \
        int q = threadIdx.x + i * kThreads;                                                                          \
        q = q < 64 * kF4 ? q : 64 * kF4 - 1;                                                                         \
        p1[i] = *reinterpret_cast<const u32x2*>(W1 + (size_t)(64 * (w) + q / kF4) * kF + 4 * (q % kF4));             \
    }                                                                                                                \
    _Pragma("unroll") for (int i = 0; i < kW2Loads; ++i) {                                                           \
        const int q = threadIdx.x + i * kThreads;                                                                    \
        p2[i] = *reinterpret_cast<const u32x4*>(W2 + (size_t)(64 * (w) + q / (kH / 8)) * kH + 8 * (q % (kH / 8)));   \
    }
        PRUNER_LOAD_SLICE(0)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (w > 0) __syncthreads();      // the previous slice has been picked up
#pragma unroll
            for (int i = 0; i < kW1Loads; ++i) {
                int q = threadIdx.x + i * kThreads;
                q = q < 64 * kF4 ? q : 64 * kF4 - 1;
                *reinterpret_cast<u32x2*>(&S1[(q / kF4) * kXs + 4 * (q % kF4)]) = p1[i];
            }
#pragma unroll
            for (int i = 0; i < kW2Loads; ++i) {
                const int q = threadIdx.x + i * kThreads;
                *reinterpret_cast<u32x4*>(&S2[(q / (kH / 8)) * kHs + 8 * (q % (kH / 8))]) = p2[i];
            }
            if (w + 1 < 4) {                 // the next slice travels while this one is picked up
                PRUNER_LOAD_SLICE(w + 1)
            }
            __syncthreads();
            if (wave == w) {
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) {
#pragma unroll
                    for (int ks = 0; ks < kK1 / 16; ++ks) w1r[nt][ks] = *reinterpret_cast<const bf16x8*>(&S1[(32 * nt + l32) * kXs + 16 * ks + 8 * half]);
#pragma unroll
                    for (int ks = 0; ks < kH / 16; ++ks) w2r[nt][ks] = *reinterpret_cast<const bf16x8*>(&S2[(32 * nt + l32) * kHs + 16 * ks + 8 * half]);
                }
            }
        }
#undef PRUNER_LOAD_SLICE
        __syncthreads();
    }
    // Biases and last-layer weights in accumulator order: register i of a 32x32 result holds hidden unit
    // 8*(i/4) + 4*half + i%4 of the tile, so a lane needs four runs of four neighbours per tile; they sit in LDS
    // and are read again for every tile instead of occupying 96 registers.
    for (int n = threadIdx.x; n < kH; n += kThreads) {
        cst[0][n] = b1[n];
        cst[1][n] = b2[n];
        cst[2][n] = __uint_as_float((uint32_t)w3[n] << 16);
    }

    // the zero padding of the feature tile (depth 164..183) is written once
    for (int q = threadIdx.x; q < kTM * ((kXs - kF) / 4); q += kThreads) {
        const int r = q / ((kXs - kF) / 4), j = q % ((kXs - kF) / 4);
        *reinterpret_cast<uint2*>(&X[r * kXs + kF + 4 * j]) = make_uint2(0, 0);
    }

    if (tile < n_tiles) {
        PRUNER_PARK()   // the first tile's features were requested before the weights
    }
    __syncthreads();

    // the last layer's weights of this lane's 32 hidden units stay in registers (they are read once per tile row otherwise)
    float w3r[2][16];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int i = 0; i < 16; ++i) w3r[nt][i] = cst[2][64 * wave + 32 * nt + 8 * (i / 4) + 4 * half + (i % 4)];

    int cur = 0;
    for (; tile < n_tiles; tile += step, cur ^= 1) {
        __syncthreads();   // the source rows refilled at the end of the previous iteration are visible
        // start fetching the next tile's features; its source rows were loaded one iteration ago
        const bool more = tile + step < n_tiles;
        int next_src = -1;   // source row of the tile after next, fetched now, stored when src[cur] is free
        if (threadIdx.x < kTM) next_src = source_of(tile + 2 * step, threadIdx.x);
        if (more) {
            PRUNER_FETCH(cur ^ 1)
        }

        // layer 1: H1^T[n][m] = b1[n] + sum_k W1[n][k] X[m][k]
        floatx16 acc[2][2];
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[nt][mt][i] = cst[0][64 * wave + 32 * nt + 8 * (i / 4) + 4 * half + (i % 4)];
        {   // operand fragments of steps ks+1 and ks+2 are on their way from LDS when the MFMAs of step ks are issued
            bf16x8 xb[3][2];
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) xb[p][mt] = *reinterpret_cast<const bf16x8*>(&X[(32 * mt + l32) * kXs + 16 * p + 8 * half]);
#pragma unroll
            for (int ks = 0; ks < kK1 / 16; ++ks) {
                if (ks + 2 < kK1 / 16) {
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt)
                        xb[(ks + 2) % 3][mt] = *reinterpret_cast<const bf16x8*>(&X[(32 * mt + l32) * kXs + 16 * (ks + 2) + 8 * half]);
                }
                __builtin_amdgcn_sched_barrier(0);   // keep the reads ahead of the MFMAs that do not need them yet
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt)
                        acc[nt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1r[nt][ks], xb[ks % 3][mt], acc[nt][mt], 0, 0, 0);
            }
        }
        // ReLU, round to bfloat16, park in LDS as H1[m][n]: a lane owns row m = 32*mt + l32 and, per group of four
        // accumulator registers, four neighbouring hidden units
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x4 o;
#pragma unroll
                    for (int j = 0; j < 4; ++j) o[j] = (__bf16)fmaxf(acc[nt][mt][4 * g + j], 0.f);
                    *reinterpret_cast<bf16x4*>(&H1[(32 * mt + l32) * kHs + 64 * wave + 32 * nt + 8 * g + 4 * half]) = o;
                }
        __syncthreads();   // H1 complete; X no longer read

        // layer 2: H2^T[n][m] = b2[n] + sum_k W2[n][k] H1[m][k]
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[nt][mt][i] = cst[1][64 * wave + 32 * nt + 8 * (i / 4) + 4 * half + (i % 4)];
        {
            bf16x8 hb[3][2];
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) hb[p][mt] = *reinterpret_cast<const bf16x8*>(&H1[(32 * mt + l32) * kHs + 16 * p + 8 * half]);
#pragma unroll
            for (int ks = 0; ks < kH / 16; ++ks) {
                if (ks + 2 < kH / 16) {
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt)
                        hb[(ks + 2) % 3][mt] = *reinterpret_cast<const bf16x8*>(&H1[(32 * mt + l32) * kHs + 16 * (ks + 2) + 8 * half]);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt)
                        acc[nt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w2r[nt][ks], hb[ks % 3][mt], acc[nt][mt], 0, 0, 0);
            }
        }

        // layer 3: this wavefront's share of w3 . relu(H2) for each row
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            float part = 0.f;
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int i = 0; i < 16; ++i) part += w3r[nt][i] * bf16_round(fmaxf(acc[nt][mt][i], 0.f));
            part += __shfl_xor(part, 32, 64);
            if (half == 0) red[wave][32 * mt + l32] = part;
        }
        // the next tile's features go to X (free since the barrier above); the source rows of the tile after next
        if (more) {
            PRUNER_PARK()
        }
        __syncthreads();   // red complete, X(next) complete
        if (threadIdx.x < kTM) {   // the first wavefront, one lane per row
            // a candidate's rows are neighbours and at most 8: three shift-and-add steps that stop at candidate borders
            // leave the candidate's sum in its first row
            const int r = threadIdx.x;
            const int sr = src[cur][r];
            const int cand = sr >> 3;   // -1 for rows past the end
            float y = (((red[0][r] + red[1][r]) + red[2][r]) + red[3][r]) + b3;
#pragma unroll
            for (int off = 1; off < kS; off <<= 1) {
                const float other = __shfl_down(y, off, 64);
                const int theirs = __shfl_down(cand, off, 64);
                if (r + off < kTM && theirs == cand) y += other;
            }
            const int ahead = __shfl_up(cand, 1, 64);
            if (sr >= 0 && (r == 0 || ahead != cand)) {
                if constexpr (FUSED) vscore[cand] = y;   // the candidate's only tile
                else atomicAdd(&vscore[cand], y);
            }
        }
        __syncthreads();   // src[cur] and red are free again
        if (threadIdx.x < kTM) src[cur][threadIdx.x] = next_src;
    }
#undef PRUNER_FETCH
#undef PRUNER_PARK
}

struct Layout {
    size_t head, chunk_rows, row_src, total;
};

Layout layout(int64_t n_d)
{
    Layout L;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += round_up(bytes, 256);
        return at;
    };
    L.head = take(sizeof(Head));
    L.chunk_rows = take(((size_t)(n_d / kRowsChunk) + 1) * sizeof(int32_t));
    L.row_src = take((size_t)n_d * kS * sizeof(int32_t));
    L.total = off;
    return L;
}

int g_num_cus = 0;
bool g_fused_ready = false;   // the in-kernel scan's LDS allowance has been raised

}  // namespace

size_t verify_workspace_bytes(int64_t n_d) { return layout(n_d < 0 ? 0 : n_d).total; }

}  // namespace pruner

using namespace pruner;

extern "C" int pruner_verify_score(const float* feat, const int32_t* n_stmt, int64_t n_d, const pruner_mlp* w, float* vscore,
                                   void* workspace, size_t workspace_bytes, void* stream)
{
    if (!feat || !n_stmt || !w || !vscore || n_d < 0 || n_d > (int64_t)(0x7FFFFFFF / kS)) return PRUNER_EINVAL;
    if (!w->W1 || !w->b1 || !w->W2 || !w->b2 || !w->w3) return PRUNER_EINVAL;
    if (!aligned(feat, 16) || !aligned(n_stmt, 4) || !aligned(vscore, 4) || !aligned(w->W1, 8) || !aligned(w->W2, 16) ||
        !aligned(w->b1, 4) || !aligned(w->b2, 4) || !aligned(w->w3, 2))
        return PRUNER_EINVAL;
    if (!workspace || !aligned(workspace, 256)) return PRUNER_EWORKSPACE;
    const Layout L = layout(n_d);
    if (workspace_bytes < L.total) return PRUNER_EWORKSPACE;
    if (n_d == 0) return PRUNER_OK;

    if (g_num_cus == 0) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
            return PRUNER_EHIP;
        g_num_cus = cus;
    }

    hipStream_t st = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    Head* head = reinterpret_cast<Head*>(ws + L.head);
    int32_t* row_src = reinterpret_cast<int32_t*>(ws + L.row_src);

    if (n_d <= kFusedMax) {
        // one launch: every workgroup numbers the rows itself
        const int64_t max_tiles = (n_d * kS + kNominal - 1) / kNominal;
        const size_t dyn_bytes = round_up((size_t)(n_d + 1) * 4 + (size_t)(max_tiles + 1) * 2, 16);
        if (!g_fused_ready) {
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(&mlp_kernel<true>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)round_up((size_t)(kFusedMax + 1) * 4 + (size_t)((kFusedMax * kS) / kNominal + 3) * 2, 16)) != hipSuccess)
                return PRUNER_EHIP;
            g_fused_ready = true;
        }
        const unsigned grid = (unsigned)(max_tiles < g_num_cus ? (max_tiles < 1 ? 1 : max_tiles) : g_num_cus);
        hipLaunchKernelGGL(mlp_kernel<true>, dim3(grid), dim3(kThreads), dyn_bytes, st, feat, row_src, head, n_stmt, (int32_t)n_d, w->W1, w->b1,
                           w->W2, w->b2, w->w3, w->b3, vscore);
        PRUNER_LAUNCH_CHECK();
        return PRUNER_OK;
    }
    const unsigned chunks = (unsigned)((n_d + kRowsChunk - 1) / kRowsChunk);
    int32_t* chunk_rows = reinterpret_cast<int32_t*>(ws + L.chunk_rows);
    hipLaunchKernelGGL(rows_total_kernel, dim3(chunks), dim3(1024), 0, st, n_stmt, n_d, chunk_rows);
    PRUNER_LAUNCH_CHECK();
    hipLaunchKernelGGL(rows_kernel, dim3(chunks), dim3(1024), 0, st, n_stmt, n_d, chunk_rows, row_src, head, vscore);
    PRUNER_LAUNCH_CHECK();
    const int64_t max_tiles = (n_d * kS + kTM - 1) / kTM;
    const unsigned grid = (unsigned)(max_tiles < g_num_cus ? max_tiles : g_num_cus);
    hipLaunchKernelGGL(mlp_kernel<false>, dim3(grid), dim3(kThreads), 0, st, feat, row_src, head, n_stmt, (int32_t)n_d, w->W1, w->b1, w->W2,
                       w->b2, w->w3, w->b3, vscore);
    PRUNER_LAUNCH_CHECK();
    return PRUNER_OK;
}
