// Verify stage: statement-feature branch of the learned cost model on the drafted candidates
// (Sec. 4.2, "Pattern-aware Transformer": statement features -> linear layers -> summation over statements).
//
//   y(c,s)   = w3 . relu(W2 relu(W1 x(c,s) + b1) + b2) + b3          164 -> 256 -> 256 -> 1
//   vscore_c = sum over s < n_stmt[c] of y(c,s)
//
// The valid statement rows get consecutive row numbers (exclusive scan of n_stmt), so the matrix cores never see
// padding rows.  Up to 16383 candidates (drafted sets are a few thousand) a workgroup of mlp_kernel owns a contiguous
// range of at most 64 candidates and numbers the rows of that range itself (one wavefront-wide scan while its weights
// arrive): one launch, no workspace traffic, no pass over the whole set, and tiles that begin and end on candidate
// boundaries, so every candidate is summed and stored by exactly one thread.  Beyond that:
//   rows kernels   the scan as two launches of their own (chunk totals, then one workgroup per chunk of 8192
//                  candidates), writing a table of source rows; clears vscore.
//   mlp_kernel     persistent workgroups (one per CU, 4 wavefronts, one per SIMD).  Wavefront w owns hidden units
//                  [64w, 64w+64) of both layers and keeps its slices of W1 and W2 in registers for the whole
//                  launch (read straight from memory, in MFMA operand layout, while the rows are numbered); feature rows stream
//                  through LDS 64 at a time as bfloat16, the next tile's rows being fetched while the current tile
//                  is computed.  Layers are computed transposed (H^T = W X^T) with v_mfma_f32_32x32x16_bf16, so
//                  that one lane holds 16 hidden units of ONE row: bias is the accumulator's initial value, ReLU
//                  and the bfloat16 rounding are lane-local, and the last layer's dot product with w3 is a
//                  lane-local sum plus one cross-lane add.  Hidden activations never leave the
//                  CU.  With one wavefront per SIMD nothing else would hide the epilogues' latency, so the two
//                  32-row halves of a tile run half a layer apart: the vector work of one half (ReLU, rounding,
//                  stores to LDS, the last layer) is issued between the MFMAs of the other.  The rows of a
//                  candidate are added in statement order by the lane of its first row; with the row table a
//                  candidate whose rows straddle two tiles receives two atomic adds onto zero, which commute.
#include "common.h"
#include "mfma_tile.h"

namespace pruner {
namespace {

using namespace tile;

constexpr int kF = PRUNER_FEAT_DIM;   // 164
constexpr int kS = PRUNER_MAX_STMT;   // 8
constexpr int kH = PRUNER_HIDDEN;     // 256
constexpr int kTM = 64;               // rows per tile
constexpr int kK1 = 176;              // 164 padded to a multiple of the MFMA depth 16
constexpr int kXs = kK1 + 8;          // LDS row strides in bfloat16 elements (rows stay 16-byte aligned)
constexpr int kHs = kH + 8;
constexpr int kThreads = 256;
constexpr int kF4 = kF / 4;           // float4 per feature row (41)
constexpr int kRowThreads = 8;                                   // threads that share a feature row: 128 contiguous bytes per request
constexpr int kXPass = kTM / (kThreads / kRowThreads);           // passes over the tile's rows (2)
constexpr int kXCols = (kF4 + kRowThreads - 1) / kRowThreads;    // float4 a thread fetches per row (6)
constexpr int kXLoads = kXPass * kXCols;                         // float4 a thread fetches per tile (12)
constexpr int kNominal = kTM - (kS - 1);   // in-kernel scan: tile t begins at the first candidate whose rows start at or after 57 t,
                                           // and therefore holds at most 57 + 7 = 64 rows
constexpr int kLocalMax = 64;              // candidates of one workgroup when it numbers its own rows (one per lane of a wavefront)
constexpr int kLocalTiles = (kLocalMax * kS + kNominal - 1) / kNominal + 1;   // tiles such a range can need (10)
constexpr int kFusedMax = 16383;           // largest set that is numbered that way

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

// One of the 16 half pieces of the last layer for 32 rows: two hidden units of row l32 (ReLU, rounded to bfloat16) times
// their weights (w3r: this lane's 32 weights in accumulator order), added to part: six vector instructions, which fit in
// the shadow of one MFMA.  Plain FMAs on the unpacked halves: the packed dot-product instruction waits for the matrix
// pipe, which is busy here.
__device__ __forceinline__ void last_layer_half(const floatx16 (&acc)[2], int hp, const float (&w3r)[2][16], float& part)
{
    const int nt = hp >> 3, at = 2 * (hp & 7);
    const uint32_t v = relu_bf16x2(acc[nt][at], acc[nt][at + 1]);
    part = __builtin_fmaf(__uint_as_float(v << 16), w3r[nt][at], part);
    part = __builtin_fmaf(__uint_as_float(v & 0xFFFF0000u), w3r[nt][at + 1], part);
}

// FUSED: row numbering in LDS from n_stmt (n_d <= kFusedMax); else the row table of rows_kernel.
template <bool FUSED>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
mlp_kernel(const float* __restrict__ feat, const int32_t* __restrict__ row_src, const Head* __restrict__ head,
           const int32_t* __restrict__ n_stmt, int32_t n_d, const uint16_t* __restrict__ W1, const float* __restrict__ b1, const uint16_t* __restrict__ W2, const float* __restrict__ b2,
           const uint16_t* __restrict__ w3, float b3, float* __restrict__ vscore)
{
    // The tile buffers.
    __shared__ __attribute__((aligned(16))) __bf16 arena[kTM * kXs + kTM * kHs];
    __shared__ float red[4][kTM];        // last-layer partial sums per wavefront
    __shared__ int32_t src[3][kTM];      // source row (candidate * 8 + statement) of the rows of three consecutive tiles
    __bf16* X = arena;                   // feature tile, bfloat16 [kTM][kXs]
    __bf16* H1 = arena + kTM * kXs;      // first hidden layer of the tile [kTM][kHs]

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int step = FUSED ? 1 : (int)gridDim.x;   // FUSED: the workgroup walks the tiles of its own candidates

    // Row numbering (FUSED).  The workgroup owns candidates [c_first, c_first + n_local); before[l] = valid rows of its
    // candidates 0..l-1; tile_first[t] = first of its candidates whose rows start at or after kNominal * t.
    __shared__ uint32_t before[kLocalMax + 1];
    __shared__ uint32_t tile_first[kLocalTiles + 2];
    // This wavefront's weights, requested first so that they travel while the rows are numbered.  As the A operand of
    // a 32x32x16 MFMA, lane (l32, half) supplies hidden unit n = base + l32 and the eight depth entries 8*half ..
    // 8*half+7 of the 16-deep step: 16 bytes of row n of the matrix, straight from memory into the lane's registers
    // (each workgroup reads the matrices once; they stay in L2 for the others).  W1's rows end at depth 164: the
    // last step is four entries for half 0 and zeros otherwise.
    // The first layer's bias rides in that last step: the feature tile holds 1 at depths 164, 165, 166 and W1's row n
    // holds b1[n] there as three bfloat16 pieces (b = hi + mid + lo exactly: 3 x 8 significand bits), so the matrix core
    // adds the bias inside its binary32 accumulation and no instruction initialises the accumulator.
    static_assert(kK1 / 16 == kF / 16 + 1 && kF % 16 == 4, "W1's last depth step holds four entries");
    bf16x8 w1r[2][kK1 / 16], w2r[2][kH / 16];
    {
        typedef u32x4 u32x4_a8 __attribute__((aligned(8)));   // W1's rows are 328 bytes
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            const int n = 64 * wave + 32 * nt + l32;
            const uint16_t* r1 = W1 + (size_t)n * kF;
            const uint16_t* r2 = W2 + (size_t)n * kH + 8 * half;
#pragma unroll
            for (int ks = 0; ks < kF / 16; ++ks) w1r[nt][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4_a8*>(r1 + 16 * ks + 8 * half));
            const u32x2 tail = *reinterpret_cast<const u32x2*>(r1 + 16 * (kF / 16));   // depth 160..163
            u32x4 last = {0u, 0u, 0u, 0u};
            const float bias = b1[n];
            const __bf16 b_hi = (__bf16)bias;
            const float rest1 = bias - (float)b_hi;
            const __bf16 b_mid = (__bf16)rest1;
            const __bf16 b_lo = (__bf16)(rest1 - (float)b_mid);
            last[0] = half == 0 ? tail[0] : 0u;
            last[1] = half == 0 ? tail[1] : 0u;
            last[2] = half == 0 ? ((uint32_t)__builtin_bit_cast(uint16_t, b_hi) | ((uint32_t)__builtin_bit_cast(uint16_t, b_mid) << 16)) : 0u;
            last[3] = half == 0 ? (uint32_t)__builtin_bit_cast(uint16_t, b_lo) : 0u;
            w1r[nt][kF / 16] = __builtin_bit_cast(bf16x8, last);
#pragma unroll
            for (int ks = 0; ks < kH / 16; ++ks) w2r[nt][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(r2 + 16 * ks));
        }
    }

    int n_rows, n_tiles, c_first = 0;
    if constexpr (FUSED) {
        // every wavefront scans the range's counts for itself (one count per lane); wavefront 0 leaves the tables in LDS
        const int per = (n_d + (int)gridDim.x - 1) / (int)gridDim.x;   // <= kLocalMax: the host sizes the grid for that
        c_first = (int)blockIdx.x * per;
        const int n_local = c_first >= n_d ? 0 : (n_d - c_first < per ? n_d - c_first : per);
        uint32_t cnt = 0;
        if (lane < n_local) {
            const int v = n_stmt[c_first + lane];
            cnt = (uint32_t)(v < 0 ? 0 : v > kS ? kS : v);
        }
        uint32_t incl = cnt;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t up = __shfl_up(incl, off, 64);
            if (lane >= off) incl += up;
        }
        const uint32_t total = __shfl(incl, 63, 64), mine = incl - cnt;   // mine: rows before this lane's candidate
        n_rows = (int)total;
        n_tiles = (n_rows + kNominal - 1) / kNominal;
        if (wave == 0) {
            if (lane < kLocalTiles + 2) tile_first[lane] = (uint32_t)n_local;
            if (lane < n_local && cnt == 0) vscore[c_first + lane] = 0.f;   // a candidate without rows scores 0
        }
        __syncthreads();
        if (wave == 0) {
            before[lane] = mine;
            if (lane == 63) before[64] = total;
            // candidate `lane` is the first at or after a multiple of kNominal when its rows start there or later and its
            // predecessor's start earlier (a candidate has at most 8 rows, so it can be that for one multiple only)
            const uint32_t prev = __shfl_up(mine, 1, 64);
            const uint32_t t = mine / kNominal;
            if (lane < n_local && (lane == 0 || (t >= 1 && prev < t * kNominal))) tile_first[lane == 0 ? 0 : t] = (uint32_t)lane;
        }
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
            return (c_first + lo) * kS + (int)(R - before[lo]);
        } else {
            const int g = t * kTM + r;
            return g < n_rows ? row_src[g] : -1;
        }
    };

    // prologue: source rows of the first two tiles, features of the first
    int tile = FUSED ? 0 : (int)blockIdx.x;
    if (threadIdx.x < kTM) {
        src[0][threadIdx.x] = source_of(tile, threadIdx.x);
        src[1][threadIdx.x] = source_of(tile + step, threadIdx.x);
    }
    __syncthreads();
    // The tile's features, fetched in twelve pieces per thread: eight threads share a row and take every eighth float4 of
    // it; thread t serves rows t/8 and t/8 + 32.  A piece is requested (source row -> registers) and much later
    // converted and stored to X; rows past the end read row 0 (their outputs are never used), and pieces past a row's
    // end repeat its last float4 and are stored beyond the depth the MFMAs read.  One load per piece, nothing between
    // the loads waits, and the pieces can be issued one by one between MFMAs.
    f32x4 xr[kXLoads];
    int fetch_src[kXPass];
    const int f_sub = threadIdx.x & (kRowThreads - 1), f_row = threadIdx.x / kRowThreads;
    auto fetch_read = [&](int buf) {
#pragma unroll
        for (int ps = 0; ps < kXPass; ++ps) fetch_src[ps] = src[buf][f_row + ps * (kThreads / kRowThreads)];
    };
    auto fetch_issue = [&](int i) {
        const int ps = i / kXCols, col = f_sub + kRowThreads * (i % kXCols);
        const int sr = fetch_src[ps];
        xr[i] = *reinterpret_cast<const f32x4*>(feat + (size_t)(sr < 0 ? 0 : sr) * kF + 4 * (col < kF4 ? col : kF4 - 1));
    };
    auto park_piece = [&](int i) {
        const int ps = i / kXCols, col = f_sub + kRowThreads * (i % kXCols);
        const f32x2 lo = {xr[i][0], xr[i][1]}, hi = {xr[i][2], xr[i][3]};
        u32x2 o;
        o[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2));
        o[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2));
        *reinterpret_cast<u32x2*>(&X[(f_row + ps * (kThreads / kRowThreads)) * kXs + (col < kF4 ? 4 * col : kK1)]) = o;   // depth 176..179 is never read
    };
    if (tile < n_tiles) {   // in flight while the weights are staged
        fetch_read(0);
#pragma unroll
        for (int i = 0; i < kXLoads; ++i) fetch_issue(i);
    }

    // The weights live in the accumulation registers (which MFMAs read as well as any), so that the ordinary vector
    // registers are left to the accumulators: the vector ALU reads those without a copy.  (This also waits for them.)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
#pragma unroll
        for (int ks = 0; ks < kK1 / 16; ++ks) asm volatile("" : "+a"(w1r[nt][ks]));
#pragma unroll
        for (int ks = 0; ks < kH / 16; ++ks) asm volatile("" : "+a"(w2r[nt][ks]));
    }
    // The second layer's bias of this lane's hidden units stays in registers, in accumulator order: the layer's first
    // MFMAs take it as their addend.  So do the last layer's weights, widened to binary32.
    floatx16 b2r[2];
    float w3r[2][16];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int n = 64 * wave + 32 * nt + 8 * (i / 4) + 4 * half + (i % 4);
            b2r[nt][i] = b2[n];
            w3r[nt][i] = __uint_as_float((uint32_t)w3[n] << 16);
        }
    // (the loads above are complete here: a load still pending at the loop's entry would make every iteration wait for
    // the feature rows it has just requested)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            asm volatile("" : "+v"(w3r[nt][i]));
            asm volatile("" : "+v"(b2r[nt][i]));
        }

    // the padding of the feature tile (depth 164..183) is written once: 1, 1, 1 (times the three pieces of b1), then zeros
    for (int q = threadIdx.x; q < kTM * ((kXs - kF) / 4); q += kThreads) {
        const int r = q / ((kXs - kF) / 4), j = q % ((kXs - kF) / 4);
        *reinterpret_cast<uint2*>(&X[r * kXs + kF + 4 * j]) = j == 0 ? make_uint2(0x3F803F80u, 0x00003F80u) : make_uint2(0, 0);
    }

    if (tile < n_tiles) {   // the first tile's features were requested before the weights
#pragma unroll
        for (int i = 0; i < kXLoads; ++i) park_piece(i);
    }
    __syncthreads();

    // Sums over statements, for the tile whose source rows sit in src[buf] and whose row outputs sit in red, in nine
    // branch-free steps (so that they can be issued between MFMAs): wavefront w owns rows 16w .. 16w+15 and looks at the
    // seven rows after them as well; the lane of a candidate's first row in the tile adds the candidate's rows in
    // statement order.
    float sum_y = 0.f, sum_total = 0.f, sum_p[4] = {0.f, 0.f, 0.f, 0.f}, sum_oy = 0.f;
    int sum_sr = -1, sum_prev = -1, sum_cand = -1, sum_oc = -1;
    // (the exchange of step q is asked for in step q - 1 and used in step q: a step never waits for its own exchange)
    auto sum_step = [&](int q, int buf) {
        const int r_raw = 16 * wave + lane;
        const bool in = lane < 16 + kS - 1 && r_raw < kTM;
        const int r = in ? r_raw : kTM - 1;
        if (q == 0) {
            sum_sr = src[buf][r];
            sum_prev = src[buf][r > 0 ? r - 1 : 0];
#pragma unroll
            for (int w = 0; w < 4; ++w) sum_p[w] = red[w][r];
        } else if (q == 1) {
            sum_sr = in ? sum_sr : -1;
            sum_prev = r > 0 ? sum_prev >> 3 : -2;
            sum_cand = sum_sr >> 3;   // -1 for rows past the end
            sum_y = (((sum_p[0] + sum_p[1]) + sum_p[2]) + sum_p[3]) + b3;
            sum_total = sum_y;
        } else {
            const int j = q - 1;   // 1 .. 7: the row j places further on
            sum_total = (sum_oc == sum_cand && lane + j < 64) ? sum_total + sum_oy : sum_total;
            asm volatile("" : "+v"(sum_total));   // (keeps the addition in this step)
        }
        if (q >= 1 && q < kS) {
            sum_oy = __shfl_down(sum_y, q, 64);
            sum_oc = __shfl_down(sum_cand, q, 64);
        }
    };
    auto sum_store = [&]() {
        if (lane < 16 && sum_sr >= 0 && sum_prev != sum_cand) {
            if constexpr (FUSED) vscore[sum_cand] = sum_total;   // the candidate's only tile
            else atomicAdd(&vscore[sum_cand], sum_total);
        }
    };
    // The source row of row 16w + lane (lanes 0..15) of tile t, in sixteen branch-free steps plus a last one: binary
    // search for the candidate whose rows contain the tile's row (FUSED), or the row table's entry.
    int find_lo = 0, find_hi = 0, find_ok = 0, next_src = -1;
    uint32_t find_R = 0, find_blo = 0, find_bhi = 0;
    auto find_step = [&](int q, int t) {
        if constexpr (FUSED) {
            if (q == 0) {
                find_ok = t < n_tiles && lane < 16;
                const int tc = t < n_tiles ? t : n_tiles - 1;
                find_lo = tile_first[tc];
                find_hi = tile_first[tc + 1];
            } else if (q == 1) {
                find_blo = before[find_lo];
                find_bhi = before[find_hi];
            } else if (q < 16) {
                if (q == 2) {
                    find_R = find_blo + (uint32_t)(16 * wave + (lane & 15));
                    find_ok = find_ok && find_R < find_bhi;
                }
                // before[lo] <= R < before[hi] while the row exists; fourteen halvings cover any range of candidates
                const int mid = (find_lo + find_hi) >> 1;
                const bool up = before[mid] <= find_R;
                find_lo = up ? mid : find_lo;
                find_hi = up ? find_hi : mid;
            } else if (q == 16) {
                find_blo = before[find_lo];
            } else {
                next_src = find_ok ? (c_first + find_lo) * kS + (int)(find_R - find_blo) : -1;
            }
        }
    };

    // A tile's two halves (rows 0..31: acc0, rows 32..63: acc1) run half a layer apart, the second half's last layer and
    // the sums over statements reaching into the next iteration; everything that is not an MFMA is issued in the gaps
    // between MFMAs (about six vector instructions fit in the shadow of one MFMA).  A layer's first MFMAs overwrite
    // their accumulator (addend: zero, or the second layer's bias), which its last reader has left by then.
    auto finish_rows = [&](float part, int first_row) {   // the last layer's partial sums of 32 rows -> red
        part += __shfl_xor(part, 32, 64);
        if (half == 0) red[wave][first_row + l32] = part;
    };
    floatx16 acc0[2], acc1[2];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc0[nt][i] = acc1[nt][i] = 0.f;
    int it = 0;
    for (; tile < n_tiles; tile += step, ++it) {
        const int prv = (it + 2) % 3, nxt = (it + 1) % 3, nxt2 = (it + 2) % 3;
        if constexpr (!FUSED) {
            const int g = (tile + 2 * step) * kTM + (int)threadIdx.x;   // the tile after next
            next_src = threadIdx.x < kTM && tile + 2 * step < n_tiles && g < n_rows ? row_src[g] : -1;
        }
        // layer 1, first half: H1^T[n][m] = sum_k W1[n][k] X[m][k] (b1 rides in the depth padding).  Meanwhile: layer 3 of
        // the previous tile's second half (this wavefront's share of w3 . relu(H2) for each row), half a piece per MFMA,
        // and the requests for the next tile's features (after the last tile they fetch row 0, which nobody uses).
        float part0 = 0.f, part1 = 0.f;
        layer_from<kK1 / 16>(acc0, nullptr, w1r, X, kXs, l32, half, [&](int i) {
            if (i == 0) fetch_read(nxt);
            if (i < 16) last_layer_half(acc1, i, w3r, part1);
            if (i >= 2 && !(i & 1)) fetch_issue((i - 2) >> 1);   // pieces 0..9
            if (i == 17) finish_rows(part1, 32);
        });
        // layer 1, second half.  Meanwhile: the first half's ReLU, rounding and stores to H1.
        layer_from<kK1 / 16>(acc1, nullptr, w1r, X + 32 * kXs, kXs, l32, half, [&](int i) {
            if (i == 1) fetch_issue(kXLoads - 2);
            if (i == 2) fetch_issue(kXLoads - 1);
            if (i >= 4 && i < 20 && !(i & 1)) park_hidden(acc0, (i - 4) >> 1, H1, kHs, wave, l32, half);   // the first half's last MFMAs are still running at first
        });
        __syncthreads();   // rows 0..31 of H1 and the previous tile's row outputs complete; X no longer read
        // layer 2, first half: H2^T[n][m] = b2[n] + sum_k W2[n][k] H1[m][k].  Meanwhile: the second half's hidden layer
        // goes to LDS, the source rows of the tile after next are found, and the previous tile's rows are summed (its
        // row outputs and source rows are written again only after the next barrier).
        layer_from<kH / 16>(acc0, b2r, w2r, H1, kHs, l32, half, [&](int i) {
            if (i & 1) find_step(i >> 1, tile + 2 * step);
            else if (i < 16) park_hidden(acc1, i >> 1, H1 + 32 * kHs, kHs, wave, l32, half);
            else sum_step((i - 16) >> 1, prv);   // steps 0..7
        });
        __syncthreads();   // rows 32..63 of H1 complete
        // layer 2, second half.  Meanwhile: layer 3 of the first half, and the next tile's features go to X (free since
        // the first barrier).
        layer_from<kH / 16>(acc1, b2r, w2r, H1 + 32 * kHs, kHs, l32, half, [&](int i) {
            if (!(i & 1)) last_layer_half(acc0, i >> 1, w3r, part0);
            if (i == 1) {
                sum_step(kS, prv);
                find_step(16, 0);
            }
            if (i == 3 && it > 0) sum_store();
            if (i == 5) find_step(17, 0);
            if (i >= 7 && i < 7 + 2 * kXLoads && (i & 1)) park_piece((i - 7) >> 1);
            if (i == 31) finish_rows(part0, 0);
        });
        // the source rows of the tile after next go to the slot last read by the sums above
        if constexpr (FUSED) {
            if (lane < 16) src[nxt2][16 * wave + lane] = next_src;
        } else {
            if (threadIdx.x < kTM) src[nxt2][threadIdx.x] = next_src;
        }
        __syncthreads();   // X(next), the first half's row outputs and the source rows complete
    }
    if (it > 0) {   // the last tile's second half and sums
        float part1 = 0.f;
#pragma unroll
        for (int hp = 0; hp < 16; ++hp) last_layer_half(acc1, hp, w3r, part1);
        finish_rows(part1, 32);
        __syncthreads();
        const int last = (it + 2) % 3;
#pragma unroll
        for (int q = 0; q < 1 + kS; ++q) sum_step(q, last);
        sum_store();
    }
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
        // one launch: a workgroup numbers the rows of its own range of at most kLocalMax candidates; as many workgroups
        // as compute units when the set is large enough to give each of them eight candidates
        int64_t grid = (n_d + 7) / 8 < g_num_cus ? (n_d + 7) / 8 : g_num_cus;
        if (grid * kLocalMax < n_d) grid = (n_d + kLocalMax - 1) / kLocalMax;
        hipLaunchKernelGGL(mlp_kernel<true>, dim3((unsigned)grid), dim3(kThreads), 0, st, feat, row_src, head, n_stmt, (int32_t)n_d, w->W1, w->b1,
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
