// The whole Pattern-aware Transformer of the verify stage (Sec. 4.2): statement branch, self-attention over the
// temporal dataflow blocks, concatenation, linear head.  The paper's figure with the dimensions is lost; the model
// taken here (hidden 256, embedding 64, one attention head and layer with a residual connection, sum pooling, one
// hidden head layer):
//   statement s < n_stmt:  h1 = relu(W1 x_s + b1);  h2 = relu(W2 h1 + b2);          v_s = sum_s h2          (256)
//   block i < n_blk:       e_i = relu(We d_i + be);  q_i, k_i, v_i = Wq e_i, Wk e_i, Wv e_i
//                          a_ij = softmax_j(q_i . k_j / 8),  o_i = sum_j a_ij v_j
//                          z_i = e_i + Wo o_i;                                     v_d = sum_i z_i         (64)
//   head:                  g = relu(Wh [v_s ; v_d] + bh);  y = wo . g + bo
// Every operand of a matrix product is bfloat16 (inputs, e, q, k, v, o, h1, h2, the pooled vectors), accumulation is
// binary32, the softmax is binary32.
//
// Three launches:
//   pacm_stmt_kernel   the two statement layers on the matrix cores, a tile = 8 candidates x 8 statement slots = 64
//                      rows (rows beyond n_stmt are computed and masked: the pooled sum then is a sum over eight
//                      neighbouring lanes); a wavefront owns 64 hidden units and keeps its W1/W2 slices in registers
//   pacm_flow_kernel   the dataflow branch, a wavefront per four candidates (their 32 block slots are one MFMA tile):
//                      embedding, q/k/v, the scores and the output projection on the matrix cores, softmax and the
//                      products with the binary32 attention weights on the vector ALU
//   pacm_head_kernel   the head's hidden layer on the matrix cores (64 candidates per tile) and its output dot product
#include "common.h"
#include "mfma_tile.h"

namespace pruner {
namespace {

using namespace tile;

constexpr int kF = PRUNER_FEAT_DIM;      // 164
constexpr int kS = PRUNER_MAX_STMT;      // 8
constexpr int kH = PRUNER_HIDDEN;        // 256
constexpr int kD = PRUNER_FLOW_DIM;      // 23
constexpr int kT = PRUNER_MAX_BLOCKS;    // 8
constexpr int kE = PRUNER_EMBED;         // 64
constexpr int kU = kH + kE;              // 320: the head's input
constexpr int kTM = 64;                  // rows per tile
constexpr int kK1 = 176;                 // 164 padded to a multiple of the MFMA depth 16
constexpr int kXs = kK1 + 8;             // LDS row strides in bfloat16 elements (rows stay 16-byte aligned)
constexpr int kHs = kH + 8;
constexpr int kUs = kU + 8;
constexpr int kThreads = 256;
constexpr int kF4 = kF / 4;              // float4 per feature row (41)
static_assert(kS == 8 && kT == 8 && kE == 64 && kTM == 64, "the lane arithmetic below assumes these");

__device__ __forceinline__ int clamp8(int v) { return v < 0 ? 0 : v > 8 ? 8 : v; }
__device__ __forceinline__ float bf16_round_f(float x) { return (float)(__bf16)x; }

// This wavefront's 64 rows of a [256][K] bfloat16 matrix as MFMA A operands: lane (l32, half) takes, per 32-row block
// and 16-deep step, the 16 bytes at row 64 wave + 32 nt + l32, depth 16 ks + 8 half.  FULL depth steps only.
template <int KS, int KFULL, typename V>
__device__ __forceinline__ void load_slices(bf16x8 (&wr)[2][KS], const uint16_t* __restrict__ W, int row_elems, int wave, int l32, int half)
{
    typedef V vec_t;
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const uint16_t* r = W + (size_t)(64 * wave + 32 * nt + l32) * row_elems + 8 * half;
#pragma unroll
        for (int ks = 0; ks < KFULL; ++ks) wr[nt][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const vec_t*>(r + 16 * ks));
    }
}

// ---- statement branch ------------------------------------------------------------------------------------------------

__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
pacm_stmt_kernel(const float* __restrict__ feat, const int32_t* __restrict__ n_stmt, int32_t n_d, const uint16_t* __restrict__ W1,
                 const float* __restrict__ b1, const uint16_t* __restrict__ W2, const float* __restrict__ b2, float* __restrict__ v_s)
{
    __shared__ __attribute__((aligned(16))) __bf16 arena[kTM * kXs + kTM * kHs];
    __shared__ __attribute__((aligned(16))) float cst[2][kH];
    __bf16* X = arena;                   // feature tile, bfloat16 [kTM][kXs]
    __bf16* H1 = arena + kTM * kXs;      // first hidden layer of the tile [kTM][kHs]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int grid = gridDim.x;
    const int n_tiles = (n_d + 7) >> 3;
    const int64_t n_rows = (int64_t)n_d * kS;

    // weights: W1's rows end at depth 164, the last step is four entries for half 0 and zeros otherwise
    static_assert(kK1 / 16 == kF / 16 + 1 && kF % 16 == 4, "W1's last depth step holds four entries");
    bf16x8 w1r[2][kK1 / 16], w2r[2][kH / 16];
    typedef u32x4 u32x4_a8 __attribute__((aligned(8)));   // W1's rows are 328 bytes
    load_slices<kK1 / 16, kF / 16, u32x4_a8>(w1r, W1, kF, wave, l32, half);
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const u32x2 tail = *reinterpret_cast<const u32x2*>(W1 + (size_t)(64 * wave + 32 * nt + l32) * kF + 16 * (kF / 16));
        u32x4 last = {0u, 0u, 0u, 0u};
        last[0] = half == 0 ? tail[0] : 0u;
        last[1] = half == 0 ? tail[1] : 0u;
        w1r[nt][kF / 16] = __builtin_bit_cast(bf16x8, last);
    }
    load_slices<kH / 16, kH / 16, u32x4>(w2r, W2, kH, wave, l32, half);
    for (int n = threadIdx.x; n < kH; n += kThreads) {
        cst[0][n] = b1[n];
        cst[1][n] = b2[n];
    }
    // the zero padding of the feature tile (depth 164..183) is written once
    for (int q = threadIdx.x; q < kTM * ((kXs - kF) / 4); q += kThreads) {
        const int r = q / ((kXs - kF) / 4), j = q % ((kXs - kF) / 4);
        *reinterpret_cast<uint2*>(&X[r * kXs + kF + 4 * j]) = make_uint2(0, 0);
    }
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {   // weights in the accumulation registers (see verify_mlp.hip)
#pragma unroll
        for (int ks = 0; ks < kK1 / 16; ++ks) asm volatile("" : "+a"(w1r[nt][ks]));
#pragma unroll
        for (int ks = 0; ks < kH / 16; ++ks) asm volatile("" : "+a"(w2r[nt][ks]));
    }

    // a tile's 64 rows are 64 consecutive feature rows: candidate 8 t + r / 8, statement slot r % 8
    constexpr int kLoads = (kTM * kF4 + kThreads - 1) / kThreads;   // float4 per thread (11)
    f32x4 xr[kLoads];
    auto fetch = [&](int t) {
#pragma unroll
        for (int i = 0; i < kLoads; ++i) {
            int q = threadIdx.x + i * kThreads;
            q = q < kTM * kF4 ? q : kTM * kF4 - 1;
            int64_t row = (int64_t)t * kTM + q / kF4;
            row = row < n_rows ? row : 0;   // rows past the end read row 0; their candidates do not exist
            xr[i] = *reinterpret_cast<const f32x4*>(feat + row * kF + 4 * (q % kF4));
        }
    };
    auto park_piece = [&](int i) {
        int q = threadIdx.x + i * kThreads;
        q = q < kTM * kF4 ? q : kTM * kF4 - 1;
        const f32x2 lo = {xr[i][0], xr[i][1]}, hi = {xr[i][2], xr[i][3]};
        u32x2 o;
        o[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2));
        o[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2));
        *reinterpret_cast<u32x2*>(&X[(q / kF4) * kXs + 4 * (q % kF4)]) = o;
    };
    // Pooled sums of 32 rows: a candidate's eight statement slots are eight neighbouring lanes (slots beyond n_stmt
    // count as zero), summed by exchanges inside the group of eight; all eight lanes then hold the sums, and lane j
    // keeps the j-th run of four hidden units for the store.  One pair of hidden units (u = 0..15) at a time, so that
    // the work fits between the MFMAs of the tile's other half.
    struct Pool {
        int cand;
        bool valid;
        f32x4 out;
    };
    auto pool_begin = [&](Pool& pl, int t, int hh, int count) {
        pl.cand = t * 8 + 4 * hh + (l32 >> 3);
        pl.valid = (l32 & 7) < (pl.cand < n_d ? clamp8(count) : 0);
        pl.out = f32x4{0.f, 0.f, 0.f, 0.f};
    };
    auto group_sum = [](float x) {   // over the eight lanes: neighbours, pairs, then the other four (same order in every lane of a four)
        x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, false));    // quad_perm 1 0 3 2
        x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, false));    // quad_perm 2 3 0 1
        x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, false));   // row_half_mirror
        return x;
    };
    auto pool_unit = [&](Pool& pl, const floatx16(&acc)[2], int u) {
        const int nt = u >> 3, p = u & 7;
        const uint32_t pr = relu_bf16x2(acc[nt][2 * p], acc[nt][2 * p + 1]);
        const float a = group_sum(pl.valid ? __uint_as_float(pr << 16) : 0.f);
        const float b = group_sum(pl.valid ? __uint_as_float(pr & 0xFFFF0000u) : 0.f);
        const bool keep = (l32 & 7) == nt * 4 + (p >> 1);   // units 2 p, 2 p + 1 of block nt lie in run 4 nt + p / 2
        const int e = 2 * (p & 1);
        pl.out[e] = keep ? a : pl.out[e];
        pl.out[e + 1] = keep ? b : pl.out[e + 1];
    };
    auto pool_store = [&](const Pool& pl) {
        const int j = l32 & 7;
        if (pl.cand < n_d) *reinterpret_cast<f32x4*>(v_s + (size_t)pl.cand * kH + 64 * wave + 32 * (j >> 2) + 8 * (j & 3) + 4 * half) = pl.out;
    };
    auto count_of = [&](int t, int hh) {
        const int cand = t * 8 + 4 * hh + (l32 >> 3);
        return cand < n_d ? n_stmt[cand] : 0;
    };

    int tile = blockIdx.x;
    if (tile < n_tiles) {
        fetch(tile);
#pragma unroll
        for (int i = 0; i < kLoads; ++i) park_piece(i);
    }
    __syncthreads();
    // A tile in four stages, each a layer of one half of the rows on the matrix cores with the other half's epilogue
    // between its MFMAs:
    //   1  layer 1, rows 0..31   | pooled sums of the previous tile's rows 32..63; the next tile's features requested
    //   2  layer 1, rows 32..63  | hidden layer 1 of rows 0..31 to LDS
    //   3  layer 2, rows 0..31   | hidden layer 1 of rows 32..63 to LDS
    //   4  layer 2, rows 32..63  | pooled sums of rows 0..31; the next tile's features to LDS
    floatx16 acc0[2], acc1[2];   // rows 0..31 and 32..63
    Pool pool0{}, pool1{};
    bool have_prev = false;
    bias_init(acc0, cst[0], wave, half);
    for (; tile < n_tiles; tile += grid) {
        const bool more = tile + grid < n_tiles;
        int count0 = 0, count1 = 0;
        layer<kK1 / 16>(acc0, w1r, X, kXs, l32, half, [&](int i) {
            if (i == 0) {
                if (more) fetch(tile + grid);
                count0 = count_of(tile, 0);
                count1 = count_of(tile, 1);
            }
            if (i >= 2 && i < 18 && have_prev) pool_unit(pool1, acc1, i - 2);
            if (i == 18 && have_prev) pool_store(pool1);
            if (i == 19) bias_init(acc1, cst[0], wave, half);
        });
        layer<kK1 / 16>(acc1, w1r, X + 32 * kXs, kXs, l32, half, [&](int i) {
            if (i >= 1 && i < 17 && (i & 1)) park_hidden(acc0, (i - 1) >> 1, H1, kHs, wave, l32, half);
            if (i == 19) bias_init(acc0, cst[1], wave, half);
        });
        __syncthreads();   // hidden layer 1 of rows 0..31 complete
        layer<kH / 16>(acc0, w2r, H1, kHs, l32, half, [&](int i) {
            if (i >= 1 && i < 17 && (i & 1)) park_hidden(acc1, (i - 1) >> 1, H1 + 32 * kHs, kHs, wave, l32, half);
            if (i == 20) bias_init(acc1, cst[1], wave, half);
        });
        __syncthreads();   // hidden layer 1 of rows 32..63 complete; X no longer read
        pool_begin(pool0, tile, 0, count0);
        layer<kH / 16>(acc1, w2r, H1 + 32 * kHs, kHs, l32, half, [&](int i) {
            if (i < 16) pool_unit(pool0, acc0, i);
            if (i == 16) pool_store(pool0);
            if (i >= 17 && i < 17 + kLoads && more) park_piece(i - 17);
            if (i == 29) bias_init(acc0, cst[0], wave, half);
        });
        pool_begin(pool1, tile, 1, count1);
        have_prev = true;
        __syncthreads();   // the next tile's features complete; hidden layer 1 may be written again
    }
    if (have_prev) {
#pragma unroll
        for (int u = 0; u < 16; ++u) pool_unit(pool1, acc1, u);
        pool_store(pool1);
    }
}

// ---- dataflow branch -------------------------------------------------------------------------------------------------
// A wavefront works on four candidates at a time: their 4 x 8 block slots are the 32 rows of one MFMA tile.  Embedding,
// the q/k/v projections, the scores Q K^T (a 32 x 32 product of which the four 8 x 8 diagonal blocks are used) and the
// output projection run on the matrix cores with the weights in registers; the softmax and the products with the
// binary32 attention weights stay on the vector ALU.  Slots beyond n_blk are zero rows, masked as keys and in the sum.

constexpr int kFlowWaves = 4;                 // wavefronts (groups of four candidates) per workgroup
constexpr int kFlowThreads = 64 * kFlowWaves;
constexpr int kGroup = 4;                     // candidates per wavefront and round
constexpr int kDk = 32;                       // 23 padded to the MFMA depth
constexpr int kDs = kDk + 8;                  // LDS row strides (bfloat16 elements)
constexpr int kEs = kE + 8;
constexpr int kFlowWaveBytes = (4 * 32 * kEs) * 2 + kGroup * kT * kT * 4;   // Db / Qb / Ob (one after the other in one place), Eb, Kb, Vb, attention weights
static_assert(kDs <= kEs, "the block features fit the place they share with Q and O");
static_assert(2 * (size_t)kFlowWaves * kFlowWaveBytes <= 160 * 1024, "two workgroups per compute unit");
constexpr size_t kFlowLds = (size_t)kFlowWaves * kFlowWaveBytes;
static_assert(kFlowWaveBytes % 16 == 0, "a wavefront's scratch keeps 16-byte alignment");

// Exchanges inside a group of eight neighbouring lanes at the vector ALU's own rate: CTRL 0xB1 brings the neighbour's value
// (lane ^ 1), 0x4E the other pair's (lane ^ 2), 0x141 mirrors the row half (lane 7 - j of the eight, i.e. the other four).
// sum8: after the first two steps the four lanes of a quad hold the quad's sum, so the mirrored lane's value is the other
// quad's sum: the same additions in the same order as exchanges by lane ^ 1, ^ 2, ^ 4.
template <int CTRL> __device__ __forceinline__ float across8(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float sum8(float x)
{
    x += across8<0xB1>(x);
    x += across8<0x4E>(x);
    x += across8<0x141>(x);
    return x;
}

// round to bfloat16 (no ReLU) and store four neighbouring units of row l32: piece = 4 nt + g
__device__ __forceinline__ void park_plain(const floatx16 (&acc)[2], int piece, __bf16* H, int stride, int l32, int half)
{
    const int nt = piece >> 2, g = piece & 3;
    const f32x2 lo = {acc[nt][4 * g + 0], acc[nt][4 * g + 1]}, hi = {acc[nt][4 * g + 2], acc[nt][4 * g + 3]};
    u32x2 o;
    o[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2));
    o[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2));
    *reinterpret_cast<u32x2*>(&H[l32 * stride + 32 * nt + 8 * g + 4 * half]) = o;
}

// Two wavefronts per SIMD (256 registers each, two workgroups' scratch in a compute unit's LDS): a round is a chain of
// dependent stages, and a second wavefront fills the waits of the first.
__global__ void __launch_bounds__(kFlowThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
pacm_flow_kernel(const float* __restrict__ flow, const int32_t* __restrict__ n_blk, int32_t n_d, const uint16_t* __restrict__ We,
                 const float* __restrict__ be, const uint16_t* __restrict__ Wq, const uint16_t* __restrict__ Wk,
                 const uint16_t* __restrict__ Wv, const uint16_t* __restrict__ Wo, float* __restrict__ v_d)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char flow_lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    unsigned char* mine = flow_lds + (size_t)wave * kFlowWaveBytes;
    // Block features (stages 1-2), Q (3-4) and the attention outputs (5-6) take turns in one place: a barrier lies between
    // the last read of one and the first write of the next.
    __bf16* Db = reinterpret_cast<__bf16*>(mine);     // [32][kDs] block features
    __bf16* Qb = Db;                                  // [32][kEs]
    __bf16* Ob = Db;                                  // [32][kEs] attention outputs
    __bf16* Eb = Db + 32 * kEs;                       // [32][kEs] embeddings
    __bf16* Kb = Eb + 32 * kEs;
    __bf16* Vb = Kb + 32 * kEs;
    float* ash = reinterpret_cast<float*>(Vb + 32 * kEs);   // [4][8][8] attention weights a[candidate][i][j]

    // weights as MFMA A operands: lane (l32, half) holds, per 32-unit block and 16-deep step, 8 entries of row 32 nt + l32
    bf16x8 wer[2][kDk / 16], wqr[2][kE / 16], wkr[2][kE / 16], wvr[2][kE / 16], wor[2][kE / 16];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
#pragma unroll
        for (int ks = 0; ks < kDk / 16; ++ks) {
            uint32_t pk[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const int k0 = 16 * ks + 8 * half + 2 * p;
                const uint32_t lo = k0 < kD ? We[(32 * nt + l32) * kD + k0] : 0u, hi = k0 + 1 < kD ? We[(32 * nt + l32) * kD + k0 + 1] : 0u;
                pk[p] = lo | (hi << 16);
            }
            wer[nt][ks] = __builtin_bit_cast(bf16x8, u32x4{pk[0], pk[1], pk[2], pk[3]});
        }
        const size_t row = (size_t)(32 * nt + l32) * kE + 8 * half;
#pragma unroll
        for (int ks = 0; ks < kE / 16; ++ks) {
            wqr[nt][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Wq + row + 16 * ks));
            wkr[nt][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Wk + row + 16 * ks));
            wvr[nt][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Wv + row + 16 * ks));
            wor[nt][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Wo + row + 16 * ks));
        }
    }
    // the embedding's bias waits in LDS (it is read once per round; thirty-two registers held for it would not fit)
    __shared__ __attribute__((aligned(16))) float be_lds[kE];
    if (threadIdx.x < kE) be_lds[threadIdx.x] = be[threadIdx.x];
    __syncthreads();

    const int n_groups = (n_d + kGroup - 1) / kGroup;
    const int stride = gridDim.x * kFlowWaves;
    const int rounds = (n_groups + stride - 1) / stride;   // the same for every wavefront of the launch: barriers stay uniform
    // A group's 32 x 23 block features are 736 contiguous floats: twelve per lane (the last lanes' twelfth lies past the
    // group and reads as 0; so does everything of a group that does not exist).  They are requested a round ahead, after the
    // stage with the most registers in use, and parked at the start of their round.
    constexpr int kPer = (32 * kD + 63) / 64;
    float ahead[kPer];
    int t_ahead[kGroup];
    auto request = [&](int rd) {
        const int64_t c0 = (int64_t)(blockIdx.x * kFlowWaves + wave + rd * stride) * kGroup;
#pragma unroll
        for (int c = 0; c < kGroup; ++c) t_ahead[c] = rd < rounds && c0 + c < n_d ? clamp8(n_blk[c0 + c]) : 0;
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int idx = lane + 64 * i, row = idx / kD;
            const int tc = row < 8 ? t_ahead[0] : row < 16 ? t_ahead[1] : row < 24 ? t_ahead[2] : t_ahead[3];
            ahead[i] = idx < 32 * kD && (row & 7) < tc ? flow[(size_t)c0 * kT * kD + idx] : 0.f;
        }
    };
    request(0);
    for (int rd = 0; rd < rounds; ++rd) {
        const int group = blockIdx.x * kFlowWaves + wave + rd * stride;
        const int cand0 = group * kGroup;
        // block counts of the four candidates (0 for candidates that do not exist)
        int t4[kGroup];
#pragma unroll
        for (int c = 0; c < kGroup; ++c) t4[c] = t_ahead[c];
        const int t_row = l32 < 8 ? t4[0] : l32 < 16 ? t4[1] : l32 < 24 ? t4[2] : t4[3];   // of this lane's row's candidate
        const bool row_valid = (l32 & 7) < t_row;
        // 1. the group's 32 x 23 block features are contiguous; slots beyond the counts become zero rows, and so does depth
        //    23..31 of every row (the place has held Q and O since the last round)
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int idx = lane + 64 * i, row = idx / kD, c = idx - row * kD;
            if (idx < 32 * kD) Db[row * kDs + c] = (__bf16)ahead[i];
        }
        for (int q = lane; q < 32 * (kDk - kD); q += 64) Db[(q / (kDk - kD)) * kDs + kD + q % (kDk - kD)] = (__bf16)0.f;
        __syncthreads();
        // 2. E^T = relu(We D^T + be)
        floatx16 acc_e[2];
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {   // accumulator entry 4 g + e is unit 32 nt + 8 g + 4 half + e
                const f32x4 b4 = *reinterpret_cast<const f32x4*>(&be_lds[32 * nt + 8 * g + 4 * half]);
#pragma unroll
                for (int e = 0; e < 4; ++e) acc_e[nt][4 * g + e] = b4[e];
            }
#pragma unroll
        for (int ks = 0; ks < kDk / 16; ++ks) {
            const bf16x8 fb = *reinterpret_cast<const bf16x8*>(&Db[l32 * kDs + 16 * ks + 8 * half]);
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) acc_e[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wer[nt][ks], fb, acc_e[nt], 0, 0, 0);
        }
#pragma unroll
        for (int piece = 0; piece < 8; ++piece) park_hidden(acc_e, piece, Eb, kEs, 0, l32, half);
        __syncthreads();
        // 3. Q^T, K^T, V^T = W E^T, rounded: one after the other, so that one pair of accumulator blocks is live at a time
        //    (all three at once do not fit beside the weights in a wavefront's 256 registers)
        {
            bf16x8 fe[kE / 16];
#pragma unroll
            for (int ks = 0; ks < kE / 16; ++ks) fe[ks] = *reinterpret_cast<const bf16x8*>(&Eb[l32 * kEs + 16 * ks + 8 * half]);
            auto project = [&](const bf16x8 (&wr)[2][kE / 16], __bf16* dst) {
                floatx16 acc[2];
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[nt][i] = 0.f;
#pragma unroll
                for (int ks = 0; ks < kE / 16; ++ks)
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt) acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[nt][ks], fe[ks], acc[nt], 0, 0, 0);
#pragma unroll
                for (int piece = 0; piece < 8; ++piece) park_plain(acc, piece, dst, kEs, l32, half);
            };
            // (Q shares its place with the block features, which the embedding has finished reading: barrier above)
            project(wqr, Qb);
            project(wkr, Kb);
            project(wvr, Vb);
        }
        __syncthreads();
        // 4. scores: S[n][m] = q_n . k_m for all 32 x 32 row pairs; lane (l32 = m, half) receives n = 8 (i / 4) + 4 half + i % 4
        //    and uses the four n of its own candidate.  Softmax over the candidate's keys = over eight neighbouring lanes.
        {
            floatx16 sc;
#pragma unroll
            for (int i = 0; i < 16; ++i) sc[i] = 0.f;
#pragma unroll
            for (int ks = 0; ks < kE / 16; ++ks) {
                const bf16x8 fq = *reinterpret_cast<const bf16x8*>(&Qb[l32 * kEs + 16 * ks + 8 * half]);
                const bf16x8 fk = *reinterpret_cast<const bf16x8*>(&Kb[l32 * kEs + 16 * ks + 8 * half]);
                sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq, fk, sc, 0, 0, 0);
            }
            const int cl = l32 >> 3, j = l32 & 7;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float s = cl == 0 ? sc[r] : cl == 1 ? sc[4 + r] : cl == 2 ? sc[8 + r] : sc[12 + r];
                s = j < t_row ? s * 0.125f : -__builtin_inff();
                float mx = s;
                mx = fmaxf(mx, across8<0xB1>(mx));
                mx = fmaxf(mx, across8<0x4E>(mx));
                mx = fmaxf(mx, across8<0x141>(mx));
                const float p = j < t_row ? expf(s - mx) : 0.f;
                const float den = sum8(p);
                ash[(cl * kT + 4 * half + r) * kT + j] = t_row > 0 ? p / den : 0.f;
            }
        }
        __syncthreads();
        request(rd + 1);
        // 5. o_i = sum_j a_ij v_j in binary32 (lane = embedding unit), rounded, back to rows
        for (int cl = 0; cl < kGroup; ++cl) {
            float vj[kT];
#pragma unroll
            for (int j2 = 0; j2 < kT; ++j2) vj[j2] = (float)Vb[(cl * kT + j2) * kEs + lane];
#pragma unroll
            for (int i = 0; i < kT; ++i) {
                const f32x4 lo = *reinterpret_cast<const f32x4*>(&ash[(cl * kT + i) * kT]), hi = *reinterpret_cast<const f32x4*>(&ash[(cl * kT + i) * kT + 4]);
                float acc = 0.f;
#pragma unroll
                for (int j2 = 0; j2 < 4; ++j2) acc = __builtin_fmaf(lo[j2], vj[j2], acc);
#pragma unroll
                for (int j2 = 0; j2 < 4; ++j2) acc = __builtin_fmaf(hi[j2], vj[4 + j2], acc);
                Ob[(cl * kT + i) * kEs + lane] = (__bf16)acc;
            }
        }
        __syncthreads();
        // 6. z = e + Wo o; v_d = sum over the candidate's valid blocks = over eight neighbouring lanes
        {
            floatx16 az[2];
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int i = 0; i < 16; ++i) az[nt][i] = 0.f;
#pragma unroll
            for (int ks = 0; ks < kE / 16; ++ks) {
                const bf16x8 fb = *reinterpret_cast<const bf16x8*>(&Ob[l32 * kEs + 16 * ks + 8 * half]);
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) az[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wor[nt][ks], fb, az[nt], 0, 0, 0);
            }
            float sum[2][16];
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    // the rounded embedding of this lane's row for the residual connection, as the embedding stage left it
                    const float e_res = (float)Eb[l32 * kEs + 32 * nt + 8 * (i / 4) + 4 * half + (i % 4)];
                    sum[nt][i] = sum8(row_valid ? e_res + az[nt][i] : 0.f);
                }
            // every lane of the eight holds the sums: lane j stores the j-th run of four units
            const int j = l32 & 7, cand = cand0 + (l32 >> 3);
            f32x4 out = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int gi = 0; gi < 8; ++gi)
#pragma unroll
                for (int e = 0; e < 4; ++e) out[e] = j == gi ? sum[gi >> 2][4 * (gi & 3) + e] : out[e];
            if (cand < n_d) *reinterpret_cast<f32x4*>(v_d + (size_t)cand * kE + 32 * (j >> 2) + 8 * (j & 3) + 4 * half) = out;
        }
        __syncthreads();   // the scratch is written again in the next round
    }
}

// ---- head ------------------------------------------------------------------------------------------------------------

__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
pacm_head_kernel(const float* __restrict__ v_s, const float* __restrict__ v_d, int32_t n_d, const uint16_t* __restrict__ Wh,
                 const float* __restrict__ bh, const uint16_t* __restrict__ wo, float bo, float* __restrict__ y)
{
    __shared__ __attribute__((aligned(16))) __bf16 U[kTM * kUs];   // the tile's concatenated pooled vectors, bfloat16
    __shared__ __attribute__((aligned(16))) float cst[kH];
    __shared__ float red[4][kTM];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int n_tiles = (n_d + kTM - 1) / kTM;

    bf16x8 whr[2][kU / 16];
    load_slices<kU / 16, kU / 16, u32x4>(whr, Wh, kU, wave, l32, half);
    float wor[2][16];   // this lane's output weights, in accumulator order
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int i = 0; i < 16; ++i) wor[nt][i] = __uint_as_float((uint32_t)wo[64 * wave + 32 * nt + 8 * (i / 4) + 4 * half + (i % 4)] << 16);
    for (int n = threadIdx.x; n < kH; n += kThreads) cst[n] = bh[n];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int ks = 0; ks < kU / 16; ++ks) asm volatile("" : "+a"(whr[nt][ks]));
    const auto nothing = [](int) {};
    constexpr int kU4 = kU / 4;   // float4 per row (80)
    // A tile's pooled vectors, twenty float4 per thread, are requested while the tile before is on the matrix cores and
    // parked (rounded to bfloat16) when that tile is done.
    constexpr int kPieces = kTM * kU4 / kThreads;
    static_assert(kTM * kU4 % kThreads == 0, "every thread fetches the same number of pieces");
    f32x4 piece[kPieces];
    auto fetch = [&](int tile) {
#pragma unroll
        for (int i = 0; i < kPieces; ++i) {
            const int q = threadIdx.x + i * kThreads, row = q / kU4, col = q % kU4;
            int cand = tile * kTM + row;
            cand = cand < n_d ? cand : 0;   // rows past the end repeat candidate 0; their outputs are not stored
            piece[i] = col < kH / 4 ? *reinterpret_cast<const f32x4*>(v_s + (size_t)cand * kH + 4 * col)
                                    : *reinterpret_cast<const f32x4*>(v_d + (size_t)cand * kE + 4 * (col - kH / 4));
        }
    };
    if ((int)blockIdx.x < n_tiles) fetch(blockIdx.x);
    for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        __syncthreads();   // cst written (first round); U and red free (later rounds)
#pragma unroll
        for (int i = 0; i < kPieces; ++i) {
            const int q = threadIdx.x + i * kThreads, row = q / kU4, col = q % kU4;
            const f32x2 lo = {piece[i][0], piece[i][1]}, hi = {piece[i][2], piece[i][3]};
            u32x2 o;
            o[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2));
            o[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2));
            *reinterpret_cast<u32x2*>(&U[row * kUs + 4 * col]) = o;
        }
        if (tile + (int)gridDim.x < n_tiles) fetch(tile + gridDim.x);
        __syncthreads();
        floatx16 acc0[2], acc1[2];
        bias_init(acc0, cst, wave, half);
        layer<kU / 16>(acc0, whr, U, kUs, l32, half, nothing);
        bias_init(acc1, cst, wave, half);
        layer<kU / 16>(acc1, whr, U + 32 * kUs, kUs, l32, half, nothing);
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            const floatx16(&acc)[2] = hh ? acc1 : acc0;
            float part = 0.f;
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int p = 0; p < 8; ++p) {
                    const uint32_t pr = relu_bf16x2(acc[nt][2 * p], acc[nt][2 * p + 1]);
                    part = __builtin_fmaf(__uint_as_float(pr << 16), wor[nt][2 * p], part);
                    part = __builtin_fmaf(__uint_as_float(pr & 0xFFFF0000u), wor[nt][2 * p + 1], part);
                }
            part += __shfl_xor(part, 32, 64);
            if (half == 0) red[wave][32 * hh + l32] = part;
        }
        __syncthreads();
        if (threadIdx.x < kTM) {
            const int cand = tile * kTM + threadIdx.x;
            if (cand < n_d) y[cand] = (((red[0][threadIdx.x] + red[1][threadIdx.x]) + red[2][threadIdx.x]) + red[3][threadIdx.x]) + bo;
        }
    }
}

PerDeviceFlag g_flow_ready;   // the dataflow kernel's allowance of dynamic LDS has been raised

}  // namespace

size_t pacm_workspace_bytes(int64_t n_d)
{
    if (n_d < 0) n_d = 0;
    return round_up((size_t)n_d * kH * sizeof(float), 256) + round_up((size_t)n_d * kE * sizeof(float), 256);
}

}  // namespace pruner

using namespace pruner;

extern "C" int pruner_pacm_score(const float* feat, const int32_t* n_stmt, const float* flow, const int32_t* n_blk, int64_t n_d,
                                 const pruner_pacm* w, float* y, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!feat || !n_stmt || !flow || !n_blk || !w || !y || n_d < 0 || n_d > (int64_t)(0x7FFFFFFF / (kS * kF))) return PRUNER_EINVAL;
    if (!w->W1 || !w->b1 || !w->W2 || !w->b2 || !w->We || !w->be || !w->Wq || !w->Wk || !w->Wv || !w->Wo || !w->Wh || !w->bh || !w->wo)
        return PRUNER_EINVAL;
    if (!aligned(feat, 16) || !aligned(flow, 4) || !aligned(n_stmt, 4) || !aligned(n_blk, 4) || !aligned(y, 4) || !aligned(w->W1, 8) ||
        !aligned(w->W2, 16) || !aligned(w->Wh, 16) || !aligned(w->b1, 4) || !aligned(w->b2, 4) || !aligned(w->be, 4) || !aligned(w->bh, 4) ||
        !aligned(w->We, 2) || !aligned(w->Wq, 2) || !aligned(w->Wk, 2) || !aligned(w->Wv, 2) || !aligned(w->Wo, 2) || !aligned(w->wo, 2))
        return PRUNER_EINVAL;
    if (!workspace || !aligned(workspace, 256)) return PRUNER_EWORKSPACE;
    if (workspace_bytes < pacm_workspace_bytes(n_d)) return PRUNER_EWORKSPACE;
    if (n_d == 0) return PRUNER_OK;
    int pacm_cus = 0;
    const int dev = current_device(&pacm_cus);
    if (dev < 0) return PRUNER_EHIP;
    if (!g_flow_ready.get(dev)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&pacm_flow_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFlowLds) !=
            hipSuccess)
            return PRUNER_EHIP;
        g_flow_ready.mark(dev);
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    float* v_s = reinterpret_cast<float*>(ws);
    float* v_d = reinterpret_cast<float*>(ws + round_up((size_t)n_d * kH * sizeof(float), 256));
    const int32_t n = (int32_t)n_d;
    const int64_t stmt_tiles = (n_d + 7) / 8, flow_groups = (n_d + kGroup * kFlowWaves - 1) / (kGroup * kFlowWaves), head_tiles = (n_d + kTM - 1) / kTM;
    hipLaunchKernelGGL(pacm_stmt_kernel, dim3((unsigned)(stmt_tiles < pacm_cus ? stmt_tiles : pacm_cus)), dim3(kThreads), 0, st, feat, n_stmt,
                       n, w->W1, w->b1, w->W2, w->b2, v_s);
    PRUNER_LAUNCH_CHECK();
    hipLaunchKernelGGL(pacm_flow_kernel, dim3((unsigned)(flow_groups < 2 * pacm_cus ? flow_groups : 2 * pacm_cus)), dim3(kFlowThreads), kFlowLds, st, flow,
                       n_blk, n, w->We, w->be, w->Wq, w->Wk, w->Wv, w->Wo, v_d);
    PRUNER_LAUNCH_CHECK();
    hipLaunchKernelGGL(pacm_head_kernel, dim3((unsigned)(head_tiles < pacm_cus ? head_tiles : pacm_cus)), dim3(kThreads), 0, st, v_s, v_d, n,
                       w->Wh, w->bh, w->wo, w->bo, y);
    PRUNER_LAUNCH_CHECK();
    return PRUNER_OK;
}
