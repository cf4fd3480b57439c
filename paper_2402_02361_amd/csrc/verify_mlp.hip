// Verify stage: statement-feature branch of the learned cost model on the drafted candidates
// (Sec. 4.2, "Pattern-aware Transformer": statement features -> linear layers -> summation over statements).
//
//   y(c,s)   = w3 . relu(W2 relu(W1 x(c,s) + b1) + b2) + b3          164 -> 256 -> 256 -> 1
//   vscore_c = sum over s < n_stmt[c] of y(c,s)
//
// The valid statement rows get consecutive row numbers (exclusive scan of n_stmt), so the matrix cores never see
// padding rows.  Workgroup b of G owns the groups of neighbouring candidates number b, b + G, b + 2 G, ...
// (interleaved, so that every workgroup gets the same mix when the set is ordered by subgraph and subgraphs differ in
// their statement counts; eight to sixty-four at a time, so that a tile's feature rows lie close together in memory) and numbers the rows of
// its own candidates itself, in LDS, while its weights arrive: one launch, no workspace traffic, no pass over the whole
// set.  Its rows form tiles of exactly 64; a candidate whose rows straddle two tiles is finished in the second one, the
// first tile's part of its sum being carried over (the workgroup takes its tiles in order), so every candidate is
// summed in statement order and stored by exactly one thread (no atomics, no clearing pass).
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
//                  candidate are added in statement order by the lane of its first row.
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
constexpr int kLocalCap = 2048;            // most candidates one workgroup takes (their running row counts and the table of its rows sit in LDS)
constexpr int kGroupMin = 8, kGroupMax = 64;   // neighbouring candidates that go to one workgroup together

__device__ __forceinline__ int32_t clamp_stmt(int32_t v) { return v < 0 ? 0 : v > kS ? kS : v; }

// ---- mlp_kernel ----------------------------------------------------------------------------------------------------

// The last layer (w3 . relu(H2) per row) runs on the matrix cores too, chained onto the second layer's result.  A lane
// holds 16 units of its row per 32-unit block (accumulator register i = unit 8 (i/4) + 4 half + i%4); rounded to bfloat16
// in pairs, registers 8 hq .. 8 hq + 7 of a block are, as they stand, the B operand of one 32x32x16 MFMA whose depth index
// (half, j) means unit 16 hq + 8 (j/4) + 4 half + j%4 of the block: any numbering of the depth will do as long as the A
// operand uses the same one.  The A operand is w3 in that numbering in row 0 and zero elsewhere, so row 0 of the product
// (register 0 of lanes 0..31) is the wavefront's share of the dot product for the 32 rows: four MFMAs per 32 rows take
// the place of 128 vector instructions (unpacking and FMAs), which is what the loop is short of.
__device__ __forceinline__ void last_layer_pack(const floatx16 (&acc)[2], int pair, uint32_t (&pk)[16])
{
    const int nt = pair >> 3, j = pair & 7;
    pk[pair] = relu_bf16x2(acc[nt][2 * j], acc[nt][2 * j + 1]);
}
__device__ __forceinline__ void last_layer_mfma(floatx16& acc3, int q, const bf16x8 (&w3f)[4], const uint32_t (&pk)[16])
{
    const u32x4 b = {pk[4 * q], pk[4 * q + 1], pk[4 * q + 2], pk[4 * q + 3]};
    floatx16 zero;
#pragma unroll
    for (int i = 0; i < 16; ++i) zero[i] = 0.f;
    acc3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w3f[q], __builtin_bit_cast(bf16x8, b), q == 0 ? zero : acc3, 0, 0, 0);
}

__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
mlp_kernel(const float* __restrict__ feat, const int32_t* __restrict__ n_stmt, int32_t n_d, int32_t kGroup, const uint16_t* __restrict__ W1,
           const float* __restrict__ b1, const uint16_t* __restrict__ W2, const float* __restrict__ b2, const uint16_t* __restrict__ w3, float b3,
           float* __restrict__ vscore)
{
    // The tile buffers.
    __shared__ __attribute__((aligned(16))) __bf16 arena[kTM * kXs + kTM * kHs];
    __shared__ float red[4][kTM];        // last-layer partial sums per wavefront
    __bf16* X = arena;                   // feature tile, bfloat16 [kTM][kXs]
    __bf16* H1 = arena + kTM * kXs;      // first hidden layer of the tile [kTM][kHs]

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int step = 1;   // the workgroup walks the tiles of its own candidates

    // Row numbering.  The workgroup owns the candidate groups b, b + G, ...: its candidate l is global_of(l), l < n_local;
    // before[l] = valid rows of its candidates 0..l-1; its tile t holds its rows 64 t .. 64 t + 63.
    extern __shared__ uint32_t dyn[];
    const int n_groups = (n_d + kGroup - 1) / kGroup, my_first = (int)blockIdx.x, group_stride = (int)gridDim.x;
    const int my_groups = my_first < n_groups ? (n_groups - my_first + group_stride - 1) / group_stride : 0;
    // (the set's last group may be short, and it is this workgroup's last one if it is this workgroup's at all)
    const bool owns_last = my_groups > 0 && my_first + (my_groups - 1) * group_stride == n_groups - 1;
    const int n_local = my_groups * kGroup - (owns_last ? n_groups * kGroup - n_d : 0);
    auto global_of = [&](int l) -> int { return kGroup * ((l / kGroup) * group_stride + my_first) + l % kGroup; };
    uint32_t* before = dyn;                                                  // [n_local + 1]
    int32_t* row_tab = reinterpret_cast<int32_t*>(dyn + (n_local + 1));      // [rows of this workgroup]: what each row is (see below)
    __shared__ float carry_slot;                 // the part of a candidate's sum that lies in the tile before
    __shared__ uint32_t scan_tot[4];
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
        }
    }
    // the second layer's bias and the last layer's weights pass through LDS (one element per thread) on their way to the
    // registers of the lanes that use them
    __shared__ __attribute__((aligned(16))) float b2_lds[kH];
    __shared__ __attribute__((aligned(16))) uint16_t w3_lds[kH];
    b2_lds[threadIdx.x] = b2[threadIdx.x];
    w3_lds[threadIdx.x] = w3[threadIdx.x];
    static_assert(kThreads == kH, "one thread per hidden unit");

    int n_rows, n_tiles;
    {
        for (int l = threadIdx.x; l < n_local; l += kThreads) {
            const int c = global_of(l);
            const uint32_t v = (uint32_t)clamp_stmt(n_stmt[c]);
            before[l] = v;
            if (v == 0) vscore[c] = 0.f;   // a candidate without rows scores 0
        }
        __syncthreads();
        // thread t owns a run of `per` candidates (odd: neighbouring threads then start in different banks)
        const int per = ((n_local + kThreads - 1) / kThreads) | 1;
        const int c_lo = (int)threadIdx.x * per < n_local ? (int)threadIdx.x * per : n_local;
        const int c_hi = c_lo + per < n_local ? c_lo + per : n_local;
        uint32_t mine = 0;
        for (int c = c_lo; c < c_hi; ++c) mine += before[c];
        const uint32_t incl = wave_inclusive_sum(mine);
        if (lane == 63) scan_tot[wave] = incl;
        __syncthreads();
        uint32_t run = incl - mine, total = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            run += w < wave ? scan_tot[w] : 0u;
            total += scan_tot[w];
        }
        for (int c = c_lo; c < c_hi; ++c) {
            const uint32_t v = before[c];
            before[c] = run;
            run += v;
        }
        if (threadIdx.x == 0) before[n_local] = total;
        n_rows = (int)total;
        n_tiles = (n_rows + kTM - 1) / kTM;
        __syncthreads();
    }
    // What a row is: ((candidate * 8 + statement) << 1) | (the candidate's last row).  The table of this workgroup's rows:
    // every candidate writes its own entries.
    for (int l = threadIdx.x; l < n_local; l += kThreads) {
        const uint32_t at = before[l], cnt = before[l + 1] - at;
        const uint32_t g = (uint32_t)global_of(l) * kS;
        for (uint32_t st = 0; st < cnt; ++st) row_tab[at + st] = (int32_t)(((g + st) << 1) | (st + 1 == cnt ? 1u : 0u));
    }
    __syncthreads();
    auto row_of = [&](int t, int r) -> int {   // row r of tile t, or -1 before the first and past the last (branch-free)
        const int R = t * kTM + r;
        const bool there = R >= 0 && R < n_rows;
        const int v = row_tab[there ? R : 0];
        return there ? v : -1;
    };

    int tile = 0;
    // The tile's features, fetched in twelve pieces per thread: eight threads share a row and take every eighth float4 of
    // it; thread t serves rows t/8 and t/8 + 32.  A piece is requested (source row -> registers) and much later
    // converted and stored to X; rows past the end read row 0 (their outputs are never used), and pieces past a row's
    // end repeat its last float4 and are stored beyond the depth the MFMAs read.  One load per piece, nothing between
    // the loads waits, and the pieces can be issued one by one between MFMAs.
    f32x4 xr[kXLoads];
    int fetch_src[kXPass];
    const int f_sub = threadIdx.x & (kRowThreads - 1), f_row = threadIdx.x / kRowThreads;
    auto fetch_read = [&](int t) {
#pragma unroll
        for (int ps = 0; ps < kXPass; ++ps) fetch_src[ps] = row_of(t, f_row + ps * (kThreads / kRowThreads));
    };
    auto fetch_issue = [&](int i) {
        const int ps = i / kXCols, col = f_sub + kRowThreads * (i % kXCols);
        const int sr = fetch_src[ps] >> 1;   // candidate * 8 + statement (-1 past the end)
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
        fetch_read(tile);
#pragma unroll
        for (int i = 0; i < kXLoads; ++i) fetch_issue(i);
    }

    // The second layer's matrix is requested after the first tile's features: it is not needed before the first tile's
    // second layer, and loads return in the order of their requests.
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const uint16_t* r2 = W2 + (size_t)(64 * wave + 32 * nt + l32) * kH + 8 * half;
#pragma unroll
        for (int ks = 0; ks < kH / 16; ++ks) w2r[nt][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(r2 + 16 * ks));
    }
    // The weights live in the accumulation registers (which MFMAs read as well as any), so that the ordinary vector
    // registers are left to the accumulators: the vector ALU reads those without a copy.  (This also waits for W1; the
    // second layer's matrix is pinned there where the loop first uses it.)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int ks = 0; ks < kK1 / 16; ++ks) asm volatile("" : "+a"(w1r[nt][ks]));
    // The second layer's bias of this lane's hidden units stays in registers, in accumulator order: the layer's first
    // MFMAs take it as their addend.  So do the last layer's weights, widened to binary32.  (b2_lds and w3_lds are complete:
    // the row numbering above went through barriers.)
    floatx16 b2r[2];
    bf16x8 w3f[4];   // fragment q = (block nt = q / 2, registers 8 hq .. 8 hq + 7 with hq = q % 2)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const f32x4 b = *reinterpret_cast<const f32x4*>(&b2_lds[64 * wave + 32 * nt + 8 * g + 4 * half]);
#pragma unroll
            for (int j = 0; j < 4; ++j) b2r[nt][4 * g + j] = b[j];
        }
#pragma unroll
        for (int hq = 0; hq < 2; ++hq) {
            const int n0 = 64 * wave + 32 * nt + 16 * hq + 4 * half;
            const u32x2 lo = *reinterpret_cast<const u32x2*>(&w3_lds[n0]), hi = *reinterpret_cast<const u32x2*>(&w3_lds[n0 + 8]);
            u32x4 f = {lo[0], lo[1], hi[0], hi[1]};
#pragma unroll
            for (int e = 0; e < 4; ++e) f[e] = l32 == 0 ? f[e] : 0u;
            w3f[2 * nt + hq] = __builtin_bit_cast(bf16x8, f);
        }
    }
    asm volatile("" : "+a"(w3f[0]), "+a"(w3f[1]), "+a"(w3f[2]), "+a"(w3f[3]));

    // the padding of the feature tile (depth 164..183) is written once: 1, 1, 1 (times the three pieces of b1), then zeros
    for (int q = threadIdx.x; q < kTM * ((kXs - kF) / 4); q += kThreads) {
        const int r = q / ((kXs - kF) / 4), j = q % ((kXs - kF) / 4);
        *reinterpret_cast<uint2*>(&X[r * kXs + kF + 4 * j]) = j == 0 ? make_uint2(0x3F803F80u, 0x00003F80u) : make_uint2(0, 0);
    }

    if (tile < n_tiles) {   // the first tile's features were requested before the weights
#pragma unroll
        for (int i = 0; i < kXLoads; ++i) park_piece(i);
        fetch_read(tile + step);   // and the second tile's are on their way when the loop begins
#pragma unroll
        for (int i = 0; i < kXLoads; ++i) fetch_issue(i);
    }
    __syncthreads();

    // Sums over statements, for tile t (its row outputs sit in red), in nine
    // branch-free steps (so that they can be issued between MFMAs): wavefront w owns rows 16w .. 16w+15 and looks at the
    // seven rows after them as well; the lane of a candidate's first row in the tile adds the candidate's rows in
    // statement order.
    float sum_y = 0.f, sum_total = 0.f, sum_p[4] = {0.f, 0.f, 0.f, 0.f}, sum_oy = 0.f, sum_carry = 0.f;
    int sum_sr = -1, sum_prev = -1, sum_cand = -1, sum_okey = -1, sum_done = 0;
    // (the exchange of step q is asked for in step q - 1 and used in step q: a step never waits for its own exchange)
    auto sum_step = [&](int q, int t) {
        const int r_raw = 16 * wave + lane;
        const bool in = lane < 16 + kS - 1 && r_raw < kTM;
        const int r = in ? r_raw : kTM - 1;
        if (q == 0) {
            sum_sr = row_of(t, r);
            sum_prev = row_of(t, r > 0 ? r - 1 : 0);
            sum_carry = carry_slot;
#pragma unroll
            for (int w = 0; w < 4; ++w) sum_p[w] = red[w][r];
        } else if (q == 1) {
            sum_sr = in ? sum_sr : -1;
            sum_prev = r > 0 ? sum_prev >> 4 : -2;
            sum_cand = sum_sr >> 4;   // -1 for rows past the end
            sum_done = sum_sr & 1;    // the candidate's last row is among the rows added so far
            sum_y = (((sum_p[0] + sum_p[1]) + sum_p[2]) + sum_p[3]) + b3;
            // a candidate that began in the tile before continues in row 0: its earlier rows' sum comes first
            sum_total = (r == 0 && ((sum_sr >> 1) & (kS - 1)) != 0) ? sum_carry + sum_y : sum_y;
        } else {
            const int j = q - 1;   // 1 .. 7: the row j places further on
            const bool same = (sum_okey >> 4) == sum_cand && lane + j < 64;
            sum_total = same ? sum_total + sum_oy : sum_total;
            sum_done |= same ? (sum_okey & 1) : 0;
            asm volatile("" : "+v"(sum_total));   // (keeps the addition in this step)
        }
        if (q >= 1 && q < kS) {
            sum_oy = __shfl_down(sum_y, q, 64);
            sum_okey = __shfl_down(sum_sr, q, 64);
        }
    };
    auto sum_store = [&]() {
        if (lane < 16 && sum_sr >= 0 && sum_prev != sum_cand) {
            if (sum_done) vscore[sum_cand] = sum_total;
            else carry_slot = sum_total;   // the one candidate that runs on into the next tile
        }
    };
    // A tile's two halves (rows 0..31: acc0, rows 32..63: acc1) run half a layer apart, the second half's last layer and
    // the sums over statements reaching into the next iteration; everything that is not an MFMA is issued in the gaps
    // between MFMAs (about six vector instructions fit in the shadow of one MFMA).  A layer's first MFMAs overwrite
    // their accumulator (addend: zero, or the second layer's bias), which its last reader has left by then.
    auto finish_rows = [&](const floatx16& acc3, int first_row) {   // the last layer's partial sums of 32 rows -> red
        if (half == 0) red[wave][first_row + l32] = acc3[0];
    };
    floatx16 y0, y1;        // last-layer products of the tile's two halves (row 0 of each is used)
    uint32_t pk[16];        // a half's second hidden layer as bfloat16 pairs
#pragma unroll
    for (int i = 0; i < 16; ++i) y0[i] = y1[i] = 0.f;
    floatx16 acc0[2], acc1[2];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc0[nt][i] = acc1[nt][i] = 0.f;
    int it = 0;
    for (; tile < n_tiles; tile += step, ++it) {
        // At this point X holds this tile's rows and the next tile's rows are on their way to registers.
        // layer 1, first half: H1^T[n][m] = sum_k W1[n][k] X[m][k] (b1 rides in the depth padding).  Meanwhile: layer 3 of
        // the previous tile's second half (this wavefront's share of w3 . relu(H2) for each row: rounding in the gaps,
        // four MFMAs of its own).
        layer_from<kK1 / 16>(acc0, nullptr, w1r, X, kXs, l32, half, [&](int i) {
            if (i < 8) {   // two pairs per MFMA, a last-layer MFMA after every four pairs
                last_layer_pack(acc1, 2 * i, pk);
                last_layer_pack(acc1, 2 * i + 1, pk);
                if (i & 1) last_layer_mfma(y1, i >> 1, w3f, pk);
            }
            if (i == 13) finish_rows(y1, 32);
        });
        // layer 1, second half.  Meanwhile: the first half's ReLU, rounding and stores to H1.
        layer_from<kK1 / 16>(acc1, nullptr, w1r, X + 32 * kXs, kXs, l32, half, [&](int i) {
            if (i >= 4 && i < 20 && !(i & 1)) park_hidden(acc0, (i - 4) >> 1, H1, kHs, wave, l32, half);   // the first half's last MFMAs are still running at first
        });
        __syncthreads();   // rows 0..31 of H1 and the previous tile's row outputs complete; X no longer read
        // layer 2, first half: H2^T[n][m] = b2[n] + sum_k W2[n][k] H1[m][k].  Meanwhile: the second half's hidden layer
        // goes to LDS, the next tile's rows go to X, and the previous tile's rows are summed (its row outputs are written
        // again only after the next barrier).
        // (no instruction: the register class, and in the first tile the wait for the matrix)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
            asm volatile("" : "+a"(w2r[nt][0]), "+a"(w2r[nt][1]), "+a"(w2r[nt][2]), "+a"(w2r[nt][3]), "+a"(w2r[nt][4]), "+a"(w2r[nt][5]),
                              "+a"(w2r[nt][6]), "+a"(w2r[nt][7]), "+a"(w2r[nt][8]), "+a"(w2r[nt][9]), "+a"(w2r[nt][10]), "+a"(w2r[nt][11]),
                              "+a"(w2r[nt][12]), "+a"(w2r[nt][13]), "+a"(w2r[nt][14]), "+a"(w2r[nt][15]));
        static_assert(kH / 16 == 16, "the second layer's sixteen depth steps are listed above");
        layer_from<kH / 16>(acc0, b2r, w2r, H1, kHs, l32, half, [&](int i) {
            if (i & 1) {
                if (i >= 2 * (kH / 16 - kXLoads)) park_piece((i - 2 * (kH / 16 - kXLoads)) >> 1);   // as late as the layer allows: the rows have far to come
                return;
            }
            if (i < 16) park_hidden(acc1, i >> 1, H1 + 32 * kHs, kHs, wave, l32, half);
            else sum_step((i - 16) >> 1, tile - step);   // steps 0..7
        });
        __syncthreads();   // rows 32..63 of H1 and X (the next tile's rows) complete
        // layer 2, second half.  Meanwhile: layer 3 of the first half, the end of the previous tile's sums, and the
        // requests for the rows of the tile after next (after the last tile they fetch row 0, which nobody uses).
        // Nothing written here is read before the next iteration's first barrier, so none is needed at its end.
        layer_from<kH / 16>(acc1, b2r, w2r, H1 + 32 * kHs, kHs, l32, half, [&](int i) {
            if (!(i & 1) && i < 16) {
                last_layer_pack(acc0, i, pk);
                last_layer_pack(acc0, i + 1, pk);
            }
            if ((i & 3) == 3 && i < 16) last_layer_mfma(y0, i >> 2, w3f, pk);
            if (i == 0) fetch_read(tile + 2 * step);
            if ((i & 1) && i < 2 * kXLoads) fetch_issue(i >> 1);
            if (i == 17) sum_step(kS, tile - step);
            if (i == 19 && it > 0) sum_store();
            if (i == 25) finish_rows(y0, 0);
        });
    }
    if (it > 0) {   // the last tile's second half and sums
#pragma unroll
        for (int pair = 0; pair < 16; ++pair) last_layer_pack(acc1, pair, pk);
#pragma unroll
        for (int q = 0; q < 4; ++q) last_layer_mfma(y1, q, w3f, pk);
        finish_rows(y1, 32);
        __syncthreads();
        const int last = tile - step;
#pragma unroll
        for (int q = 0; q < 1 + kS; ++q) sum_step(q, last);
        sum_store();
    }
}

PerDeviceFlag g_lds_ready;   // the kernel's allowance of dynamic LDS (the row numbers of a workgroup's candidates) has been raised

size_t numbering_bytes(int64_t per_group)   // LDS for the running row counts and the row table of per_group candidates
{
    return round_up((size_t)(per_group + 1) * 4 + (size_t)per_group * kS * 4, 16);
}

}  // namespace

// (nothing of the verify stage lives in the workspace any more; a caller still passes one, for the boundary's sake)
size_t verify_workspace_bytes(int64_t n_d)
{
    (void)n_d;
    return 256;
}

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
    if (workspace_bytes < verify_workspace_bytes(n_d)) return PRUNER_EWORKSPACE;
    if (n_d == 0) return PRUNER_OK;

    int num_cus = 0;
    const int dev = current_device(&num_cus);
    if (dev < 0) return PRUNER_EHIP;
    if (!g_lds_ready.get(dev)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&mlp_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)numbering_bytes(kLocalCap)) != hipSuccess)
            return PRUNER_EHIP;
        g_lds_ready.mark(dev);
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    // One launch per kLocalCap x (compute units) candidates (2 M on this part): as many workgroups as compute units once the
    // set gives each of them a group of eight candidates; workgroup b takes groups b, b + G, b + 2 G, ... of the launch's range.
    const int64_t per_launch = (int64_t)kLocalCap * num_cus;
    for (int64_t c0 = 0; c0 < n_d; c0 += per_launch) {
        const int64_t n = n_d - c0 < per_launch ? n_d - c0 : per_launch;
        const int64_t grid = (n + 7) / 8 < num_cus ? (n + 7) / 8 : num_cus;
        // groups of 8 candidates, or more (up to 64) once a workgroup gets at least eight groups of that size: a tile's
        // feature rows then come from fewer places
        int32_t group = kGroupMin;
        while (group < kGroupMax && n / (2 * group) >= 8 * grid) group *= 2;
        const int64_t groups = (n + group - 1) / group;
        const size_t dyn_bytes = numbering_bytes((groups + grid - 1) / grid * group);
        hipLaunchKernelGGL(mlp_kernel, dim3((unsigned)grid), dim3(kThreads), dyn_bytes, st, feat + (size_t)c0 * kS * kF, n_stmt + c0, (int32_t)n, group,
                           w->W1, w->b1, w->W2, w->b2, w->w3, w->b3, vscore + c0);
        PRUNER_LAUNCH_CHECK();
    }
    return PRUNER_OK;
}
