// Verify stage: statement-feature branch of the learned cost model on the drafted candidates
// (Sec. 4.2, "Pattern-aware Transformer": statement features -> linear layers -> summation over statements).
//
//   y(c,s)   = w3 . relu(W2 relu(W1 x(c,s) + b1) + b2) + b3          164 -> 256 -> 256 -> 1
//   vscore_c = sum over s < n_stmt[c] of y(c,s)
//
// Three launches:
//   rows_kernel    exclusive scan of n_stmt: the valid statement rows of all candidates get consecutive row
//                  numbers, so the matrix cores never see padding rows;
//   mlp_kernel     persistent workgroups (one per CU, 4 wavefronts).  Wavefront w owns hidden units
//                  [64w, 64w+64) of both layers and keeps its slices of W1 and W2 in registers for the whole
//                  launch; feature rows stream through LDS 64 at a time as bfloat16.  Layers are computed
//                  transposed (H^T = W X^T) with v_mfma_f32_32x32x16_bf16, so that one lane holds 16 hidden units
//                  of ONE row: bias is the accumulator's initial value, ReLU and the bfloat16 rounding are
//                  lane-local, and the last layer's dot product with w3 is a lane-local sum plus one cross-lane add.
//                  Hidden activations never leave the CU.
//   sum_kernel     per candidate, the rows' outputs added in statement order.
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

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

struct Head {
    int32_t n_rows;   // valid statement rows in total
    int32_t pad[3];
};

// ---- rows_kernel: compact numbering of the valid rows ------------------------------------------------------------

__global__ void __launch_bounds__(1024) rows_kernel(const int32_t* __restrict__ n_stmt, int64_t n_d, int32_t* __restrict__ row_off /* [n_d+1] */,
                                                    int32_t* __restrict__ row_src /* [n_d*8] */, Head* __restrict__ head)
{
    __shared__ int32_t wave_tot[16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int32_t carry = 0;
    for (int64_t base = 0; base < n_d; base += 1024) {
        const int64_t c = base + threadIdx.x;
        int32_t v = c < n_d ? n_stmt[c] : 0;
        v = v < 0 ? 0 : v > kS ? kS : v;
        int32_t incl = v;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int32_t up = __shfl_up(incl, off, 64);
            if (lane >= off) incl += up;
        }
        __syncthreads();
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        int32_t before = 0, all = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const int32_t t = wave_tot[w];
            before += w < wave ? t : 0;
            all += t;
        }
        const int32_t first = carry + before + incl - v;
        if (c < n_d) {
            row_off[c] = first;
            for (int s = 0; s < v; ++s) row_src[first + s] = (int32_t)(c * kS + s);
        }
        carry += all;
    }
    if (threadIdx.x == 0) {
        row_off[n_d] = carry;
        head->n_rows = carry;
    }
}

// ---- mlp_kernel ----------------------------------------------------------------------------------------------------

__device__ __forceinline__ bf16x8 load_w8(const uint16_t* __restrict__ row, int k0, int k_end)
{
    // eight consecutive bfloat16 weights row[k0 .. k0+7]; entries at or beyond k_end read as zero.  k0 is a multiple
    // of 8 and rows are 8-byte aligned.
    union {
        bf16x8 v;
        uint2 h[2];
    } u;
    u.h[0] = k0 + 4 <= k_end ? *reinterpret_cast<const uint2*>(row + k0) : make_uint2(0, 0);
    u.h[1] = k0 + 8 <= k_end ? *reinterpret_cast<const uint2*>(row + k0 + 4) : make_uint2(0, 0);
    return u.v;
}

__device__ __forceinline__ float bf16_round(float x) { return (float)(__bf16)x; }

__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
mlp_kernel(const float* __restrict__ feat, const int32_t* __restrict__ row_src, const Head* __restrict__ head,
           const uint16_t* __restrict__ W1, const float* __restrict__ b1, const uint16_t* __restrict__ W2, const float* __restrict__ b2,
           const uint16_t* __restrict__ w3, float b3, float* __restrict__ y /* [rows] */)
{
    __shared__ __attribute__((aligned(16))) __bf16 X[kTM * kXs];    // feature tile, bfloat16
    __shared__ __attribute__((aligned(16))) __bf16 H1[kTM * kHs];   // first hidden layer of the tile
    __shared__ float red[4][kTM];                                   // last-layer partial sums per wavefront

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int n_rows = head->n_rows;
    const int n_tiles = (n_rows + kTM - 1) / kTM;

    // This wavefront's weights.  As the A operand of a 32x32x16 MFMA, lane (l32, half) supplies hidden unit
    // n = base + l32 and the eight depth entries 8*half .. 8*half+7 of the 16-deep step.
    bf16x8 w1r[2][kK1 / 16], w2r[2][kH / 16];
    float bias1[2][16], bias2[2][16], w3f[2][16];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const int n = 64 * wave + 32 * nt + l32;
#pragma unroll
        for (int ks = 0; ks < kK1 / 16; ++ks) w1r[nt][ks] = load_w8(W1 + (size_t)n * kF, 16 * ks + 8 * half, kF);
#pragma unroll
        for (int ks = 0; ks < kH / 16; ++ks) w2r[nt][ks] = load_w8(W2 + (size_t)n * kH, 16 * ks + 8 * half, kH);
        // accumulator register i of a 32x32 result holds hidden unit 8*(i/4) + 4*half + i%4 of the tile
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int nn = 64 * wave + 32 * nt + 8 * (i / 4) + 4 * half + (i % 4);
            bias1[nt][i] = b1[nn];
            bias2[nt][i] = b2[nn];
            w3f[nt][i] = __uint_as_float((uint32_t)w3[nn] << 16);
        }
    }

    for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int row0 = tile * kTM;
        __syncthreads();  // the previous tile's readers of X, H1 and red are done

        // stage the tile's feature rows: binary32 in HBM -> bfloat16 in LDS, depth padded with zeros
        for (int q = threadIdx.x; q < kTM * (kXs / 4); q += kThreads) {
            const int r = q / (kXs / 4), j = q % (kXs / 4);
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row0 + r < n_rows && j < kF / 4) v = *reinterpret_cast<const float4*>(feat + (size_t)row_src[row0 + r] * kF + 4 * j);
            bf16x4 o;
            o[0] = (__bf16)v.x;
            o[1] = (__bf16)v.y;
            o[2] = (__bf16)v.z;
            o[3] = (__bf16)v.w;
            *reinterpret_cast<bf16x4*>(&X[r * kXs + 4 * j]) = o;
        }
        __syncthreads();

        // layer 1: H1^T[n][m] = b1[n] + sum_k W1[n][k] X[m][k]
        floatx16 acc[2][2];
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[nt][mt][i] = bias1[nt][i];
#pragma unroll
        for (int ks = 0; ks < kK1 / 16; ++ks) {
            bf16x8 xb[2];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) xb[mt] = *reinterpret_cast<const bf16x8*>(&X[(32 * mt + l32) * kXs + 16 * ks + 8 * half]);
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) acc[nt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1r[nt][ks], xb[mt], acc[nt][mt], 0, 0, 0);
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
        __syncthreads();

        // layer 2: H2^T[n][m] = b2[n] + sum_k W2[n][k] H1[m][k]
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[nt][mt][i] = bias2[nt][i];
#pragma unroll
        for (int ks = 0; ks < kH / 16; ++ks) {
            bf16x8 hb[2];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) hb[mt] = *reinterpret_cast<const bf16x8*>(&H1[(32 * mt + l32) * kHs + 16 * ks + 8 * half]);
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) acc[nt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w2r[nt][ks], hb[mt], acc[nt][mt], 0, 0, 0);
        }

        // layer 3: this wavefront's share of w3 . relu(H2) for each row
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            float part = 0.f;
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int i = 0; i < 16; ++i) part += w3f[nt][i] * bf16_round(fmaxf(acc[nt][mt][i], 0.f));
            part += __shfl_xor(part, 32, 64);
            if (half == 0) red[wave][32 * mt + l32] = part;
        }
        __syncthreads();
        if (threadIdx.x < kTM && row0 + threadIdx.x < n_rows) {
            const int r = threadIdx.x;
            y[row0 + r] = (((red[0][r] + red[1][r]) + red[2][r]) + red[3][r]) + b3;
        }
    }
}

// ---- sum_kernel: statements of a candidate added in order -------------------------------------------------------------

__global__ void __launch_bounds__(256) sum_kernel(const float* __restrict__ y, const int32_t* __restrict__ row_off, int64_t n_d,
                                                  float* __restrict__ vscore)
{
    const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (c >= n_d) return;
    const int32_t lo = row_off[c], hi = row_off[c + 1];
    float total = 0.f;
    for (int32_t r = lo; r < hi; ++r) total = total + y[r];
    vscore[c] = total;
}

struct Layout {
    size_t head, row_off, row_src, y, total;
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
    L.row_off = take((size_t)(n_d + 1) * sizeof(int32_t));
    L.row_src = take((size_t)n_d * kS * sizeof(int32_t));
    L.y = take((size_t)n_d * kS * sizeof(float));
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
    int32_t* row_off = reinterpret_cast<int32_t*>(ws + L.row_off);
    int32_t* row_src = reinterpret_cast<int32_t*>(ws + L.row_src);
    float* y = reinterpret_cast<float*>(ws + L.y);

    hipLaunchKernelGGL(rows_kernel, dim3(1), dim3(1024), 0, st, n_stmt, n_d, row_off, row_src, head);
    PRUNER_LAUNCH_CHECK();
    const int64_t max_tiles = (n_d * kS + kTM - 1) / kTM;
    const unsigned grid = (unsigned)(max_tiles < g_num_cus ? max_tiles : g_num_cus);
    hipLaunchKernelGGL(mlp_kernel, dim3(grid), dim3(kThreads), 0, st, feat, row_src, head, w->W1, w->b1, w->W2, w->b2, w->w3, w->b3, y);
    PRUNER_LAUNCH_CHECK();
    hipLaunchKernelGGL(sum_kernel, dim3((unsigned)((n_d + 255) / 256)), dim3(256), 0, st, y, row_off, n_d, vscore);
    PRUNER_LAUNCH_CHECK();
    return PRUNER_OK;
}
