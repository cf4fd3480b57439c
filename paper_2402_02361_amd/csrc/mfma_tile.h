// Pieces shared by the kernels that run small dense layers on the matrix cores (v_mfma_f32_32x32x16_bf16), computed
// transposed: H^T = W X^T, a wavefront owning 64 output units (two 32-unit blocks) whose weight fragments it keeps in
// registers, the rows (32 at a time) coming from LDS as bfloat16.  A lane (l32 = lane & 31, half = lane >> 5) then
// holds, per 32-unit block, 16 output units of ONE row: register i is unit 8*(i/4) + 4*half + i%4.
#pragma once
#include "common.h"

namespace pruner {
namespace tile {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short i16x2 __attribute__((ext_vector_type(2)));

// bfloat16(max(a, 0)), bfloat16(max(b, 0)) in one register: rounding keeps the sign, and a bfloat16 with the sign bit
// set is a negative 16-bit integer, so the integer maximum with 0 is the ReLU of both halves (-0 included).
__device__ __forceinline__ uint32_t relu_bf16x2(float a, float b)
{
    const f32x2 v = {a, b};
    const i16x2 zero = {0, 0};
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(i16x2, __builtin_convertvector(v, bf16x2)), zero));
}

// acc <- the layer's bias (cst: 256 binary32 values in LDS): register i of a 32x32 result holds hidden unit
// 8*(i/4) + 4*half + i%4 of its 32-unit block
__device__ __forceinline__ void bias_init(floatx16 (&acc)[2], const float* cst, int wave, int half)
{
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const f32x4 b = *reinterpret_cast<const f32x4*>(&cst[64 * wave + 32 * nt + 8 * g + 4 * half]);
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[nt][4 * g + j] = b[j];
        }
}

// acc += W_slice . B^T for 32 rows: B points at the rows' first element in LDS (row stride `stride` bfloat16), wr holds
// this wavefront's weight fragments.  Operand fragments of steps ks+1 and ks+2 are on their way from LDS when the MFMAs
// of step ks are issued.  side(i), i = 0 .. 2 KS - 1, is other work of this wavefront (epilogues of the tile's other
// half, bookkeeping), issued after the i-th MFMA: the vector ALU would otherwise idle while the matrix pipe is busy.
template <int KS, typename Side>
__device__ __forceinline__ void layer(floatx16 (&acc)[2], const bf16x8 (&wr)[2][KS], const __bf16* B, int stride, int l32, int half, Side&& side)
{
    bf16x8 fb[3];
#pragma unroll
    for (int p = 0; p < 2; ++p) fb[p] = *reinterpret_cast<const bf16x8*>(&B[l32 * stride + 16 * p + 8 * half]);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        if (ks + 2 < KS) fb[(ks + 2) % 3] = *reinterpret_cast<const bf16x8*>(&B[l32 * stride + 16 * (ks + 2) + 8 * half]);
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            __builtin_amdgcn_sched_barrier(0);   // keep the order: reads ahead of the MFMAs that do not need them yet, side work between MFMAs
            acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[nt][ks], fb[ks % 3], acc[nt], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            side(2 * ks + nt);
        }
    }
}

// As layer(), but the accumulators start from `init` (two 32x32 results' worth of registers: a bias in accumulator
// layout) or, with init == nullptr, from zero: the first depth step's MFMAs take that as their addend, so no instruction
// initialises an accumulator.  What acc held before is overwritten.
template <int KS, typename Side>
__device__ __forceinline__ void layer_from(floatx16 (&acc)[2], const floatx16* init, const bf16x8 (&wr)[2][KS], const __bf16* B, int stride, int l32,
                                           int half, Side&& side)
{
    bf16x8 fb[3];
#pragma unroll
    for (int p = 0; p < 2; ++p) fb[p] = *reinterpret_cast<const bf16x8*>(&B[l32 * stride + 16 * p + 8 * half]);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        if (ks + 2 < KS) fb[(ks + 2) % 3] = *reinterpret_cast<const bf16x8*>(&B[l32 * stride + 16 * (ks + 2) + 8 * half]);
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            __builtin_amdgcn_sched_barrier(0);
            if (ks == 0) {
                floatx16 zero;
#pragma unroll
                for (int i = 0; i < 16; ++i) zero[i] = 0.f;
                acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[nt][ks], fb[ks % 3], init ? init[nt] : zero, 0, 0, 0);
            } else {
                acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[nt][ks], fb[ks % 3], acc[nt], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            side(2 * ks + nt);
        }
    }
}

// One of the 8 pieces of a hidden layer's epilogue for 32 rows: ReLU, rounding to bfloat16, and the store of four
// neighbouring hidden units of row l32 (H points at the rows' first element, row stride `stride` bfloat16).
__device__ __forceinline__ void park_hidden(const floatx16 (&acc)[2], int piece, __bf16* H, int stride, int wave, int l32, int half)
{
    const int nt = piece >> 2, g = piece & 3;
    u32x2 o;
    o[0] = relu_bf16x2(acc[nt][4 * g + 0], acc[nt][4 * g + 1]);
    o[1] = relu_bf16x2(acc[nt][4 * g + 2], acc[nt][4 * g + 3]);
    *reinterpret_cast<u32x2*>(&H[l32 * stride + 64 * wave + 32 * nt + 8 * g + 4 * half]) = o;
}

}  // namespace tile
}  // namespace pruner
