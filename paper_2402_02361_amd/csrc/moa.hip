// Momentum online Adaptation (Sec. 4.3; Update_MoA of Alg. 1; m = 0.99): after a round's fine-tuning of the target
// model, the Siamese model's weights follow the target's,
//     phi_s <- m phi_s + (1 - m) phi_t,
// with no forward or backward pass of the Siamese model.  (The paper's formula sits in a lost figure: this is the
// momentum-contrast form, equal to phi_s - (1 - m) lr sum Delta_t when phi_t = phi_s - lr sum Delta_t.)
// binary32, each operation rounded on its own, in this order: c = 1 - m (on the host); (m * phi_s) + (c * phi_t).
// The kernel also writes the new weights as bfloat16 (nearest, ties to even), the form the verify stage reads.
// A model is a few hundred kilobytes: one launch, bound by launch latency; at scale by its 12 to 14 bytes per weight.
#include "common.h"

namespace pruner {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float moa_one(float s, float t, float m, float c)
{
    const float a = m * s, b = c * t;   // compiled without contraction: two products, one sum
    return a + b;
}

// VEC = 4: pointers 16-byte aligned (bf16: 8), n4 groups of four; the tail and unaligned calls take VEC = 1
template <int VEC>
__global__ void __launch_bounds__(256) moa_kernel(float* __restrict__ phi_s, const float* __restrict__ phi_t, int64_t n, float m, float c,
                                                  uint16_t* __restrict__ bf16)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    if constexpr (VEC == 4) {
        const int64_t n4 = n >> 2;
        for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
            const f32x4 s = reinterpret_cast<const f32x4*>(phi_s)[i], t = reinterpret_cast<const f32x4*>(phi_t)[i];
            f32x4 v;
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = moa_one(s[j], t[j], m, c);
            reinterpret_cast<f32x4*>(phi_s)[i] = v;
            if (bf16) {
                const f32x2 lo = {v[0], v[1]}, hi = {v[2], v[3]};
                uint2 o;
                o.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2));
                o.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2));
                reinterpret_cast<uint2*>(bf16)[i] = o;
            }
        }
        for (int64_t i = 4 * n4 + (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
            const float v = moa_one(phi_s[i], phi_t[i], m, c);
            phi_s[i] = v;
            if (bf16) bf16[i] = __builtin_bit_cast(uint16_t, (__bf16)v);
        }
    } else {
        for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
            const float v = moa_one(phi_s[i], phi_t[i], m, c);
            phi_s[i] = v;
            if (bf16) bf16[i] = __builtin_bit_cast(uint16_t, (__bf16)v);
        }
    }
}

}  // namespace
}  // namespace pruner

using namespace pruner;

extern "C" int pruner_moa_update(float* phi_s, const float* phi_t, int64_t n, float m, uint16_t* phi_s_bf16, void* stream)
{
    if (n < 0 || !(m >= 0.0f && m <= 1.0f)) return PRUNER_EINVAL;
    if (n == 0) return PRUNER_OK;
    if (!phi_s || !phi_t || !aligned(phi_s, 4) || !aligned(phi_t, 4) || (phi_s_bf16 && !aligned(phi_s_bf16, 2))) return PRUNER_EINVAL;
    int moa_cus = 0;
    if (current_device(&moa_cus) < 0) return PRUNER_EHIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const float c = 1.0f - m;
    const bool wide = aligned(phi_s, 16) && aligned(phi_t, 16) && (!phi_s_bf16 || aligned(phi_s_bf16, 8));
    const int64_t items = wide ? (n + 3) / 4 : n;
    int64_t blocks = (items + 255) / 256;
    if (blocks > 8ll * moa_cus) blocks = 8ll * moa_cus;
    if (wide)
        hipLaunchKernelGGL(moa_kernel<4>, dim3((unsigned)blocks), dim3(256), 0, st, phi_s, phi_t, n, m, c, phi_s_bf16);
    else
        hipLaunchKernelGGL(moa_kernel<1>, dim3((unsigned)blocks), dim3(256), 0, st, phi_s, phi_t, n, m, c, phi_s_bf16);
    PRUNER_LAUNCH_CHECK();
    return PRUNER_OK;
}
