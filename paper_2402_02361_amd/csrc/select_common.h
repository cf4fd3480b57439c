// Device helpers shared by the selection kernels and by the draft kernel when it counts first digits on the fly.
#pragma once
#include "common.h"

namespace pruner {

constexpr int kBins = 2048;   // 11-bit digits (the last pass uses the lower 1024 bins)

// Larger score <=> larger key; -0.0 and +0.0 share a key.
__device__ __forceinline__ uint32_t key_of(float x)
{
    uint32_t u = __float_as_uint(x);
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// The score with a given key (every key but the one that -0.0 and +0.0 share belongs to exactly one bit pattern).
constexpr uint32_t kZeroKey = 0x80000000u;
__device__ __forceinline__ float score_of_key(uint32_t key) { return __uint_as_float((key & 0x80000000u) ? (key & 0x7FFFFFFFu) : ~key); }

__device__ __forceinline__ int lane_id() { return __lane_id(); }

// LDS histogram increment.  Lanes that share the first active lane's bin are counted with one atomic when they
// are many (leading digits of scores are nearly constant, and a segment of equal scores would otherwise make
// all 64 lanes queue on one address); everyone else adds 1 to its own bin.
__device__ __forceinline__ void wave_hist_add(uint32_t* hist, uint32_t digit, bool active)
{
    const unsigned long long pending = __ballot(active);
    if (__popcll(pending) >= 8) {   // (fewer lanes cannot hold eight of a kind: they add one by one)
        const int leader = __ffsll(pending) - 1;
        const uint32_t d0 = __builtin_amdgcn_readlane(digit, leader);
        const unsigned long long same = __ballot(active && digit == d0);
        if (__popcll(same) >= 8) {
            if (lane_id() == leader) atomicAdd(&hist[d0], (uint32_t)__popcll(same));
            active = active && digit != d0;
        }
    }
    if (active) atomicAdd(&hist[digit], 1u);
}

// Merge a workgroup's LDS histogram into its copy of segment s's global histogram ([copies][n_seg][kBins]).
template <int NT>
__device__ __forceinline__ void flush_hist(const uint32_t* hist, uint32_t* __restrict__ ghist, int copies, int n_seg, int s)
{
    uint32_t* mine = ghist + ((int64_t)(blockIdx.x % copies) * n_seg + s) * kBins;
    for (int i = threadIdx.x; i < kBins; i += NT) {
        const uint32_t c = hist[i];
        if (c) atomicAdd(&mine[i], c);
    }
}

}  // namespace pruner
