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

// LDS histogram increment.  Leading digits of scores take few values, and lanes that add to one bin queue on its
// address; so the lanes that share the first pending lane's bin are counted with one atomic, up to four bins in turn
// (a segment of equal scores, or of two or three neighbouring leading digits, costs a wavefront a handful of atomics
// instead of sixty-four); lanes still pending after that (digits that scatter) add 1 to their own bins.
__device__ __forceinline__ void wave_hist_add(uint32_t* hist, uint32_t digit, bool active)
{
    unsigned long long pending = __ballot(active);
#pragma unroll
    for (int round = 0; round < 4; ++round) {
        if (__popcll(pending) < 4) break;   // (same for every lane) a few stragglers add one by one
        const int leader = __ffsll(pending) - 1;
        const uint32_t d0 = __builtin_amdgcn_readlane(digit, leader);
        const unsigned long long same = __ballot(active && digit == d0);
        if (lane_id() == leader) atomicAdd(&hist[d0], (uint32_t)__popcll(same));
        active = active && digit != d0;
        pending &= ~same;
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
