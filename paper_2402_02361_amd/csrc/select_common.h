// Device helpers shared by the selection kernels and by the draft kernel when it counts first digits on the fly.
#pragma once
#include "common.h"

#include <type_traits>

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

// The segment a workgroup belongs to: the last entry of a table sorted by first_block whose first_block is not after
// block b (entry 0 starts at block 0; empty segments share a first block with their successor and are never picked).
// A binary search is a chain of dependent reads, each a round trip to the cache; for tables of up to 256 entries
// every lane reads up to four entries at once instead and the wavefront counts those not after b.  The result is
// the same in every lane.
template <typename Seg> __device__ __forceinline__ int segment_of_block(const Seg* __restrict__ segs, int n_seg, int b)
{
    if (n_seg <= 2) return n_seg == 2 && segs[1].first_block <= b ? 1 : 0;
    if (n_seg <= 4 * kWave) {
        int not_after = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int i = q * kWave + lane_id();
            const bool hit = i < n_seg && segs[i < n_seg ? i : 0].first_block <= b;
            not_after += (int)__popcll(__ballot(hit));
        }
        return not_after - 1;
    }
    int lo = 0, hi = n_seg - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (segs[mid].first_block <= b) lo = mid; else hi = mid - 1;
    }
    return lo;
}

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

// Blocks of 256 neighbouring entries of a segment, counted from the segment's begin: the block whose first entry has the
// global index `first` in segment s keeps its largest key in slot (first >> 8) + s of the block-maximum array.  Slots of
// different blocks differ (inside a segment `first` grows by 256 from block to block; the next segment begins behind
// the last block's first entry and adds one more), so the array needs (n >> 8) + n_seg + 1 words.  Whoever holds the
// scores in registers (the draft kernel, or the first-digit pass) writes it; the pass that sets entries aside reads it and
// steps over every block whose maximum lies below the rank-k bucket: nearly all of them.
__device__ __forceinline__ int64_t block_max_slot(int64_t first, int s) { return (first >> 8) + s; }

// (key, index) packed so that a larger word is a better entry: key descending, then index ascending.
__device__ __forceinline__ uint64_t compose(uint32_t key, uint32_t gidx) { return ((uint64_t)key << 32) | (uint64_t)(0xFFFFFFFFu - gidx); }
__device__ __forceinline__ uint32_t index_of(uint64_t w) { return 0xFFFFFFFFu - (uint32_t)w; }

// ---- selection of a few entries from a short segment (at most 8192 entries, k at most 64) ------------------------------
//
// The final selection after the verify stage (a few thousand scores per subgraph, a few dozen kept) and small draft
// populations.  No digit passes: an entry is the word (key, index), all words of a segment are distinct, and the k best
// entries are the k largest words.  One workgroup of four wavefronts per segment:
//   1. a thread holds up to 32 words in registers and finds its largest;
//   2. the k-th largest of the 256 thread maxima is a pivot at or below the k-th largest word of the segment (k words,
//      those maxima, are at or above it), and words at or above it can only belong to the k threads whose maxima are:
//      at most 32 k of them, about k on scores in no particular order.  The pivot: every wavefront sorts its 64 maxima
//      across its lanes; a maximum's rank among all 256 is its place in its own wavefront plus, by bisection, the
//      number of larger ones in the other three sorted lists;
//   3. the words at or above the pivot go to a list in LDS; a word's row is the number of larger words in the list.
// 3 us where the one-workgroup route of sixteen wavefronts and three digit passes takes 12.

constexpr int kTinyThreads = 256;
constexpr int kTinyPer = 32;
constexpr int kTinyMax = kTinyThreads * kTinyPer;   // 8192 entries per segment
constexpr int kTinyK = 64;
constexpr int kTinyList = kTinyK * kTinyPer;        // words that can reach the pivot

// The word of lane (lane ^ STRIDE).  Inside a row of 16 lanes the data-parallel primitives do it at the vector ALU's own
// rate: a permutation of each group of four lanes for strides 1 and 2, a rotation of the row by 8 for stride 8, and for
// stride 4 the rotation by 12 (which brings lane + 4) or by 4 (lane - 4), whichever the lane needs; across rows the word
// goes through the LDS crossbar.  Every lane of the wavefront must be active.
template <int CTRL> __device__ __forceinline__ uint32_t dpp_move(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xf, 0xf, true);
}
template <int STRIDE> __device__ __forceinline__ uint32_t lane_xor_u32(uint32_t v)
{
    if constexpr (STRIDE == 1) return dpp_move<0xB1>(v);        // quad_perm:[1,0,3,2]
    else if constexpr (STRIDE == 2) return dpp_move<0x4E>(v);   // quad_perm:[2,3,0,1]
    else if constexpr (STRIDE == 4) {
        // both moves run with every lane active (a move whose source lane is switched off reads nothing), then each lane picks
        const uint32_t from_below = dpp_move<0x124>(v), from_above = dpp_move<0x12C>(v);   // row_ror:4 (lane - 4), row_ror:12 (lane + 4)
        return (lane_id() & 4) ? from_below : from_above;
    }
    else if constexpr (STRIDE == 8) return dpp_move<0x128>(v);  // row_ror:8
    else return __shfl_xor(v, STRIDE, kWave);
}
template <int STRIDE> __device__ __forceinline__ uint64_t lane_xor_u64(uint64_t w)
{
    const uint32_t lo = lane_xor_u32<STRIDE>((uint32_t)w), hi = lane_xor_u32<STRIDE>((uint32_t)(w >> 32));
    return ((uint64_t)hi << 32) | lo;
}

// The wavefront's 64 words in descending order over its lanes (bitonic network; partner = lane ^ stride).  Equal words
// (only the all-zero filler) may end up in either order.
__device__ __forceinline__ uint64_t wave_sort_descending(uint64_t w)
{
    const int lane = lane_id();
    auto exchange = [&](auto stride_c, int size) {
        constexpr int stride = decltype(stride_c)::value;
        const uint64_t other = lane_xor_u64<stride>(w);
        const bool lower = (lane & stride) == 0;           // the lower lane of the pair
        const bool down = (lane & size) == 0;              // this merge block is ordered largest first (always, in the last merge)
        w = ((lower == down) == (w > other)) ? w : other;
    };
#pragma unroll
    for (int size = 2; size <= kWave; size <<= 1) {
        if (size >= 64) exchange(std::integral_constant<int, 32>{}, size);
        if (size >= 32) exchange(std::integral_constant<int, 16>{}, size);
        if (size >= 16) exchange(std::integral_constant<int, 8>{}, size);
        if (size >= 8) exchange(std::integral_constant<int, 4>{}, size);
        if (size >= 4) exchange(std::integral_constant<int, 2>{}, size);
        exchange(std::integral_constant<int, 1>{}, size);
    }
    return w;
}

struct TinyLds {
    uint64_t sorted[kTinyThreads / kWave][kWave];   // every wavefront's thread maxima, largest first
    uint64_t pivot_slot;
    uint32_t fill;
    __attribute__((aligned(16))) uint64_t list[kTinyList + 2];
};

// The k best entries of score[seg_begin .. seg_end) as rows idx_out[row * k ..] (and val_out), best first.  A workgroup of
// kTinyThreads threads calls it with all its threads; it begins and ends with everything it read or wrote in L settled
// (callers need no barrier around it except for their own data).
__device__ __forceinline__ void tiny_select(TinyLds& L, const float* __restrict__ score, int64_t seg_begin, int64_t seg_end, int64_t row, int k,
                                            int32_t* __restrict__ idx_out, float* __restrict__ val_out)
{
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const float* seg_score = score + seg_begin;
    const int len = (int)(seg_end - seg_begin);

    uint64_t w[kTinyPer], best = 0;   // 0: no entry (below every word of a number)
#pragma unroll
    for (int j = 0; j < kTinyPer; ++j) {
        const int i = j * kTinyThreads + (int)threadIdx.x;
        w[j] = i < len ? compose(key_of(seg_score[i]), (uint32_t)(seg_begin + i)) : 0ull;
    }
#pragma unroll
    for (int j = 0; j < kTinyPer; ++j) best = w[j] > best ? w[j] : best;
    if (threadIdx.x == 0) L.fill = 0;

    const uint64_t mine = wave_sort_descending(best);   // lane p of this wavefront holds its p-th largest maximum
    L.sorted[wave][lane] = mine;
    __syncthreads();
    // rank of `mine` among the 256 maxima = larger ones in this wavefront (lane) + larger ones in the others.  At least k
    // maxima are words of entries (a segment holds at least k entries); the fillers rank behind all of them.
    uint32_t rank = (uint32_t)lane;
#pragma unroll
    for (int o = 1; o < kTinyThreads / kWave; ++o) {
        const uint64_t* other = L.sorted[(wave + o) % (kTinyThreads / kWave)];
        int lo = 0, hi = kWave;   // other[0 .. lo) > mine >= other[hi .. 64): lo ends as the number of larger ones
#pragma unroll
        for (int step = 0; step < 7; ++step) {   // the range halves from 64 to nothing
            const int mid = (lo + hi) >> 1;
            const bool larger = lo < hi && other[mid < kWave ? mid : kWave - 1] > mine;
            lo = larger ? mid + 1 : lo;
            hi = larger ? hi : mid;
        }
        rank += (uint32_t)lo;
    }
    if (mine != 0 && rank == (uint32_t)(k - 1)) L.pivot_slot = mine;
    __syncthreads();
    const uint64_t pivot = L.pivot_slot;
    // A thread's words at or above the pivot go to consecutive places of the list: the wavefront's threads share out a
    // range that one of them reserves (one atomic per wavefront, not one per word).
    uint32_t mine_count = 0;
#pragma unroll
    for (int j = 0; j < kTinyPer; ++j) mine_count += w[j] >= pivot && w[j] != 0 ? 1u : 0u;
    const uint32_t upto = wave_inclusive_sum(mine_count);
    uint32_t wave_base = 0;
    if (lane == kWave - 1 && upto != 0) wave_base = atomicAdd(&L.fill, upto);
    uint32_t at = (uint32_t)__builtin_amdgcn_readlane((int)wave_base, kWave - 1) + upto - mine_count;
    if (mine_count != 0) {
#pragma unroll
        for (int j = 0; j < kTinyPer; ++j)
            if (w[j] >= pivot && w[j] != 0) L.list[at++] = w[j];
    }
    __syncthreads();
    const int n_list = (int)L.fill;   // k .. 32 k
    if (threadIdx.x == 0) L.list[n_list] = L.list[n_list + 1] = 0;   // the comparison below reads two words at a time
    __syncthreads();
    typedef uint64_t u64x2 __attribute__((ext_vector_type(2)));
    for (int e = threadIdx.x; e < n_list; e += kTinyThreads) {
        const uint64_t me = L.list[e];
        uint32_t r = 0;
        for (int f = 0; f < n_list; f += 2) {
            const u64x2 two = *reinterpret_cast<const u64x2*>(L.list + f);
            r += two.x > me ? 1u : 0u;
            r += two.y > me ? 1u : 0u;
        }
        if (r < (uint32_t)k) {
            const uint32_t gi = index_of(me), kk = (uint32_t)(me >> 32);
            idx_out[row * k + r] = (int32_t)gi;
            // a key names its score, except the one that -0.0 and +0.0 share
            if (val_out) val_out[row * k + r] = kk == kZeroKey ? score[gi] : score_of_key(kk);
        }
    }
    __syncthreads();
}

}  // namespace pruner
