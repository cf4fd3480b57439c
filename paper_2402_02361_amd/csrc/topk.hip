// Selection of the k best entries per segment (PriorFilter of Alg. 2; the choice of S_measured in Alg. 1).
//
// Exact radix selection on an order-preserving 32-bit image of the scores: three digit passes (11, 11, 10 bits,
// most significant first) find the key T of rank k; entries above T are all taken, entries equal to T are taken
// in index order until k is reached; the k survivors are then sorted by (key descending, index ascending) with a
// bitonic network in LDS.  Nothing depends on the order in which blocks or wavefronts run.
//
// Two routes, same result:
//   small  - every segment fits one workgroup's patience (<= kSmallMax entries): one launch, one workgroup of
//            1024 threads per segment does all passes (configs with many mid-sized subgraphs, and the final
//            selection after the verify stage);
//   large  - segments are cut into chunks of 4096 entries, one workgroup of 256 threads each; histograms are
//            built in LDS and merged with global atomics; a handful of launches.
#include "common.h"

#include <vector>

namespace pruner {
namespace {

constexpr int kBins = 2048;          // 11-bit digits (the last pass uses the lower 1024 bins)
constexpr int kSmallThreads = 1024;
constexpr int64_t kSmallMax = 131072;
constexpr int kChunkThreads = 256;
constexpr int kChunkPer = 16;
constexpr int kChunk = kChunkThreads * kChunkPer;

struct alignas(8) SegT {
    int64_t begin, end;
    int32_t first_block, pad;
};

struct alignas(16) SelState {
    uint32_t prefix;   // digits fixed so far (after the last pass: the key T of rank k)
    uint32_t k_rem;    // entries still to take among those matching the prefix (after the last pass: ties to take)
    uint32_t n_gt;     // entries above T
    uint32_t gt_fill;  // fill counter of the unordered "above T" part of the selection
};

// ---- keys ------------------------------------------------------------------------------------------------------

// Larger score <=> larger key; -0.0 and +0.0 share a key.
__device__ __forceinline__ uint32_t key_of(float x)
{
    uint32_t u = __float_as_uint(x);
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// (key, index) packed so that a larger word is a better entry: key descending, then index ascending.
__device__ __forceinline__ uint64_t compose(uint32_t key, uint32_t gidx) { return ((uint64_t)key << 32) | (uint64_t)(0xFFFFFFFFu - gidx); }
__device__ __forceinline__ uint32_t index_of(uint64_t w) { return 0xFFFFFFFFu - (uint32_t)w; }

template <int PASS> __device__ __forceinline__ uint32_t digit_of(uint32_t key)
{
    return PASS == 0 ? key >> 21 : PASS == 1 ? (key >> 10) & 0x7FFu : key & 0x3FFu;
}
template <int PASS> __device__ __forceinline__ bool matches(uint32_t key, uint32_t prefix)
{
    return PASS == 0 ? true : PASS == 1 ? (key >> 21) == prefix : (key >> 10) == prefix;
}

// ---- wavefront / workgroup primitives -----------------------------------------------------------------------

__device__ __forceinline__ int lane_id() { return __lane_id(); }

// LDS histogram increment that stays cheap when most lanes of a wavefront hit the same few bins (the leading
// digits of scores are nearly constant): up to four rounds elect a leader bin and add its whole population with
// one atomic; what is left uses one atomic per lane.
__device__ __forceinline__ void wave_hist_add(uint32_t* hist, uint32_t digit, bool active)
{
    unsigned long long pending = __ballot(active);
    for (int round = 0; round < 4 && pending; ++round) {
        const int leader = __ffsll(pending) - 1;
        const uint32_t d0 = __builtin_amdgcn_readlane(digit, leader);
        const unsigned long long same = __ballot(active && digit == d0);
        if (lane_id() == leader) atomicAdd(&hist[d0], (uint32_t)__popcll(same));
        active = active && digit != d0;
        pending &= ~same;
    }
    if (active) atomicAdd(&hist[digit], 1u);
}

// Exclusive prefix sum over the workgroup (NT threads, NT/64 <= 16 wavefronts); all threads must call.
// wave_tot: LDS, 16 entries.  *total receives the workgroup sum.
template <int NT> __device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* wave_tot, uint32_t* total)
{
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    uint32_t incl = v;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t up = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += up;
    }
    __syncthreads();  // wave_tot may still be read from an earlier call
    if (lane == kWave - 1) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < NT / kWave; ++w) {
        const uint32_t t = wave_tot[w];
        before += w < wave ? t : 0u;
        all += t;
    }
    *total = all;
    return before + incl - v;
}

// Digit bucket that holds the entry of rank k_rem (ranks counted from the largest digit down) and the rank left
// inside that bucket.  hist: kBins counters (LDS or global); NT = 1024 threads, two bins each.
__device__ __forceinline__ void find_bucket(const uint32_t* hist, uint32_t k_rem, uint32_t* wave_tot, uint32_t* out /* [2] in LDS */)
{
    const int a = kBins - 1 - 2 * (int)threadIdx.x, b = a - 1;
    const uint32_t ha = hist[a], hb = hist[b];
    uint32_t total;
    const uint32_t above = block_excl_scan<kSmallThreads>(ha + hb, wave_tot, &total);
    if (above < k_rem && k_rem <= above + ha) {
        out[0] = (uint32_t)a;
        out[1] = k_rem - above;
    } else if (above + ha < k_rem && k_rem <= above + ha + hb) {
        out[0] = (uint32_t)b;
        out[1] = k_rem - above - ha;
    }
    __syncthreads();
}

// Bitonic sort of P = 2^m words in LDS, largest first.
template <int NT> __device__ __forceinline__ void sort_descending(uint64_t* w, int P)
{
    for (int size = 2; size <= P; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (int i = threadIdx.x; i < (P >> 1); i += NT) {
                const int pos = 2 * i - (i & (stride - 1));
                const uint64_t x = w[pos], y = w[pos + stride];
                const bool down = (pos & size) == 0;
                if ((x < y) == down) {
                    w[pos] = y;
                    w[pos + stride] = x;
                }
            }
        }
    }
    __syncthreads();
}

__device__ __forceinline__ int pow2_at_least(int k)
{
    int P = 1;
    while (P < k) P <<= 1;
    return P;
}

// Sort the k selected words and write the result rows of one segment.
template <int NT>
__device__ __forceinline__ void finish_segment(uint64_t* sel, int k, const float* __restrict__ score, int32_t* __restrict__ idx_out,
                                               float* __restrict__ val_out, int64_t row)
{
    const int P = pow2_at_least(k);
    for (int i = k + threadIdx.x; i < P; i += NT) sel[i] = 0;  // below every real word
    sort_descending<NT>(sel, P);
    for (int r = threadIdx.x; r < k; r += NT) {
        const uint32_t gi = index_of(sel[r]);
        idx_out[row * k + r] = (int32_t)gi;
        if (val_out) val_out[row * k + r] = score[gi];
    }
}

// ---- small route: one workgroup per segment -------------------------------------------------------------------

template <int PASS>
__device__ __forceinline__ void small_pass(const float* __restrict__ seg_score, int64_t len, uint32_t* hist, uint32_t* wave_tot,
                                           uint32_t* found, uint32_t& prefix, uint32_t& k_rem)
{
    for (int i = threadIdx.x; i < kBins; i += kSmallThreads) hist[i] = 0;
    __syncthreads();
    for (int64_t base = 0; base < len; base += kSmallThreads) {
        const int64_t i = base + threadIdx.x;
        const bool valid = i < len;
        const uint32_t key = valid ? key_of(seg_score[i]) : 0u;
        wave_hist_add(hist, digit_of<PASS>(key), valid && matches<PASS>(key, prefix));
    }
    __syncthreads();
    find_bucket(hist, k_rem, wave_tot, found);
    prefix = PASS == 2 ? (prefix << 10) | found[0] : (prefix << 11) | found[0];
    k_rem = found[1];
    __syncthreads();
}

__global__ void __launch_bounds__(kSmallThreads) topk_small_kernel(const float* __restrict__ score, const SegT* __restrict__ segs,
                                                                   int k, int32_t* __restrict__ idx_out, float* __restrict__ val_out)
{
    __shared__ uint32_t hist[kBins];
    __shared__ uint32_t wave_tot[16];
    __shared__ uint32_t found[2];
    __shared__ uint32_t gt_fill;
    __shared__ uint64_t sel[PRUNER_MAX_K];

    const SegT seg = segs[blockIdx.x];
    const float* seg_score = score + seg.begin;
    const int64_t len = seg.end - seg.begin;

    uint32_t prefix = 0, k_rem = (uint32_t)k;
    small_pass<0>(seg_score, len, hist, wave_tot, found, prefix, k_rem);
    small_pass<1>(seg_score, len, hist, wave_tot, found, prefix, k_rem);
    small_pass<2>(seg_score, len, hist, wave_tot, found, prefix, k_rem);
    const uint32_t T = prefix, k_eq = k_rem, n_gt = (uint32_t)k - k_eq;

    if (threadIdx.x == 0) gt_fill = 0;
    __syncthreads();
    uint32_t eq_before = 0;  // ties seen in earlier rounds (same value in every thread)
    for (int64_t base = 0; base < len; base += kSmallThreads) {
        const int64_t i = base + threadIdx.x;
        const bool valid = i < len;
        const uint32_t key = valid ? key_of(seg_score[i]) : 0u;
        if (valid && key > T) sel[atomicAdd(&gt_fill, 1u)] = compose(key, (uint32_t)(seg.begin + i));
        if (eq_before < k_eq) {  // ties in index order until enough are taken
            const bool tie = valid && key == T;
            uint32_t total;
            const uint32_t rank = eq_before + block_excl_scan<kSmallThreads>(tie ? 1u : 0u, wave_tot, &total);
            if (tie && rank < k_eq) sel[n_gt + rank] = compose(key, (uint32_t)(seg.begin + i));
            eq_before += total;
        }
    }
    __syncthreads();
    finish_segment<kSmallThreads>(sel, k, score, idx_out, val_out, blockIdx.x);
}

// ---- large route ------------------------------------------------------------------------------------------------

__global__ void __launch_bounds__(256) fill_zero_kernel(uint32_t* __restrict__ p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0;
}

__device__ __forceinline__ int segment_of_block(const SegT* __restrict__ segs, int n_seg, int b)
{
    int lo = 0, hi = n_seg - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (segs[mid].first_block <= b) lo = mid; else hi = mid - 1;
    }
    return lo;
}

template <int PASS>
__global__ void __launch_bounds__(kChunkThreads) hist_kernel(const float* __restrict__ score, const SegT* __restrict__ segs, int n_seg,
                                                             const SelState* __restrict__ state, uint32_t* __restrict__ ghist /* [n_seg][kBins] */)
{
    __shared__ uint32_t hist[kBins];
    const int s = segment_of_block(segs, n_seg, blockIdx.x);
    const SegT seg = segs[s];
    const uint32_t prefix = PASS == 0 ? 0u : state[s].prefix;
    for (int i = threadIdx.x; i < kBins; i += kChunkThreads) hist[i] = 0;
    __syncthreads();
    const int64_t c0 = seg.begin + (int64_t)(blockIdx.x - seg.first_block) * kChunk;
#pragma unroll 4
    for (int j = 0; j < kChunkPer; ++j) {
        const int64_t i = c0 + j * kChunkThreads + threadIdx.x;
        const bool valid = i < seg.end;
        const uint32_t key = valid ? key_of(score[i]) : 0u;
        wave_hist_add(hist, digit_of<PASS>(key), valid && matches<PASS>(key, prefix));
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kBins; i += kChunkThreads) {
        const uint32_t c = hist[i];
        if (c) atomicAdd(&ghist[(int64_t)s * kBins + i], c);
    }
}

template <int PASS>
__global__ void __launch_bounds__(kSmallThreads) bucket_kernel(const uint32_t* __restrict__ ghist, SelState* __restrict__ state, int k)
{
    __shared__ uint32_t wave_tot[16];
    __shared__ uint32_t found[2];
    const int s = blockIdx.x;
    const uint32_t prefix = PASS == 0 ? 0u : state[s].prefix;
    const uint32_t k_rem = PASS == 0 ? (uint32_t)k : state[s].k_rem;
    find_bucket(ghist + (int64_t)s * kBins, k_rem, wave_tot, found);
    if (threadIdx.x == 0) {
        SelState st;
        st.prefix = PASS == 2 ? (prefix << 10) | found[0] : (prefix << 11) | found[0];
        st.k_rem = found[1];
        st.n_gt = (uint32_t)k - found[1];
        st.gt_fill = 0;
        state[s] = st;
    }
}

// Entries above T go to the front part of the segment's selection in any order; ties are counted per chunk.
__global__ void __launch_bounds__(kChunkThreads) collect_kernel(const float* __restrict__ score, const SegT* __restrict__ segs, int n_seg,
                                                                SelState* __restrict__ state, uint64_t* __restrict__ sel /* [n_seg][k] */,
                                                                int k, uint32_t* __restrict__ eq_cnt /* per block */)
{
    __shared__ uint32_t n_tie;
    const int s = segment_of_block(segs, n_seg, blockIdx.x);
    const SegT seg = segs[s];
    const uint32_t T = state[s].prefix;
    if (threadIdx.x == 0) n_tie = 0;
    __syncthreads();
    const int64_t c0 = seg.begin + (int64_t)(blockIdx.x - seg.first_block) * kChunk;
    uint32_t ties = 0;
#pragma unroll 4
    for (int j = 0; j < kChunkPer; ++j) {
        const int64_t i = c0 + j * kChunkThreads + threadIdx.x;
        if (i < seg.end) {
            const uint32_t key = key_of(score[i]);
            if (key > T) sel[(int64_t)s * k + atomicAdd(&state[s].gt_fill, 1u)] = compose(key, (uint32_t)i);
            ties += key == T ? 1u : 0u;
        }
    }
    // one LDS atomic per wavefront that saw ties
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) ties += __shfl_down(ties, off, kWave);
    if (lane_id() == 0 && ties) atomicAdd(&n_tie, ties);
    __syncthreads();
    if (threadIdx.x == 0) eq_cnt[blockIdx.x] = n_tie;
}

// Exclusive scan of the chunks' tie counts within each segment: eq_cnt[b] becomes the number of ties before chunk b.
// The chunk's own count moves to eq_own[b].
__global__ void __launch_bounds__(kSmallThreads) tie_scan_kernel(const SegT* __restrict__ segs, int n_seg, int32_t total_blocks,
                                                                 uint32_t* __restrict__ eq_cnt, uint32_t* __restrict__ eq_own)
{
    __shared__ uint32_t wave_tot[16];
    const int s = blockIdx.x;
    const int b0 = segs[s].first_block, b1 = s + 1 < n_seg ? segs[s + 1].first_block : total_blocks;
    uint32_t carry = 0;
    for (int base = b0; base < b1; base += kSmallThreads) {
        const int b = base + threadIdx.x;
        const uint32_t v = b < b1 ? eq_cnt[b] : 0u;
        uint32_t total;
        const uint32_t before = carry + block_excl_scan<kSmallThreads>(v, wave_tot, &total);
        if (b < b1) {
            eq_cnt[b] = before;
            eq_own[b] = v;
        }
        carry += total;
    }
}

// Chunks that hold ties which still fit write them, in index order, behind the "above T" part.
__global__ void __launch_bounds__(kChunkThreads) tie_write_kernel(const float* __restrict__ score, const SegT* __restrict__ segs, int n_seg,
                                                                  const SelState* __restrict__ state, uint64_t* __restrict__ sel, int k,
                                                                  const uint32_t* __restrict__ eq_before, const uint32_t* __restrict__ eq_own)
{
    __shared__ uint32_t wave_tot[16];
    const int s = segment_of_block(segs, n_seg, blockIdx.x);
    const SelState st = state[s];
    const uint32_t k_eq = st.k_rem;
    uint32_t taken = eq_before[blockIdx.x];
    if (eq_own[blockIdx.x] == 0 || taken >= k_eq) return;  // same for the whole workgroup
    const SegT seg = segs[s];
    const int64_t c0 = seg.begin + (int64_t)(blockIdx.x - seg.first_block) * kChunk;
    for (int j = 0; j < kChunkPer && taken < k_eq; ++j) {
        const int64_t i = c0 + j * kChunkThreads + threadIdx.x;
        const bool tie = i < seg.end && key_of(score[i]) == st.prefix;
        uint32_t total;
        const uint32_t rank = taken + block_excl_scan<kChunkThreads>(tie ? 1u : 0u, wave_tot, &total);
        if (tie && rank < k_eq) sel[(int64_t)s * k + st.n_gt + rank] = compose(st.prefix, (uint32_t)i);
        taken += total;
    }
}

__global__ void __launch_bounds__(kSmallThreads) sort_kernel(const float* __restrict__ score, const uint64_t* __restrict__ gsel, int k,
                                                             int32_t* __restrict__ idx_out, float* __restrict__ val_out)
{
    __shared__ uint64_t sel[PRUNER_MAX_K];
    for (int i = threadIdx.x; i < k; i += kSmallThreads) sel[i] = gsel[(int64_t)blockIdx.x * k + i];
    finish_segment<kSmallThreads>(sel, k, score, idx_out, val_out, blockIdx.x);
}

struct Layout {
    size_t segs, state, hist, sel, eq_cnt, eq_own, total;
};

Layout layout(int64_t n, int32_t n_sg, int32_t k)
{
    Layout L;
    const size_t blocks = (size_t)(n / kChunk) + (size_t)n_sg + 1;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += round_up(bytes, 256);
        return at;
    };
    L.segs = take((size_t)n_sg * sizeof(SegT));
    L.state = take((size_t)n_sg * sizeof(SelState));
    L.hist = take((size_t)3 * n_sg * kBins * sizeof(uint32_t));
    L.sel = take((size_t)n_sg * (size_t)k * sizeof(uint64_t));
    L.eq_cnt = take(blocks * sizeof(uint32_t));
    L.eq_own = take(blocks * sizeof(uint32_t));
    L.total = off;
    return L;
}

}  // namespace

size_t topk_workspace_bytes(int64_t n, int32_t n_sg, int32_t k)
{
    if (n < 0) n = 0;
    if (n_sg < 1) n_sg = 1;
    if (k < 1) k = 1;
    return layout(n, n_sg, k).total;
}

}  // namespace pruner

using namespace pruner;

extern "C" int pruner_topk(const float* score, const int64_t* seg_off, int32_t n_sg, int32_t k, int32_t* idx_out, float* val_out,
                           void* workspace, size_t workspace_bytes, void* stream)
{
    if (!score || !seg_off || !idx_out || n_sg < 1 || n_sg > PRUNER_MAX_SUBGRAPHS || k < 1 || k > PRUNER_MAX_K) return PRUNER_EINVAL;
    if (!aligned(score, 4) || !aligned(idx_out, 4) || (val_out && !aligned(val_out, 4))) return PRUNER_EINVAL;
    if (seg_off[0] != 0) return PRUNER_EINVAL;
    int64_t longest = 0;
    for (int32_t s = 0; s < n_sg; ++s) {
        const int64_t len = seg_off[s + 1] - seg_off[s];
        if (len < k) return PRUNER_EINVAL;
        longest = len > longest ? len : longest;
    }
    const int64_t n = seg_off[n_sg];
    if (n > 0x7FFFFFFFll) return PRUNER_EINVAL;  // indices are int32
    if (!workspace || !aligned(workspace, 256)) return PRUNER_EWORKSPACE;
    const Layout L = layout(n, n_sg, k);
    if (workspace_bytes < L.total) return PRUNER_EWORKSPACE;

    hipStream_t st = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    SegT* d_segs = reinterpret_cast<SegT*>(ws + L.segs);

    std::vector<SegT> segs(n_sg);
    int64_t blocks = 0;
    for (int32_t s = 0; s < n_sg; ++s) {
        segs[s] = SegT{seg_off[s], seg_off[s + 1], (int32_t)blocks, 0};
        blocks += (seg_off[s + 1] - seg_off[s] + kChunk - 1) / kChunk;
    }
    int rc = put_table(d_segs, segs.data(), segs.size() * sizeof(SegT), st);
    if (rc) return rc;

    if (longest <= kSmallMax) {
        hipLaunchKernelGGL(topk_small_kernel, dim3(n_sg), dim3(kSmallThreads), 0, st, score, d_segs, k, idx_out, val_out);
        PRUNER_LAUNCH_CHECK();
        return PRUNER_OK;
    }

    SelState* d_state = reinterpret_cast<SelState*>(ws + L.state);
    uint32_t* d_hist = reinterpret_cast<uint32_t*>(ws + L.hist);
    uint64_t* d_sel = reinterpret_cast<uint64_t*>(ws + L.sel);
    uint32_t* d_eq_cnt = reinterpret_cast<uint32_t*>(ws + L.eq_cnt);
    uint32_t* d_eq_own = reinterpret_cast<uint32_t*>(ws + L.eq_own);
    const int64_t hist_words = (int64_t)3 * n_sg * kBins;
    const size_t per_pass = (size_t)n_sg * kBins;
    const dim3 chunks((unsigned)blocks), segsGrid((unsigned)n_sg);

    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((hist_words + 255) / 256)), dim3(256), 0, st, d_hist, hist_words);
    PRUNER_LAUNCH_CHECK();
    hipLaunchKernelGGL(hist_kernel<0>, chunks, dim3(kChunkThreads), 0, st, score, d_segs, n_sg, d_state, d_hist);
    PRUNER_LAUNCH_CHECK();
    hipLaunchKernelGGL(bucket_kernel<0>, segsGrid, dim3(kSmallThreads), 0, st, d_hist, d_state, k);
    PRUNER_LAUNCH_CHECK();
    hipLaunchKernelGGL(hist_kernel<1>, chunks, dim3(kChunkThreads), 0, st, score, d_segs, n_sg, d_state, d_hist + per_pass);
    PRUNER_LAUNCH_CHECK();
    hipLaunchKernelGGL(bucket_kernel<1>, segsGrid, dim3(kSmallThreads), 0, st, d_hist + per_pass, d_state, k);
    PRUNER_LAUNCH_CHECK();
    hipLaunchKernelGGL(hist_kernel<2>, chunks, dim3(kChunkThreads), 0, st, score, d_segs, n_sg, d_state, d_hist + 2 * per_pass);
    PRUNER_LAUNCH_CHECK();
    hipLaunchKernelGGL(bucket_kernel<2>, segsGrid, dim3(kSmallThreads), 0, st, d_hist + 2 * per_pass, d_state, k);
    PRUNER_LAUNCH_CHECK();
    hipLaunchKernelGGL(collect_kernel, chunks, dim3(kChunkThreads), 0, st, score, d_segs, n_sg, d_state, d_sel, k, d_eq_cnt);
    PRUNER_LAUNCH_CHECK();
    hipLaunchKernelGGL(tie_scan_kernel, segsGrid, dim3(kSmallThreads), 0, st, d_segs, n_sg, (int32_t)blocks, d_eq_cnt, d_eq_own);
    PRUNER_LAUNCH_CHECK();
    hipLaunchKernelGGL(tie_write_kernel, chunks, dim3(kChunkThreads), 0, st, score, d_segs, n_sg, d_state, d_sel, k, d_eq_cnt, d_eq_own);
    PRUNER_LAUNCH_CHECK();
    hipLaunchKernelGGL(sort_kernel, segsGrid, dim3(kSmallThreads), 0, st, score, d_sel, k, idx_out, val_out);
    PRUNER_LAUNCH_CHECK();
    return PRUNER_OK;
}
