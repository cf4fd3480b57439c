// Selection of the k best entries per segment (PriorFilter of Alg. 2; the choice of S_measured in Alg. 1).
//
// Exact radix selection on an order-preserving 32-bit image of the scores: three digit passes (11, 11, 10 bits,
// most significant first) find the key T of rank k; entries above T are all taken, entries equal to T are taken
// in index order until k is reached; the k survivors are then sorted by (key descending, index ascending) with a
// bitonic network in LDS.  Nothing depends on the order in which blocks or wavefronts run.
//
// Two routes, same result:
//   small  - every segment fits one workgroup's patience (<= kSmallMax entries): one launch, one workgroup of
//            1024 threads per segment does all passes (the final selection after the verify stage; beyond 32768
//            entries the passes of a single workgroup take longer than the large route's six launches);
//   large  - segments are cut into spans of whole 16384-entry sweeps, one workgroup of 1024 threads each; the
//            scores are read twice at most (first-digit histogram, which also notes the largest key of every 256
//            entries; then everything at or above that digit's rank-k bucket is set aside, a few thousand entries as
//            a rule, and blocks of 256 whose largest key lies below the bucket are not read again) and the later
//            passes work on what was set aside; six launches.
#include "select_common.h"

#include <string.h>

#include <vector>

namespace pruner {
namespace {

constexpr int kSmallThreads = 1024;
constexpr int64_t kSmallMax = 32768;
constexpr int kTieCap = 1024;        // ties the small route ranks instead of scanning for
constexpr int kSmallPer = 8;         // loads a thread of the small route keeps in flight

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

template <int PASS> __device__ __forceinline__ uint32_t digit_of(uint32_t key)
{
    return PASS == 0 ? key >> 21 : PASS == 1 ? (key >> 10) & 0x7FFu : key & 0x3FFu;
}
template <int PASS> __device__ __forceinline__ bool matches(uint32_t key, uint32_t prefix)
{
    return PASS == 0 ? true : PASS == 1 ? (key >> 21) == prefix : (key >> 10) == prefix;
}

// ---- wavefront / workgroup primitives -----------------------------------------------------------------------

// Exclusive prefix sum over the workgroup (NT threads, NT/64 <= 16 wavefronts); all threads must call.
// wave_tot: LDS, 16 entries.  *total receives the workgroup sum.
template <int NT> __device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* wave_tot, uint32_t* total)
{
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const uint32_t incl = wave_inclusive_sum(v);
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
// inside that bucket (out[0], out[1]) and the bucket's population (out[2]).  hist: kBins counters (LDS or global);
// NT = 1024 threads, two bins each.
__device__ __forceinline__ void find_bucket(const uint32_t* hist, uint32_t k_rem, uint32_t* wave_tot, uint32_t* out /* [3] in LDS */)
{
    const int a = kBins - 1 - 2 * (int)threadIdx.x, b = a - 1;
    const uint32_t ha = hist[a], hb = hist[b];
    uint32_t total;
    const uint32_t above = block_excl_scan<kSmallThreads>(ha + hb, wave_tot, &total);
    if (above < k_rem && k_rem <= above + ha) {
        out[0] = (uint32_t)a;
        out[1] = k_rem - above;
        out[2] = ha;
    } else if (above + ha < k_rem && k_rem <= above + ha + hb) {
        out[0] = (uint32_t)b;
        out[1] = k_rem - above - ha;
        out[2] = hb;
    }
    __syncthreads();
}

// The selection lives in LDS with one spare word after every 32: neighbouring threads of the sort then touch different
// banks also when they walk 8-word groups (logical index e sits in slot(e)).
constexpr int kSelWords = PRUNER_MAX_K + PRUNER_MAX_K / 32 + 2;
__device__ __forceinline__ uint32_t slot(uint32_t e) { return e + (e >> 5); }

// Bitonic sort of P = 2^m words in LDS, largest first.  One round trip through LDS performs up to three consecutive
// strides (4s, 2s, s): a thread takes the 2, 4 or 8 words base + i*s, which those strides permute among themselves,
// and exchanges them in registers.  All words of such a group lie in one half of the current merge size, so they
// share the direction.
template <int LOG> __device__ __forceinline__ void bitonic_group(uint64_t* w, int g, int s, int size)
{
    constexpr int N = 1 << LOG;
    const int base = (g / s) * (N * s) + (g % s);
    const bool down = (base & size) == 0;
    uint64_t x[N];
#pragma unroll
    for (int i = 0; i < N; ++i) x[i] = w[slot(base + i * s)];
#pragma unroll
    for (int h = N >> 1; h > 0; h >>= 1) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            if ((i & h) == 0) {
                const uint64_t a = x[i], b = x[i + h];
                const bool swap = (a < b) == down;
                x[i] = swap ? b : a;
                x[i + h] = swap ? a : b;
            }
        }
    }
#pragma unroll
    for (int i = 0; i < N; ++i) w[slot(base + i * s)] = x[i];
}

template <int NT> __device__ __forceinline__ void sort_descending(uint64_t* w, int P)
{
    for (int size = 2; size <= P; size <<= 1) {
        int stride = size >> 1;   // largest stride still to do in this merge
        while (stride > 0) {
            __syncthreads();
            if (stride >= 4) {
                const int s = stride >> 2;
                for (int g = threadIdx.x; g < (P >> 3); g += NT) bitonic_group<3>(w, g, s, size);
                stride >>= 3;
            } else if (stride == 2) {
                for (int g = threadIdx.x; g < (P >> 2); g += NT) bitonic_group<2>(w, g, 1, size);
                stride = 0;
            } else {
                for (int g = threadIdx.x; g < (P >> 1); g += NT) bitonic_group<1>(w, g, 1, size);
                stride = 0;
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
                                               float* __restrict__ val_out, int64_t row, int64_t seg_begin, int64_t seg_end, int row_len)
{
    const int P = pow2_at_least(k);
    for (int i = k + threadIdx.x; i < P; i += NT) sel[slot(i)] = 0;  // below every real word
    sort_descending<NT>(sel, P);
    for (int r0 = threadIdx.x; r0 < k; r0 += 4 * NT) {
        uint32_t gi[4];
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {   // the scores of four rows are requested together
            gi[u] = r0 + u * NT < k ? index_of(sel[slot(r0 + u * NT)]) : 0xFFFFFFFFu;
            v[u] = val_out && gi[u] >= seg_begin && gi[u] < seg_end ? score[gi[u]] : 0.f;   // never read outside the segment
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (r0 + u * NT < k) {
                idx_out[row * row_len + r0 + u * NT] = (int32_t)gi[u];
                if (val_out) val_out[row * row_len + r0 + u * NT] = v[u];
            }
        }
    }
}

// Output rows for n of the k selected words (their positions: which[i], or first + i * stride without a list) without
// sorting: the words are distinct
// (they carry the index), so the rank of a word is the number of larger words among all k.  A wavefront holds
// R = 64, 32 or 16 of the n words at a time (the fewest lanes that still hold them all: idle lanes would cost the same
// as busy ones) and 64 / R parts of its sixteenth of the k words to compare with; the lanes of one part read the same
// word at a time (a broadcast LDS access).  Cheap when the k words' ranks are shared out over many workgroups; a full
// sort in one workgroup is better served by the bitonic network.  cnt: NT LDS words.  All NT threads call.
template <int NT>
__device__ __forceinline__ void rank_rows(const uint64_t* sel, int k, const uint16_t* which, int first, int stride, int n, uint32_t* cnt,
                                          const float* __restrict__ score, int32_t* __restrict__ idx_out, float* __restrict__ val_out, int64_t row,
                                          int64_t seg_begin, int64_t seg_end, int row_len)
{
    typedef uint64_t u64x2 __attribute__((ext_vector_type(2)));
    constexpr int W = NT / kWave;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int R = n <= 16 ? 16 : n <= 32 ? 32 : kWave, parts = kWave / R;
    const int mine_at = lane & (R - 1), piece = wave * parts + lane / R;
    // the comparison runs over the padded storage itself, two words per LDS access; the spare words and the words
    // past the last selected one hold 0 (the caller clears them), which is below every real word
    const int n_raw = ((int)slot((uint32_t)k - 1u) + 2) & ~1;
    const int per_piece = (((n_raw + W * parts - 1) / (W * parts)) + 1) & ~1;
    const int j_lo = piece * per_piece < n_raw ? piece * per_piece : n_raw, j_hi = j_lo + per_piece < n_raw ? j_lo + per_piece : n_raw;
    for (int e0 = 0; e0 < n; e0 += R) {
        const bool live = e0 + mine_at < n;
        const uint64_t mine = live ? sel[slot(which ? (uint32_t)which[e0 + mine_at] : (uint32_t)(first + (e0 + mine_at) * stride))] : ~0ull;
        uint32_t c = 0;
#pragma unroll 4
        for (int j = j_lo; j < j_hi; j += 2) {
            const u64x2 w = *reinterpret_cast<const u64x2*>(sel + j);
            c += w.x > mine ? 1u : 0u;
            c += w.y > mine ? 1u : 0u;
        }
        cnt[threadIdx.x] = c;
        __syncthreads();
        if (wave == 0 && lane < R && live) {
            uint32_t r = 0;
            for (int q = lane; q < NT; q += R) r += cnt[q];   // the counts of this word from every piece
            const uint32_t gi = index_of(mine);
            if (r < (uint32_t)k) {
                idx_out[row * row_len + r] = (int32_t)gi;
                if (val_out) val_out[row * row_len + r] = gi >= seg_begin && gi < seg_end ? score[gi] : 0.f;   // never read outside the segment
            }
        }
        __syncthreads();
    }
}

// ---- small route: one workgroup per segment -------------------------------------------------------------------

template <int PASS, bool RES>
__device__ __forceinline__ void small_pass(const float* __restrict__ seg_score, int64_t len, const uint32_t (&held)[kSmallPer],
                                           uint32_t* hist, uint32_t* wave_tot, uint32_t* found, uint32_t& prefix, uint32_t& k_rem)
{
    for (int i = threadIdx.x; i < kBins; i += kSmallThreads) hist[i] = 0;
    __syncthreads();
    if constexpr (RES) {
        // the whole segment sits in registers (one batch): no memory traffic in this pass
#pragma unroll
        for (int j = 0; j < kSmallPer; ++j) {
            const int64_t i = j * kSmallThreads + threadIdx.x;
            wave_hist_add(hist, digit_of<PASS>(held[j]), i < len && matches<PASS>(held[j], prefix));
        }
    } else {
        for (int64_t base = 0; base < len; base += kSmallThreads * kSmallPer) {
            float val[kSmallPer];   // a batch of loads in flight together
#pragma unroll
            for (int j = 0; j < kSmallPer; ++j) {
                const int64_t i = base + j * kSmallThreads + threadIdx.x;
                val[j] = i < len ? seg_score[i] : 0.f;
            }
#pragma unroll
            for (int j = 0; j < kSmallPer; ++j) {
                const int64_t i = base + j * kSmallThreads + threadIdx.x;
                const uint32_t key = key_of(val[j]);
                wave_hist_add(hist, digit_of<PASS>(key), i < len && matches<PASS>(key, prefix));
            }
        }
    }
    __syncthreads();
    find_bucket(hist, k_rem, wave_tot, found);
    prefix = PASS == 2 ? (prefix << 10) | found[0] : (prefix << 11) | found[0];
    k_rem = found[1];
    __syncthreads();
}

// Up to kInlineSegs segment ranges travel as kernel arguments (no table upload, one launch for the whole call).
constexpr int kInlineSegs = 128;
struct InlineSegs {
    SegT s[kInlineSegs];
};

// RES: no segment is longer than one batch (8192 entries): its keys are loaded once and stay in registers.
template <bool INLINE, bool RES>
__global__ void __launch_bounds__(kSmallThreads) topk_small_kernel(const float* __restrict__ score, const SegT* __restrict__ segs,
                                                                   InlineSegs inl, int k, int32_t* __restrict__ idx_out,
                                                                   float* __restrict__ val_out)
{
    __shared__ uint32_t hist[kBins];
    __shared__ uint32_t wave_tot[16];
    __shared__ uint32_t found[3];
    __shared__ uint32_t gt_fill, tie_fill;
    __shared__ uint32_t tie_buf[kTieCap];
    __shared__ uint64_t sel[kSelWords];

    const SegT seg = INLINE ? inl.s[blockIdx.x] : segs[blockIdx.x];
    const float* seg_score = score + seg.begin;
    const int64_t len = seg.end - seg.begin;

    uint32_t held[kSmallPer];
#pragma unroll
    for (int j = 0; j < kSmallPer; ++j) {
        const int64_t i = j * kSmallThreads + threadIdx.x;
        held[j] = RES && i < len ? key_of(seg_score[i]) : 0u;   // 0 is below every key of a number
    }
    uint32_t prefix = 0, k_rem = (uint32_t)k;
    small_pass<0, RES>(seg_score, len, held, hist, wave_tot, found, prefix, k_rem);
    small_pass<1, RES>(seg_score, len, held, hist, wave_tot, found, prefix, k_rem);
    small_pass<2, RES>(seg_score, len, held, hist, wave_tot, found, prefix, k_rem);
    const uint32_t T = prefix, k_eq = k_rem, n_gt = (uint32_t)k - k_eq;

    const uint32_t n_tie = found[2];   // entries equal to T in the whole segment
    if (threadIdx.x == 0) gt_fill = tie_fill = 0;
    __syncthreads();
    if (n_tie <= (uint32_t)kTieCap) {
        // few ties: gather their indices in any order, then keep the k_eq smallest by rank
        for (int64_t base = 0; base < len; base += kSmallThreads * kSmallPer) {
            uint32_t key[kSmallPer];
#pragma unroll
            for (int j = 0; j < kSmallPer; ++j) {
                const int64_t i = base + j * kSmallThreads + threadIdx.x;
                key[j] = RES ? held[j] : i < len ? key_of(seg_score[i]) : 0u;   // 0 is below every key of a number
            }
#pragma unroll
            for (int j = 0; j < kSmallPer; ++j) {
                const int64_t i = base + j * kSmallThreads + threadIdx.x;
                if (key[j] > T) sel[slot(atomicAdd(&gt_fill, 1u))] = compose(key[j], (uint32_t)(seg.begin + i));
                else if (key[j] == T) tie_buf[atomicAdd(&tie_fill, 1u)] = (uint32_t)(seg.begin + i);
            }
        }
        __syncthreads();
        for (uint32_t i = threadIdx.x; i < n_tie; i += kSmallThreads) {
            const uint32_t me = tie_buf[i];
            uint32_t rank = 0;
            for (uint32_t j = 0; j < n_tie; ++j) rank += tie_buf[j] < me ? 1u : 0u;
            if (rank < k_eq) sel[slot(n_gt + rank)] = compose(T, me);
        }
    } else {
        // many ties: walk the segment in index order and number the ties with a workgroup scan until enough are taken
        uint32_t eq_before = 0;  // ties seen in earlier rounds (same value in every thread)
        for (int64_t base = 0; base < len; base += kSmallThreads * kSmallPer) {
            uint32_t key[kSmallPer];
#pragma unroll
            for (int j = 0; j < kSmallPer; ++j) {
                const int64_t i = base + j * kSmallThreads + threadIdx.x;
                key[j] = RES ? held[j] : i < len ? key_of(seg_score[i]) : 0u;
            }
#pragma unroll
            for (int j = 0; j < kSmallPer; ++j) {
                const int64_t i = base + j * kSmallThreads + threadIdx.x;
                if (key[j] > T) sel[slot(atomicAdd(&gt_fill, 1u))] = compose(key[j], (uint32_t)(seg.begin + i));
                if (eq_before < k_eq) {
                    const bool tie = key[j] == T;
                    uint32_t total;
                    const uint32_t rank = eq_before + block_excl_scan<kSmallThreads>(tie ? 1u : 0u, wave_tot, &total);
                    if (tie && rank < k_eq) sel[slot(n_gt + rank)] = compose(key[j], (uint32_t)(seg.begin + i));
                    eq_before += total;
                }
            }
        }
    }
    __syncthreads();
    finish_segment<kSmallThreads>(sel, k, score, idx_out, val_out, blockIdx.x, seg.begin, seg.end, k);
}

// ---- tiny route: segments of at most 8192 entries, k at most 64 ---------------------------------------------------
// (tiny_select in select_common.h: the final selection after the verify stage and small draft populations)

template <bool INLINE>
__global__ void __launch_bounds__(kTinyThreads) topk_tiny_kernel(const float* __restrict__ score, const SegT* __restrict__ segs, InlineSegs inl,
                                                                 int k, int32_t* __restrict__ idx_out, float* __restrict__ val_out)
{
    __shared__ TinyLds L;
    const SegT seg = INLINE ? inl.s[blockIdx.x] : segs[blockIdx.x];
    tiny_select(L, score, seg.begin, seg.end, blockIdx.x, k, idx_out, val_out);
}

// ---- large route ------------------------------------------------------------------------------------------------
//
// Workgroups of 1024 threads each own `span` consecutive entries of one segment (span = a multiple of 16384, sized
// so that a launch is a single wave of workgroups).  No global atomics with a return value, no cross-workgroup
// order, and every launch after the first finds the digit bucket of the pass before it by itself (all workgroups
// of a segment compute the same bucket from the merged histogram; the segment's first workgroup records it):
//   hist0        LDS histogram of the first digit, merged into one of R global copies (R > 1 spreads same-address
//                atomics when few segments share many workgroups)
//   funnel       bucket of digit 0; entries above it are final and are staged as such; entries inside it are
//                candidates: staged in the workgroup's own list and counted into the second digit's histogram
//   refine       bucket of digit 1; third digit's histogram over the staged candidates
//   settle       bucket of digit 2 = the key T of rank k; candidates above T join the staged winners, candidates
//                equal to T become the staged ties
//   gather_sort  one workgroup per segment: concatenates the staged lists in workgroup (= index) order, keeps the
//                first ties, re-reads the span of a workgroup whose list overflowed, sorts, writes the result
// A workgroup whose candidate list overflows (more than kCandCap entries of its span fall into one first-digit
// bucket: scores in a very narrow band, or equal) reads its span again in refine and settle instead.

constexpr int kBigThreads = 1024;
constexpr int kBigPer = 16;
constexpr int kRow = kBigThreads * kBigPer;   // 16384 entries per sweep of a workgroup
constexpr int kStageCap = 256;                // staged winners / ties per workgroup
constexpr int kCandCap = 1024;                // staged candidates per workgroup

struct Stage {
    uint32_t n_gt, n_tie, n_cand;              // n_gt, n_tie: true counts (may exceed the capacities); n_cand: above its capacity = overflowed
    uint32_t pad;
    uint64_t gt[kStageCap];                    // composed words of entries above T, any order
    uint32_t tie[kStageCap];                   // global indices of ties, any order
    uint64_t cand[kCandCap];                   // composed words of entries in the first digit's rank-k bucket, any order
};

// One sweep of a workgroup over kRow consecutive entries starting at `row`: thread t receives kBigPer of them.
// WIDE (segments start on 16-byte boundaries): four neighbours per 16-byte load; else one entry per load.
// sweep_index gives the global index of the thread's j-th entry; entries at or past `hi` read as 0.
template <bool WIDE> __device__ __forceinline__ int64_t sweep_index(int64_t row, int j)
{
    return WIDE ? row + ((int64_t)(j >> 2) * kBigThreads + threadIdx.x) * 4 + (j & 3) : row + (int64_t)j * kBigThreads + threadIdx.x;
}
template <bool WIDE> __device__ __forceinline__ void load_sweep(const float* __restrict__ score, int64_t row, int64_t hi, float (&val)[kBigPer])
{
    if (WIDE) {
#pragma unroll
        for (int q = 0; q < kBigPer / 4; ++q) {
            const int64_t i = sweep_index<true>(row, 4 * q);
            if (i + 3 < hi) {
                const float4 v = *reinterpret_cast<const float4*>(score + i);
                val[4 * q] = v.x, val[4 * q + 1] = v.y, val[4 * q + 2] = v.z, val[4 * q + 3] = v.w;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) val[4 * q + e] = i + e < hi ? score[i + e] : 0.f;
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < kBigPer; ++j) {
            const int64_t i = sweep_index<false>(row, j);
            val[j] = i < hi ? score[i] : 0.f;
        }
    }
}

// The digit bucket that holds rank k_rem, from the merged histogram of a finished pass.  hist: kBins LDS words
// (overwritten); found: 3 LDS words (bucket, rank left inside it, its population).  All 1024 threads call.
template <int kMaxCopies>   // the most copies the pass's histogram can have (R <= kMaxCopies)
__device__ __forceinline__ void bucket_of_pass(const uint32_t* __restrict__ ghist, int R, int n_seg, int s, uint32_t k_rem,
                                               uint32_t* hist, uint32_t* wave_tot, uint32_t* found)
{
    uint32_t part[kBins / kBigThreads][kMaxCopies];   // all loads in flight together
#pragma unroll
    for (int q = 0; q < kBins / kBigThreads; ++q) {
#pragma unroll
        for (int r = 0; r < kMaxCopies; ++r)
            part[q][r] = ghist[((int64_t)(r < R ? r : 0) * n_seg + s) * kBins + q * kBigThreads + threadIdx.x];
    }
#pragma unroll
    for (int q = 0; q < kBins / kBigThreads; ++q) {
        uint32_t c = 0;
#pragma unroll
        for (int r = 0; r < kMaxCopies; ++r) c += r < R ? part[q][r] : 0u;
        hist[q * kBigThreads + threadIdx.x] = c;
    }
    __syncthreads();
    find_bucket(hist, k_rem, wave_tot, found);
}

template <bool WIDE>
__global__ void __launch_bounds__(kBigThreads) hist0_kernel(const float* __restrict__ score, const SegT* __restrict__ segs, int n_seg,
                                                            int64_t span, int R, uint32_t* __restrict__ ghist /* [R][n_seg][kBins] */,
                                                            uint32_t* __restrict__ block_max /* WIDE only; or null */)
{
    __shared__ uint32_t hist[kBins];
    const int s = segment_of_block(segs, n_seg, blockIdx.x);
    const SegT seg = segs[s];
    for (int i = threadIdx.x; i < kBins; i += kBigThreads) hist[i] = 0;
    __syncthreads();
    const int64_t lo = seg.begin + (int64_t)(blockIdx.x - seg.first_block) * span;
    const int64_t hi = lo + span < seg.end ? lo + span : seg.end;
    for (int64_t row = lo; row < hi; row += kRow) {
        float val[kBigPer];
        load_sweep<WIDE>(score, row, hi, val);
        uint32_t top[kBigPer / 4] = {};
#pragma unroll
        for (int j = 0; j < kBigPer; ++j) {
            const int64_t i = sweep_index<WIDE>(row, j);
            const uint32_t key = key_of(val[j]);
            wave_hist_add(hist, digit_of<0>(key), i < hi);
            if (i < hi && key > top[j >> 2]) top[j >> 2] = key;
        }
        if constexpr (WIDE) {
            // a wavefront's q-th load is one block of 256 neighbouring entries (spans are whole sweeps from the segment's begin)
            if (block_max) {
#pragma unroll
                for (int q = 0; q < kBigPer / 4; ++q) {
                    const uint32_t m = wave_inclusive_max(top[q]);
                    const int64_t first = sweep_index<true>(row, 4 * q) - 4 * lane_id();
                    if (lane_id() == 63 && first < hi) block_max[block_max_slot(first, s)] = m;
                }
            }
        }
    }
    __syncthreads();
    flush_hist<kBigThreads>(hist, ghist, R, n_seg, s);
}

// BLK (with WIDE): block_max holds the largest key of every block of 256 neighbouring entries; a block whose maximum
// lies below the bucket is not read.  Wavefront w takes blocks w, w + 16, ... of the span, 64 of them per look at the
// maxima (one per lane), and reads those that are left four at a time.
// (held to 64 registers: a compute unit then holds two of these workgroups, and a launch of up to 512 runs in one round)
template <bool WIDE, bool BLK>
__global__ void __launch_bounds__(kBigThreads) __attribute__((amdgpu_waves_per_eu(8))) funnel_kernel(const float* __restrict__ score, const SegT* __restrict__ segs, int n_seg,
                                                             int64_t span, int R, int k, const uint32_t* __restrict__ ghist0,
                                                             uint32_t* __restrict__ ghist1, SelState* __restrict__ state,
                                                             Stage* __restrict__ stage, const uint32_t* __restrict__ block_max)
{
    static_assert(WIDE || !BLK, "blocks are what the wide loads cover");
    __shared__ uint32_t hist[kBins];
    __shared__ uint32_t wave_tot[16];
    __shared__ uint32_t found[3];
    __shared__ uint32_t n_gt, n_cand, live_blocks;
    const int s = segment_of_block(segs, n_seg, blockIdx.x);
    const SegT seg = segs[s];
    const int64_t lo = seg.begin + (int64_t)(blockIdx.x - seg.first_block) * span;
    const int64_t hi = lo + span < seg.end ? lo + span : seg.end;
    float val[kBigPer];
    const int wave = threadIdx.x >> 6;
    if (BLK && threadIdx.x == 0) live_blocks = 0;   // (the bucket search below has barriers before anyone adds to it)
    const int64_t n_blk = (hi - lo + 255) >> 8;
    uint32_t top = 0;
    // the first sweep (the first maxima) travel while the bucket is looked up
    if constexpr (BLK) {
        const int64_t b = wave + 16 * lane_id();
        if (b < n_blk) top = block_max[block_max_slot(lo + (b << 8), s)];
    } else {
        load_sweep<WIDE>(score, lo, hi, val);
    }
    bucket_of_pass<8>(ghist0, R, n_seg, s, (uint32_t)k, hist, wave_tot, found);
    const uint32_t b0 = found[0], k_rem = found[1];
    if constexpr (BLK) {
        // how many of the span's (first 1024) blocks will have to be read
        const unsigned long long first_left = __ballot(top >= (b0 << 21) && wave + 16 * lane_id() < n_blk);
        if (lane_id() == 0) atomicAdd(&live_blocks, (uint32_t)__popcll(first_left));
    }
    __syncthreads();
    if (blockIdx.x == seg.first_block && threadIdx.x == 0) state[s] = SelState{b0, k_rem, (uint32_t)k - k_rem, 0u};
    for (int i = threadIdx.x; i < kBins; i += kBigThreads) hist[i] = 0;
    if (threadIdx.x == 0) n_gt = n_cand = 0;
    __syncthreads();
    // Where most blocks hold an entry of the bucket (a population of copies: ties by the hundred thousand), stepping over
    // the others gains nothing and the plain sweeps, whole rows of loads in flight, are the faster way through the span.
    const bool dense = BLK && 2 * (int64_t)live_blocks > (n_blk < 16 * kWave ? n_blk : 16 * kWave);
    Stage& mine = stage[blockIdx.x];
    // The smallest score whose first digit is b0.  Nearly every entry lies below it, and one comparison tells: a
    // wavefront steps over an entry unless one of its lanes is not below (a NaN never is; the exact test follows).
    const uint32_t low_key = b0 << 21;
    const float t0 = __uint_as_float((low_key & 0x80000000u) ? (low_key & 0x7FFFFFFFu) : ~low_key);
    // What happens to one entry (every lane of the wavefront calls it, `mine_to_look_at` says whether the lane holds one).
    auto look_at = [&](float x, int64_t i, bool mine_to_look_at, bool list_open) {
        const uint32_t key = mine_to_look_at && i < hi ? key_of(x) : 0u;   // 0 is below every key of a number
        const uint32_t d0 = digit_of<0>(key);
        const bool inside = mine_to_look_at && i < hi && d0 == b0;
        if (mine_to_look_at && i < hi && d0 > b0) {
            const uint32_t at = atomicAdd(&n_gt, 1u);
            if (at < kStageCap) mine.gt[at] = compose(key, (uint32_t)i);
        } else if (inside && list_open) {
            const uint32_t at = atomicAdd(&n_cand, 1u);
            if (at < kCandCap) mine.cand[at] = compose(key, (uint32_t)i);
        }
        wave_hist_add(hist, digit_of<1>(key), inside);
    };
    if constexpr (BLK) {
        for (int64_t g = 0; !dense && g < n_blk; g += 16 * kWave) {
            if (g > 0) {
                const int64_t b = g + wave + 16 * lane_id();
                top = b < n_blk ? block_max[block_max_slot(lo + (b << 8), s)] : 0u;
            }
            // (a lane past the span's last block holds 0 and is left out: no key of a number is 0, and low_key = 0 takes all)
            unsigned long long left = __ballot(top >= low_key && g + wave + 16 * lane_id() < n_blk);
            while (left) {
                int32_t at[4];   // (global indices are below 2^31)
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    at[u] = -1;
                    if (left) {
                        const int l = __ffsll(left) - 1;
                        left &= left - 1;
                        at[u] = (int32_t)(lo + ((g + wave + 16 * (int64_t)l) << 8)) + 4 * lane_id();
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int64_t i = at[u];
                    if (i >= 0 && i + 3 < hi) {
                        const float4 v = *reinterpret_cast<const float4*>(score + i);
                        val[4 * u] = v.x, val[4 * u + 1] = v.y, val[4 * u + 2] = v.z, val[4 * u + 3] = v.w;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) val[4 * u + e] = i >= 0 && i + e < hi ? score[i + e] : 0.f;
                    }
                }
                // One comparison per entry tells whether it can matter at all (nearly none does; a NaN is never below,
                // the exact test on the key follows).  The few that can are then looked at together: every lane picks the
                // first such entry it holds and the wavefront goes through the motions once, again while a lane holds more.
                bool can[kBigPer], any = false;
#pragma unroll
                for (int j = 0; j < kBigPer; ++j) {
                    can[j] = at[j >> 2] >= 0 && !(val[j] < t0);
                    any = any || can[j];
                }
                const bool list_open = n_cand <= (uint32_t)kCandCap;
                while (__ballot(any) != 0ull) {
                    bool picked = false;
                    float x = 0.f;
                    int32_t i = 0;
                    any = false;
#pragma unroll
                    for (int j = 0; j < kBigPer; ++j) {
                        if (__ballot(can[j]) == 0ull) continue;
                        const bool take = can[j] && !picked;
                        x = take ? val[j] : x;
                        i = take ? at[j >> 2] + (j & 3) : i;
                        picked = picked || take;
                        can[j] = can[j] && !take;
                        any = any || can[j];
                    }
                    look_at(x, (int64_t)i, picked, list_open);
                }
            }
        }
    }
    for (int64_t row = lo; (!BLK || dense) && row < hi; row += kRow) {
        if (BLK || row > lo) load_sweep<WIDE>(score, row, hi, val);
        // once the candidate list has overflowed, the later passes read the span again: nothing more is staged in it
        // (the count only has to stay above the list's capacity)
        const bool list_open = n_cand <= (uint32_t)kCandCap;
#pragma unroll
        for (int j = 0; j < kBigPer; ++j) {
            // a wavefront steps over an entry unless one of its lanes is not below the bucket's smallest score
            if (__ballot(!(val[j] < t0)) == 0ull) continue;
            look_at(val[j], sweep_index<WIDE>(row, j), true, list_open);
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        mine.n_gt = n_gt;
        mine.n_cand = n_cand;
        mine.n_tie = 0;
    }
    flush_hist<kBigThreads>(hist, ghist1, 1, n_seg, s);   // few contributors as a rule: one copy
}

template <bool WIDE>
__global__ void __launch_bounds__(kBigThreads) refine_kernel(const float* __restrict__ score, const SegT* __restrict__ segs, int n_seg,
                                                             int64_t span, const uint32_t* __restrict__ ghist1,
                                                             uint32_t* __restrict__ ghist2, SelState* __restrict__ state,
                                                             const Stage* __restrict__ stage)
{
    __shared__ uint32_t hist[kBins];
    __shared__ uint32_t wave_tot[16];
    __shared__ uint32_t found[3];
    const int s = segment_of_block(segs, n_seg, blockIdx.x);
    const SegT seg = segs[s];
    const SelState before = state[s];
    bucket_of_pass<1>(ghist1, 1, n_seg, s, before.k_rem, hist, wave_tot, found);
    const uint32_t prefix = (before.prefix << 11) | found[0], k_rem = found[1];
    __syncthreads();
    for (int i = threadIdx.x; i < kBins; i += kBigThreads) hist[i] = 0;
    __syncthreads();
    const Stage& mine = stage[blockIdx.x];
    const uint32_t n_cand = mine.n_cand;
    if (n_cand <= (uint32_t)kCandCap) {
        for (uint32_t base = 0; base < n_cand; base += kBigThreads) {
            const uint32_t i = base + threadIdx.x;
            const uint32_t key = i < n_cand ? (uint32_t)(mine.cand[i] >> 32) : 0u;
            wave_hist_add(hist, digit_of<2>(key), i < n_cand && matches<2>(key, prefix));
        }
    } else {
        const int64_t lo = seg.begin + (int64_t)(blockIdx.x - seg.first_block) * span;
        const int64_t hi = lo + span < seg.end ? lo + span : seg.end;
        for (int64_t row = lo; row < hi; row += kRow) {
            float val[kBigPer];
            load_sweep<WIDE>(score, row, hi, val);
#pragma unroll
            for (int j = 0; j < kBigPer; ++j) {
                const int64_t i = sweep_index<WIDE>(row, j);
                const uint32_t key = key_of(val[j]);
                wave_hist_add(hist, digit_of<2>(key), i < hi && matches<2>(key, prefix));
            }
        }
    }
    __syncthreads();
    flush_hist<kBigThreads>(hist, ghist2, 1, n_seg, s);
    // every workgroup of the segment has read the old state before this launch ends; the new one is for the next launch
    if (blockIdx.x == seg.first_block && threadIdx.x == 0) state[n_seg + s] = SelState{prefix, k_rem, before.n_gt, 0u};
}

template <bool WIDE>
__global__ void __launch_bounds__(kBigThreads) settle_kernel(const float* __restrict__ score, const SegT* __restrict__ segs, int n_seg,
                                                             int64_t span, int k, const uint32_t* __restrict__ ghist2,
                                                             SelState* __restrict__ state, Stage* __restrict__ stage)
{
    __shared__ uint32_t hist[kBins];
    __shared__ uint32_t wave_tot[16];
    __shared__ uint32_t found[3];
    __shared__ uint32_t n_gt, n_tie;
    const int s = segment_of_block(segs, n_seg, blockIdx.x);
    const SegT seg = segs[s];
    const SelState before = state[n_seg + s];
    bucket_of_pass<1>(ghist2, 1, n_seg, s, before.k_rem, hist, wave_tot, found);
    const uint32_t T = (before.prefix << 10) | found[0], k_eq = found[1];
    __syncthreads();
    if (blockIdx.x == seg.first_block && threadIdx.x == 0) state[2 * n_seg + s] = SelState{T, k_eq, (uint32_t)k - k_eq, 0u};
    Stage& mine = stage[blockIdx.x];
    const uint32_t n_cand = mine.n_cand;
    if (n_cand <= (uint32_t)kCandCap) {
        // winners staged so far keep their places; candidates above T follow them
        if (threadIdx.x == 0) {
            n_gt = mine.n_gt;
            n_tie = 0;
        }
        __syncthreads();
        for (uint32_t i = threadIdx.x; i < n_cand; i += kBigThreads) {
            const uint64_t w = mine.cand[i];
            const uint32_t key = (uint32_t)(w >> 32);
            if (key > T) {
                const uint32_t at = atomicAdd(&n_gt, 1u);
                if (at < kStageCap) mine.gt[at] = w;
            } else if (key == T) {
                const uint32_t at = atomicAdd(&n_tie, 1u);
                if (at < kStageCap) mine.tie[at] = index_of(w);
            }
        }
    } else {
        if (threadIdx.x == 0) n_gt = n_tie = 0;
        __syncthreads();
        const int64_t lo = seg.begin + (int64_t)(blockIdx.x - seg.first_block) * span;
        const int64_t hi = lo + span < seg.end ? lo + span : seg.end;
        for (int64_t row = lo; row < hi; row += kRow) {
            float val[kBigPer];
            load_sweep<WIDE>(score, row, hi, val);
#pragma unroll
            for (int j = 0; j < kBigPer; ++j) {
                const int64_t i = sweep_index<WIDE>(row, j);
                const uint32_t key = i < hi ? key_of(val[j]) : 0u;   // 0 is below every key of a number
                if (key > T) {
                    const uint32_t at = atomicAdd(&n_gt, 1u);
                    if (at < kStageCap) mine.gt[at] = compose(key, (uint32_t)i);
                } else if (key == T) {
                    const uint32_t at = atomicAdd(&n_tie, 1u);
                    if (at < kStageCap) mine.tie[at] = (uint32_t)i;
                }
            }
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        mine.n_gt = n_gt;
        mine.n_tie = n_tie;
    }
}

// Store into the selection only inside its k words: the positions are sums of counts that other launches left in the
// workspace, and a workspace shared by two overlapping calls (which the boundary forbids) must not turn into a wild
// LDS address.
__device__ __forceinline__ void put_selected(uint64_t* sel, int k, uint32_t e, uint64_t w)
{
    if (e < (uint32_t)k) sel[slot(e)] = w;
}

// One output row: entry gi of the population at rank r of segment `row`'s k.
__device__ __forceinline__ void put_row(int k, uint32_t r, uint32_t gi, const float* __restrict__ score, int32_t* __restrict__ idx_out,
                                        float* __restrict__ val_out, int64_t row, int64_t seg_begin, int64_t seg_end)
{
    if (r < (uint32_t)k) {
        idx_out[row * k + r] = (int32_t)gi;
        if (val_out) val_out[row * k + r] = gi >= seg_begin && gi < seg_end ? score[gi] : 0.f;   // never read outside the segment
    }
}

// The same for a tie, whose score the key T gives without a read (a read in the middle of a run of such rows would
// hold each of them up by a memory round trip); the key of zero stands for two bit patterns and is looked up.
__device__ __forceinline__ void put_tie_row(int k, uint32_t r, uint32_t gi, uint32_t T, const float* __restrict__ score, int32_t* __restrict__ idx_out,
                                            float* __restrict__ val_out, int64_t row, int64_t seg_begin, int64_t seg_end)
{
    if (T == kZeroKey) {
        put_row(k, r, gi, score, idx_out, val_out, row, seg_begin, seg_end);
    } else if (r < (uint32_t)k) {
        idx_out[row * k + r] = (int32_t)gi;
        if (val_out) val_out[row * k + r] = score_of_key(T);
    }
}

// `share` workgroups per segment.  The entries above T need ranking: each workgroup assembles all n_gt of them in
// LDS (the same work, from the same staged lists, the same set of words, in an order that may differ) and then ranks
// and writes the rows of the words whose index hashes to it.  The ties need none: they share the key T, come in
// index order, and the tie of rank r among them owns row n_gt + r; they go from the staged lists (or from a span
// that is read again) straight to the output, each list and each span by one of the workgroups.
__global__ void __launch_bounds__(kSmallThreads) gather_sort_kernel(const float* __restrict__ score, const SegT* __restrict__ segs, int n_seg,
                                                                    int32_t total_blocks, int64_t span, const SelState* __restrict__ state,
                                                                    const Stage* __restrict__ stage, int k, int share,
                                                                    int32_t* __restrict__ idx_out, float* __restrict__ val_out)
{
    __shared__ __align__(16) uint64_t sel[kSelWords];
    __shared__ uint32_t cnt[kSmallThreads];
    __shared__ uint16_t own[PRUNER_MAX_K];   // positions of the words this workgroup ranks
    __shared__ uint32_t n_own;
    __shared__ uint32_t wave_tot[16];
    __shared__ uint32_t tie_buf[kStageCap];
    __shared__ int32_t redo[64];          // workgroups whose span must be read again (list overflow)
    __shared__ uint32_t redo_gt_at[64], redo_tie_before[64];
    __shared__ uint8_t redo_what[64];     // 1: for its entries above T (every workgroup does), 2: for its ties (one does)
    __shared__ uint32_t n_redo, redo_fill;
    __shared__ uint32_t gt_reread;        // a span is read again for its entries above T: their places then differ between workgroups
    __shared__ int32_t partial_block;     // the workgroup in which the tie quota runs out
    __shared__ uint32_t partial_before;
    __shared__ uint32_t first_g[kSmallThreads + 1], first_t[kSmallThreads + 1];   // where each workgroup's lists begin
    __shared__ uint8_t list_skip[kSmallThreads];   // 1: the list of entries above T is not copied, 2: nor the list of ties

    const int s = blockIdx.x / share, part = blockIdx.x % share;
    const SegT seg = segs[s];
    const SelState st = state[2 * n_seg + s];   // as left by the settle launch
    const uint32_t T = st.prefix, k_eq = st.k_rem;
    const uint32_t n_gt = st.n_gt < (uint32_t)k ? st.n_gt : (uint32_t)k;   // (a workspace that overlapping calls share must not turn into wild addresses)
    const int b0 = seg.first_block, b1 = s + 1 < n_seg ? segs[s + 1].first_block : total_blocks;
    if (threadIdx.x == 0) {
        n_redo = 0;
        gt_reread = 0;
        partial_block = -1;
    }
    // (the first batch of list lengths is on its way while the selection is cleared)
    const uint32_t first_cg = b0 + (int)threadIdx.x < b1 ? stage[b0 + threadIdx.x].n_gt : 0u;
    const uint32_t first_ct = b0 + (int)threadIdx.x < b1 ? stage[b0 + threadIdx.x].n_tie : 0u;
    for (int i = threadIdx.x; i < kSelWords; i += kSmallThreads) sel[i] = 0;   // spare words must read as "below everything"
    __syncthreads();

    // Pass over the segment's workgroups in order, kSmallThreads of them at a time: running offsets of both lists.
    // The lists are then copied entry by entry, not list by list: position e finds its list by a search over the
    // offsets, so that all threads copy whatever the lists' lengths (a thread per list would walk the long ones
    // alone).
    uint32_t gt_carry = 0, tie_carry = 0;
    for (int base = b0; base < b1; base += kSmallThreads) {
        const int b = base + threadIdx.x;
        const bool live = b < b1;
        const uint32_t cg = base == b0 ? first_cg : live ? stage[b].n_gt : 0u, ct = base == b0 ? first_ct : live ? stage[b].n_tie : 0u;
        uint32_t tot_g, tot_t;
        const uint32_t at_g = gt_carry + block_excl_scan<kSmallThreads>(cg, wave_tot, &tot_g);
        const uint32_t before_t = tie_carry + block_excl_scan<kSmallThreads>(ct, wave_tot, &tot_t);
        const bool tie_needed = ct > 0 && before_t < k_eq;
        const bool tie_all = tie_needed && before_t + ct <= k_eq;
        const bool over_g = cg > kStageCap, over_t = tie_needed && ct > kStageCap;
        const bool mine = b % share == part;   // this workgroup looks after the ties of that span
        if (live && over_g) gt_reread = 1u;
        if (live && (over_g || (over_t && mine))) {
            const uint32_t slot = atomicAdd(&n_redo, 1u);
            if (slot < 64) {
                redo[slot] = b;
                redo_gt_at[slot] = at_g;
                redo_tie_before[slot] = before_t;
                redo_what[slot] = (uint8_t)((over_g ? 1 : 0) | (over_t && mine ? 2 : 0));
            }
        }
        if (live && tie_needed && !tie_all && !over_t && mine) {
            partial_block = b;       // exactly one workgroup of the launch crosses the quota
            partial_before = before_t;
        }
        first_g[threadIdx.x] = at_g;
        first_t[threadIdx.x] = before_t;
        list_skip[threadIdx.x] = (uint8_t)((over_g ? 1 : 0) | (over_t || !tie_all ? 2 : 0));
        if (threadIdx.x == 0) {
            first_g[kSmallThreads] = gt_carry + tot_g;
            first_t[kSmallThreads] = tie_carry + tot_t;
        }
        __syncthreads();
        // entries above T: position e of the selection is entry e - first_g[j] of the list j with first_g[j] <= e < first_g[j + 1]
        const uint32_t end_g = gt_carry + tot_g;
        for (uint32_t e0 = gt_carry + threadIdx.x; e0 < end_g; e0 += 4 * kSmallThreads) {
            uint64_t w[4];
            bool take[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {   // four loads in flight
                const uint32_t e = e0 + u * kSmallThreads < end_g ? e0 + u * kSmallThreads : end_g - 1;
                int lo = 0;
#pragma unroll
                for (int step = kSmallThreads / 2; step > 0; step >>= 1) lo += first_g[lo + step] <= e ? step : 0;
                const uint32_t i = e - first_g[lo];
                take[u] = e0 + u * kSmallThreads < end_g && (list_skip[lo] & 1) == 0;
                w[u] = stage[base + lo].gt[i < (uint32_t)kStageCap ? i : (uint32_t)kStageCap - 1u];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (take[u]) put_selected(sel, (int)n_gt, e0 + u * kSmallThreads, w[u]);
        }
        // Ties from the lists that are taken whole (the quota does not run out inside them): list j's ties hold the
        // ranks first_t[j] .. first_t[j + 1] - 1 among the segment's ties, in the order of their indices.  A list
        // itself is in no order, so its entries are ranked among themselves, from a copy in LDS behind the entries
        // above T.  The segment's workgroups take turns list by list.
        const uint32_t end_t = tie_carry + tot_t < k_eq ? tie_carry + tot_t : k_eq;
        for (uint32_t r0 = tie_carry + threadIdx.x; r0 < end_t; r0 += 4 * kSmallThreads) {
            uint32_t w[4];
            bool take[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {   // four loads in flight
                const uint32_t r = r0 + u * kSmallThreads < end_t ? r0 + u * kSmallThreads : end_t - 1;
                int lo = 0;
#pragma unroll
                for (int step = kSmallThreads / 2; step > 0; step >>= 1) lo += first_t[lo + step] <= r ? step : 0;
                const uint32_t i = r - first_t[lo];
                take[u] = r0 + u * kSmallThreads < end_t && (list_skip[lo] & 2) == 0 && (base + lo) % share == part && i < (uint32_t)kStageCap;
                w[u] = stage[base + lo].tie[i < (uint32_t)kStageCap ? i : (uint32_t)kStageCap - 1u];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (take[u]) put_selected(sel, k, n_gt + r0 + u * kSmallThreads, (uint64_t)w[u]);
        }
        __syncthreads();
        for (uint32_t r = tie_carry + threadIdx.x; r < end_t; r += kSmallThreads) {
            int lo = 0;
#pragma unroll
            for (int step = kSmallThreads / 2; step > 0; step >>= 1) lo += first_t[lo + step] <= r ? step : 0;
            if ((list_skip[lo] & 2) == 0 && (base + lo) % share == part && n_gt + first_t[lo + 1] <= (uint32_t)k) {
                const uint32_t me = (uint32_t)sel[slot(n_gt + r)];
                uint32_t rank = 0;
                for (uint32_t q = first_t[lo]; q < first_t[lo + 1]; ++q) rank += (uint32_t)sel[slot(n_gt + q)] < me ? 1u : 0u;
                put_tie_row(k, n_gt + first_t[lo] + rank, me, T, score, idx_out, val_out, s, seg.begin, seg.end);
            }
        }
        gt_carry += tot_g;
        tie_carry += tot_t;
        __syncthreads();   // the offsets are rewritten for the next kSmallThreads lists
    }
    __syncthreads();

    // the workgroup where the quota runs out: its smallest indices, by rank among its (at most kStageCap) ties
    if (partial_block >= 0) {
        const Stage& pb = stage[partial_block];
        const uint32_t ct = pb.n_tie < (uint32_t)kStageCap ? pb.n_tie : (uint32_t)kStageCap, want = k_eq - partial_before;
        for (uint32_t i = threadIdx.x; i < ct; i += kSmallThreads) tie_buf[i] = pb.tie[i];
        __syncthreads();
        for (uint32_t i = threadIdx.x; i < ct; i += kSmallThreads) {
            const uint32_t me = tie_buf[i];
            uint32_t rank = 0;
            for (uint32_t j = 0; j < ct; ++j) rank += tie_buf[j] < me ? 1u : 0u;
            if (rank < want) put_tie_row(k, n_gt + partial_before + rank, me, T, score, idx_out, val_out, s, seg.begin, seg.end);
        }
    }
    __syncthreads();

    // overflowed lists: read those spans again, entries above T to their reserved range, ties in index order
    const uint32_t todo = n_redo < 64 ? n_redo : 64;
    for (uint32_t r = 0; r < todo; ++r) {
        const int b = redo[r];
        const bool for_gt = (redo_what[r] & 1) != 0, for_ties = (redo_what[r] & 2) != 0;
        const int64_t lo = seg.begin + (int64_t)(b - b0) * span;
        const int64_t hi = lo + span < seg.end ? lo + span : seg.end;
        if (threadIdx.x == 0) redo_fill = 0;
        __syncthreads();
        uint32_t tie_before = redo_tie_before[r];
        // A wavefront takes kWave * kRedoPer neighbouring entries, lane by lane (coalesced reads): ties keep their index
        // order through counts of comparison masks inside the wavefront and one exchange of the wavefronts' totals per
        // kSmallThreads * kRedoPer entries.
        constexpr int kRedoPer = 16;
        const int lane = lane_id(), wave = threadIdx.x >> 6;
        for (int64_t base = lo; base < hi; base += (int64_t)kSmallThreads * kRedoPer) {
            if (!for_gt && tie_before >= k_eq) break;   // the quota ran out inside this span: nothing more to find
            const int64_t first = base + (int64_t)wave * (kWave * kRedoPer) + lane;
            float val[kRedoPer];   // all loads in flight together (an entry past the end reads the last one and is not used)
#pragma unroll
            for (int j = 0; j < kRedoPer; ++j) val[j] = score[first + j * kWave < hi ? first + j * kWave : hi - 1];
            uint32_t key[kRedoPer];
#pragma unroll
            for (int j = 0; j < kRedoPer; ++j) key[j] = key_of(val[j]);
            if (for_gt) {
#pragma unroll
                for (int j = 0; j < kRedoPer; ++j)
                    if (first + j * kWave < hi && key[j] > T)
                        put_selected(sel, (int)n_gt, redo_gt_at[r] + atomicAdd(&redo_fill, 1u), compose(key[j], (uint32_t)(first + j * kWave)));
            }
            if (for_ties && tie_before < k_eq) {
                uint32_t before_mine[kRedoPer], wave_ties = 0;   // ties of this wavefront before each of this lane's entries
#pragma unroll
                for (int j = 0; j < kRedoPer; ++j) {
                    const unsigned long long m = __ballot(first + j * kWave < hi && key[j] == T);
                    before_mine[j] = wave_ties + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
                    wave_ties += (uint32_t)__popcll(m);
                }
                __syncthreads();  // wave_tot may still be read from an earlier exchange
                if (lane == 0) wave_tot[wave] = wave_ties;
                __syncthreads();
                uint32_t before = 0, all = 0;
#pragma unroll
                for (int w2 = 0; w2 < kSmallThreads / kWave; ++w2) {
                    const uint32_t t = wave_tot[w2];
                    before += w2 < wave ? t : 0u;
                    all += t;
                }
#pragma unroll
                for (int j = 0; j < kRedoPer; ++j) {
                    const uint32_t rank = tie_before + before + before_mine[j];
                    if (first + j * kWave < hi && key[j] == T && rank < k_eq)
                        put_tie_row(k, n_gt + rank, (uint32_t)(first + j * kWave), T, score, idx_out, val_out, s, seg.begin, seg.end);
                }
                tie_before += all;
            }
        }
        __syncthreads();
    }
    if (n_gt == 0) return;
    if (share == 1) {
        finish_segment<kSmallThreads>(sel, (int)n_gt, score, idx_out, val_out, s, seg.begin, seg.end, k);
    } else {
        // Which words this workgroup ranks.  Copied from the lists alone, the words have the same places in every
        // workgroup of the segment, and the places are dealt out in turn: no workgroup gets more than the others.
        // Places filled from a span that was read again differ between workgroups; then a hash of the index decides.
        if (threadIdx.x == 0) n_own = 0;
        __syncthreads();
        if (gt_reread == 0) {
            // places part, part + share, ...: no list to build
            const int mine = (int)n_gt > part ? ((int)n_gt - part + share - 1) / share : 0;
            rank_rows<kSmallThreads>(sel, (int)n_gt, nullptr, part, share, mine, cnt, score, idx_out, val_out, s, seg.begin, seg.end, k);
        } else {
            for (int e = threadIdx.x; e < (int)n_gt; e += kSmallThreads) {
                const uint32_t h = (index_of(sel[slot(e)]) * 2654435761u) >> 16;
                if ((int)(h % (uint32_t)share) == part) own[atomicAdd(&n_own, 1u)] = (uint16_t)e;
            }
            __syncthreads();
            rank_rows<kSmallThreads>(sel, (int)n_gt, own, 0, 1, (int)n_own, cnt, score, idx_out, val_out, s, seg.begin, seg.end, k);
        }
    }
}

struct Layout {
    size_t segs, state, hist, stage, block_max, total;
    size_t stage_slots;
    int R;
};

constexpr int kFewSegs = 64;   // segment tables up to this length are built on the stack
constexpr int kComputeUnits = 256;   // of the part this library is written for (gfx950 in its full configuration)

int hist_copies(int32_t n_sg) { return n_sg <= 16 ? 8 : n_sg <= 64 ? 4 : 1; }

// entries per workgroup of the large route: whole sweeps, and at most 512 workgroups per launch, which is what 256
// CUs hold at once (two workgroups of 1024 threads each): a launch then runs as a single wave of workgroups
// (quarter sweeps for populations that leave CUs idle were measured: more workgroups add to the segment's histograms
// and lists, 11 -> 14 us for the funnel launch on a million entries)
int64_t span_for(int64_t n, int32_t n_sg)
{
    const int64_t sweeps = (n + kRow - 1) / kRow + n_sg;
    return kRow * ((sweeps + 511) / 512);
}

// with_block_max: room for the largest key of every 256 entries (4 bytes per 256 entries: the one part that grows with n)
Layout layout(int64_t n, int32_t n_sg, int32_t k, bool with_block_max)
{
    (void)k;
    Layout L;
    L.R = hist_copies(n_sg);
    // workgroups of a sweep launch: at most 512 whole spans plus one partial span per segment
    const size_t sweeps = (size_t)(n / kRow);
    const size_t blocks = (sweeps < 512 ? sweeps : 512) + (size_t)n_sg + 1;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += round_up(bytes, 256);
        return at;
    };
    L.segs = take((size_t)n_sg * sizeof(SegT));
    L.state = take((size_t)3 * n_sg * sizeof(SelState));
    L.hist = take(((size_t)L.R + 2) * n_sg * kBins * sizeof(uint32_t));   // first digit in R copies, one each for the others
    L.stage = take(blocks * sizeof(Stage));
    L.stage_slots = blocks;
    L.block_max = with_block_max ? take(((size_t)(n >> 8) + (size_t)n_sg + 1) * sizeof(uint32_t)) : 0;
    L.total = off;
    return L;
}

}  // namespace

size_t topk_workspace_bytes(int64_t n, int32_t n_sg, int32_t k)
{
    if (n < 0) n = 0;
    if (n_sg < 1) n_sg = 1;
    if (k < 1) k = 1;
    return layout(n, n_sg, k, true).total;
}


// what every selection call refuses about its segments and k (host pointers only); *longest: the longest segment
static int topk_check(const int64_t* seg_off, int32_t n_sg, int32_t k, int64_t* longest)
{
    if (!seg_off || n_sg < 1 || n_sg > PRUNER_MAX_SUBGRAPHS || k < 1 || k > PRUNER_MAX_K) return PRUNER_EINVAL;
    if (seg_off[0] != 0) return PRUNER_EINVAL;
    *longest = 0;
    for (int32_t s = 0; s < n_sg; ++s) {
        const int64_t len = seg_off[s + 1] - seg_off[s];
        if (len < k) return PRUNER_EINVAL;
        *longest = len > *longest ? len : *longest;
    }
    if (seg_off[n_sg] > 0x7FFFFFFFll) return PRUNER_EINVAL;  // indices are int32
    return PRUNER_OK;
}

int topk_prepare(const int64_t* seg_off, int32_t n_sg, int32_t k, void* workspace, size_t workspace_bytes, hipStream_t st, TopkCtx* ctx,
                 Upload* defer, bool with_block_max)
{
    int64_t longest = 0;
    const int bad = topk_check(seg_off, n_sg, k, &longest);
    if (bad) return bad;
    const int64_t n = seg_off[n_sg];
    if (!workspace || !aligned(workspace, 256)) return PRUNER_EWORKSPACE;
    const Layout L = layout(n, n_sg, k, with_block_max);
    if (workspace_bytes < L.total) return PRUNER_EWORKSPACE;

    char* ws = static_cast<char*>(workspace);
    SegT* d_segs = reinterpret_cast<SegT*>(ws + L.segs);
    const bool small = longest <= kSmallMax;
    const int64_t span = span_for(n, n_sg);

    // the segment table: on the stack when it is short (a call that must not allocate stays off the heap as well)
    SegT few[kFewSegs];
    std::vector<SegT> many;
    if (n_sg > kFewSegs) many.resize(n_sg);
    SegT* const segs = n_sg > kFewSegs ? many.data() : few;
    int64_t blocks = 0;
    for (int32_t s = 0; s < n_sg; ++s) {
        segs[s] = SegT{seg_off[s], seg_off[s + 1], (int32_t)blocks, 0};
        blocks += (seg_off[s + 1] - seg_off[s] + span - 1) / span;
    }
    ctx->large = !small;
    ctx->n_sg = n_sg;
    ctx->k = k;
    ctx->n = n;
    ctx->span = span;
    ctx->blocks = (int32_t)blocks;
    ctx->copies = L.R;
    ctx->wide = false;
    ctx->d_segs = d_segs;
    ctx->d_state = ws + L.state;
    ctx->d_hist = reinterpret_cast<uint32_t*>(ws + L.hist);
    ctx->d_stage = ws + L.stage;
    // Block maxima pay where nearly every block of 256 entries can be stepped over: at most one entry in 1024 selected
    // in the longest segment (with k = 512 of 50,000 nine blocks in ten hold a selected entry and the maxima are one
    // more read: 10.7 -> 11.5 us measured).
    const bool sparse = longest >= (int64_t)k * 1024;
    ctx->d_block_max = with_block_max && sparse ? reinterpret_cast<uint32_t*>(ws + L.block_max) : nullptr;
    ctx->inline_ok = false;
    static_assert(sizeof(InlineSegs) <= sizeof(ctx->inline_segs), "inline segment table");
    if (small) {
        if (n_sg <= kInlineSegs) {
            memset(ctx->inline_segs, 0, sizeof(InlineSegs));
            memcpy(ctx->inline_segs, segs, (size_t)n_sg * sizeof(SegT));
            ctx->inline_ok = true;
            return PRUNER_OK;
        }
        if (defer) {
            defer->bytes.assign(reinterpret_cast<const char*>(segs), reinterpret_cast<const char*>(segs + n_sg));
            defer->dst = d_segs;
            return PRUNER_OK;
        }
        return put_table(d_segs, segs, (size_t)n_sg * sizeof(SegT), st);
    }
    if ((size_t)blocks > L.stage_slots) return PRUNER_EWORKSPACE;   // cannot happen: spans are sized for at most that many
    // segment table, and histograms cleared, in one launch
    const size_t per_pass = (size_t)n_sg * kBins;
    const size_t hist_bytes = ((size_t)L.R + 2) * per_pass * sizeof(uint32_t);
    if (defer) {
        defer->bytes.assign(reinterpret_cast<const char*>(segs), reinterpret_cast<const char*>(segs + n_sg));
        defer->dst = d_segs;
        defer->zero = ctx->d_hist;
        defer->zero_bytes = hist_bytes;
        return PRUNER_OK;
    }
    return put_table(d_segs, segs, (size_t)n_sg * sizeof(SegT), st, ctx->d_hist, hist_bytes);
}

int topk_finish(const TopkCtx& ctx, const float* score, const int64_t* seg_off, int32_t* idx_out, float* val_out, bool have_first_digit,
                hipStream_t st)
{
    if (!score || !idx_out) return PRUNER_EINVAL;
    if (!aligned(score, 4) || !aligned(idx_out, 4) || (val_out && !aligned(val_out, 4))) return PRUNER_EINVAL;
    const int32_t n_sg = ctx.n_sg, k = ctx.k;
    const SegT* d_segs = static_cast<const SegT*>(ctx.d_segs);
    bool resident = true;   // small route: every segment fits one batch of a workgroup
    for (int32_t s2 = 0; s2 < n_sg; ++s2) resident = resident && seg_off[s2 + 1] - seg_off[s2] <= (int64_t)kSmallThreads * kSmallPer;
    if (!ctx.large) {
        InlineSegs args;
        memset(&args, 0, sizeof args);
        bool tiny = k <= kTinyK;
        for (int32_t s2 = 0; s2 < n_sg; ++s2) tiny = tiny && seg_off[s2 + 1] - seg_off[s2] <= (int64_t)kTinyMax;
        if (tiny) {
            if (ctx.inline_ok) {
                memcpy(&args, ctx.inline_segs, sizeof args);
                hipLaunchKernelGGL(topk_tiny_kernel<true>, dim3(n_sg), dim3(kTinyThreads), 0, st, score, d_segs, args, k, idx_out, val_out);
            } else {
                hipLaunchKernelGGL(topk_tiny_kernel<false>, dim3(n_sg), dim3(kTinyThreads), 0, st, score, d_segs, args, k, idx_out, val_out);
            }
            PRUNER_LAUNCH_CHECK();
            return PRUNER_OK;
        }
        if (ctx.inline_ok) {
            memcpy(&args, ctx.inline_segs, sizeof args);
            if (resident) hipLaunchKernelGGL((topk_small_kernel<true, true>), dim3(n_sg), dim3(kSmallThreads), 0, st, score, d_segs, args, k, idx_out, val_out);
            else hipLaunchKernelGGL((topk_small_kernel<true, false>), dim3(n_sg), dim3(kSmallThreads), 0, st, score, d_segs, args, k, idx_out, val_out);
        } else {
            if (resident) hipLaunchKernelGGL((topk_small_kernel<false, true>), dim3(n_sg), dim3(kSmallThreads), 0, st, score, d_segs, args, k, idx_out, val_out);
            else hipLaunchKernelGGL((topk_small_kernel<false, false>), dim3(n_sg), dim3(kSmallThreads), 0, st, score, d_segs, args, k, idx_out, val_out);
        }
        PRUNER_LAUNCH_CHECK();
        return PRUNER_OK;
    }

    SelState* d_state = static_cast<SelState*>(ctx.d_state);
    Stage* d_stage = static_cast<Stage*>(ctx.d_stage);
    const int R = ctx.copies;
    const int64_t span = ctx.span;
    const size_t per_pass = (size_t)n_sg * kBins;
    uint32_t *hist0 = ctx.d_hist, *hist1 = ctx.d_hist + (size_t)R * per_pass, *hist2 = hist1 + per_pass;
    const dim3 chunks((unsigned)ctx.blocks);
    bool wide = aligned(score, 16);
    for (int32_t s2 = 0; s2 < n_sg; ++s2) wide = wide && seg_off[s2] % 4 == 0;
#define PRUNER_SWEEP_LAUNCH(KERNEL, ...)                                                                          \
    do {                                                                                                          \
        if (wide) hipLaunchKernelGGL((KERNEL<true>), chunks, dim3(kBigThreads), 0, st, __VA_ARGS__);              \
        else hipLaunchKernelGGL((KERNEL<false>), chunks, dim3(kBigThreads), 0, st, __VA_ARGS__);                  \
        PRUNER_LAUNCH_CHECK();                                                                                    \
    } while (0)
    // (the draft kernel writes the block maxima when it counts the first digit: at its full load width, which is `wide` here)
    uint32_t* const block_max = wide ? ctx.d_block_max : nullptr;
    if (!have_first_digit) PRUNER_SWEEP_LAUNCH(hist0_kernel, score, d_segs, n_sg, span, R, hist0, block_max);
    if (block_max) hipLaunchKernelGGL((funnel_kernel<true, true>), chunks, dim3(kBigThreads), 0, st, score, d_segs, n_sg, span, R, k, hist0, hist1, d_state, d_stage, block_max);
    else if (wide) hipLaunchKernelGGL((funnel_kernel<true, false>), chunks, dim3(kBigThreads), 0, st, score, d_segs, n_sg, span, R, k, hist0, hist1, d_state, d_stage, block_max);
    else hipLaunchKernelGGL((funnel_kernel<false, false>), chunks, dim3(kBigThreads), 0, st, score, d_segs, n_sg, span, R, k, hist0, hist1, d_state, d_stage, block_max);
    PRUNER_LAUNCH_CHECK();
    PRUNER_SWEEP_LAUNCH(refine_kernel, score, d_segs, n_sg, span, hist1, hist2, d_state, d_stage);
    PRUNER_SWEEP_LAUNCH(settle_kernel, score, d_segs, n_sg, span, k, hist2, d_state, d_stage);
#undef PRUNER_SWEEP_LAUNCH
    // the ranking of a segment's k rows is shared out over up to k / 32 workgroups, as long as the launch is one
    // workgroup per compute unit at most (a compute unit holds one of these workgroups at a time: a launch of more
    // takes a second round, which costs more than longer rankings do)
    int share = (k + 31) / 32;
    if (share > kComputeUnits / n_sg) share = kComputeUnits / n_sg;
    if (share < 1) share = 1;
    hipLaunchKernelGGL(gather_sort_kernel, dim3((unsigned)(n_sg * share)), dim3(kSmallThreads), 0, st, score, d_segs, n_sg, ctx.blocks, span,
                       d_state, d_stage, k, share, idx_out, val_out);
    PRUNER_LAUNCH_CHECK();
    return PRUNER_OK;
}

}  // namespace pruner

using namespace pruner;

extern "C" int pruner_topk(const float* score, const int64_t* seg_off, int32_t n_sg, int32_t k, int32_t* idx_out, float* val_out,
                           void* workspace, size_t workspace_bytes, void* stream)
{
    if (!score || !idx_out) return PRUNER_EINVAL;
    if (!aligned(score, 4) || !aligned(idx_out, 4) || (val_out && !aligned(val_out, 4))) return PRUNER_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    TopkCtx ctx;
    const int rc = topk_prepare(seg_off, n_sg, k, workspace, workspace_bytes, st, &ctx);
    if (rc) return rc;
    return topk_finish(ctx, score, seg_off, idx_out, val_out, false, st);
}


// ---- selection without a workspace argument -------------------------------------------------------------------------
// The scratch of pruner_topk (segment table, selection state, digit histograms, staging slots) in a file-scope device
// array, for callers that cannot allocate.  One array per device, held until the process ends; every call on a device
// uses it, so calls that overlap on one device race.  Nothing in it has to survive between calls: the histograms are
// cleared by the call's first launch, every other part is written before it is read.
namespace {
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
void* g_scratch_ptr[kMaxDevices];   // the array's device address on each device, looked up once
}  // namespace

extern "C" int pruner_topk_static(const float* score, const int64_t* seg_off, int32_t n_sg, int32_t k, int32_t* idx_out, float* val_out,
                                  void* stream)
{
    if (!score || !idx_out || !seg_off) return PRUNER_EINVAL;
    if (!aligned(score, 4) || !aligned(idx_out, 4) || (val_out && !aligned(val_out, 4))) return PRUNER_EINVAL;
    if (n_sg > PRUNER_STATIC_MAX_SEGMENTS) return PRUNER_EINVAL;
    static_assert(PRUNER_STATIC_MAX_SEGMENTS <= kFewSegs, "the segment table of a static call is built on the stack");
    int64_t longest = 0;
    const int bad = topk_check(seg_off, n_sg, k, &longest);
    if (bad) return bad;
    // the scratch a call of this size needs (it grows with the segment count, hardly with n)
    if (layout(seg_off[n_sg], n_sg, k, false).total > kStaticScratchBytes) return PRUNER_EWORKSPACE;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return PRUNER_EHIP;
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PRUNER_EHIP;
        g_scratch_ptr[dev] = p;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    TopkCtx ctx;
    const int rc = topk_prepare(seg_off, n_sg, k, g_scratch_ptr[dev], kStaticScratchBytes, st, &ctx, nullptr, false);
    if (rc) return rc;
    return topk_finish(ctx, score, seg_off, idx_out, val_out, false, st);
}
