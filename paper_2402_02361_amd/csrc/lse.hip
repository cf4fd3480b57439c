// Latent Schedule Explorer (Alg. 2) with the population resident on the device:
//   n_steps times { costs = C_SA(S_x);  S_spec = PriorFilter(S_x U S_spec);  S_x = SchMutation(S_x, costs) }.
//
// C_SA and the k best of S_x are the launches of pruner_prior_filter.  The rest of a step:
//   lse_keys    one thread per entry of the union: score key and schedule hash (the k best sit at random places of
//               the population; many workgroups share those reads)
//   lse_merge   one workgroup per subgraph: the union of S_spec and the k best of S_x as a union of SETS (a schedule
//               counts once; identity = score and a 64-bit hash of the tile factors): the order is (score descending,
//               hash ascending, position ascending); the k best of S_x are sorted in LDS, S_spec is in that order
//               already, the two are merged by bisection; copies of a predecessor are dropped, the first k of the
//               rest are the new S_spec
//   lse_copy    the tile factors of the new S_spec, from the old S_spec or from the population; also as one 64-byte
//               record per schedule, from which the mutation reads its parents
//   lse_mutate  one thread per child: a parent drawn uniformly from S_spec (truncation selection: the paper names a
//               genetic algorithm guided by the draft fitness and gives no operator), and with the given probability
//               one prime factor of one tile factor moved to another level of the same axis, fragment multiples kept
// When the population is large enough for one draft launch per loop-nest class, the mutation of a step is not a
// launch of its own: the next step's draft kernels make the children, store them and score them while they are in
// registers (the population is then written once per step and never read for scoring); only the last step's
// mutation, whose children nobody scores, is a launch.
// Random numbers are counter-based (SplitMix64, Steele/Lea/Flood OOPSLA 2014: draw c is the c-th output of the
// generator started from the seed), so the result does not depend on how the work is laid out.
#include "lse_child.h"

#include <string.h>

#include <vector>

namespace pruner {
namespace {

constexpr int kLseThreads = 1024;

__device__ __forceinline__ uint64_t splitmix64_draw(uint64_t seed, uint64_t c)
{
    uint64_t z = seed + c * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// identity of a schedule: its own tile slots, in slot order (all slots are requested before the first is hashed)
__device__ __forceinline__ uint64_t schedule_hash(const uint16_t* __restrict__ col, int64_t stride, int n_slots)
{
    uint16_t f[PRUNER_MAX_SLOTS];
#pragma unroll
    for (int r = 0; r < PRUNER_MAX_SLOTS; ++r) f[r] = r < n_slots ? col[r * stride] : (uint16_t)0;
    uint64_t h = (uint64_t)n_slots;
#pragma unroll
    for (int r = 0; r < PRUNER_MAX_SLOTS; ++r)
        if (r < n_slots) h = splitmix64_draw(h, (uint64_t)f[r] + 1);
    return h;
}

__device__ __forceinline__ uint32_t lse_key_of(float x)   // larger score <=> larger key; -0 and +0 share a key
{
    uint32_t u = __float_as_uint(x);
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float lse_score_of(uint32_t key) { return __uint_as_float((key & 0x80000000u) ? (key & 0x7FFFFFFFu) : ~key); }

constexpr int32_t kNoSource = (int32_t)0x80000000;

// Entry e of the sort arrays sits at pad(e): one spare entry after every 32, so that threads that walk groups of 8
// neighbouring entries do not all land in the same LDS banks.
__device__ __forceinline__ int pad(int e) { return e + (e >> 5); }
constexpr int padded(int n) { return n + (n >> 5) + 2; }

// 2^LOG entries base + i*s of a bitonic merge of `size`: the strides 2^(LOG-1) s ... s permute them among themselves,
// and they lie in one half of the merge, so they share the direction.
template <int LOG> __device__ __forceinline__ void sort_group(uint64_t* hi, uint64_t* lo, int g, int s, int size)
{
    constexpr int N = 1 << LOG;
    const int base = (g / s) * (N * s) + (g % s);
    const bool down = (base & size) == 0;
    uint64_t xh[N], xl[N];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        xh[i] = hi[pad(base + i * s)];
        xl[i] = lo[pad(base + i * s)];
    }
#pragma unroll
    for (int h = N >> 1; h > 0; h >>= 1) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            if ((i & h) == 0) {
                const uint64_t ah = xh[i], al = xl[i], bh = xh[i + h], bl = xl[i + h];
                const bool a_less = ah < bh || (ah == bh && al < bl);
                const bool swap = a_less == down;
                xh[i] = swap ? bh : ah;
                xl[i] = swap ? bl : al;
                xh[i + h] = swap ? ah : bh;
                xl[i + h] = swap ? al : bl;
            }
        }
    }
#pragma unroll
    for (int i = 0; i < N; ++i) {
        hi[pad(base + i * s)] = xh[i];
        lo[pad(base + i * s)] = xl[i];
    }
}

// The sort keys of the union's P entries per subgraph (old S_spec first, then the k best of S_x, then padding), one
// thread per entry: hi = score key << 32 | upper half of ~hash, lo = lower half of ~hash << 32 | ~position.  The
// schedules of the k best sit at random places of the population: many workgroups share those reads.
// (One wavefront per workgroup: the reads are random single elements of a population far larger than the caches, and
// what bounds them is how many misses a compute unit keeps in flight; the launch therefore spreads over all units.)
constexpr int kKeysThreads = 64;
__global__ void __launch_bounds__(kKeysThreads) lse_keys_kernel(const LseSeg* __restrict__ segs, int k, int P, const uint16_t* __restrict__ tiles,
                                                       int64_t pitch, const int32_t* __restrict__ best_idx, const float* __restrict__ best_val,
                                                       const uint16_t* __restrict__ old_tiles, const float* __restrict__ old_score,
                                                       const int32_t* __restrict__ old_count, int64_t spec_pitch,
                                                       uint64_t* __restrict__ key_hi, uint64_t* __restrict__ key_lo)
{
    const int s = blockIdx.y;
    const int i = blockIdx.x * kKeysThreads + threadIdx.x;
    if (i >= P) return;
    const int n_slots = segs[s].n_slots;
    const int64_t col0 = (int64_t)s * k;
    const int n_old = old_count[s] < 0 ? 0 : old_count[s] > k ? k : old_count[s];
    uint64_t h = 0, l = 0;   // padding sorts last: every real entry has a non-zero key
    if (i < n_old + k) {
        float sc;
        uint64_t hash;
        if (i < n_old) {
            sc = old_score[col0 + i];
            hash = schedule_hash(old_tiles + col0 + i, spec_pitch, n_slots);
        } else {
            const int r = i - n_old;
            sc = best_val[col0 + r];
            hash = schedule_hash(tiles + best_idx[col0 + r], pitch, n_slots);
        }
        const uint64_t inv = ~hash;
        h = ((uint64_t)lse_key_of(sc) << 32) | (inv >> 32);
        l = (inv << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)i);
    }
    key_hi[(int64_t)s * P + i] = h;
    key_lo[(int64_t)s * P + i] = l;
}

// One workgroup per subgraph.  The old S_spec arrives in order (it is an earlier call's output: keys strictly
// descending), so only the k best of S_x are sorted (Pn = 2^m >= k entries, padding last), and the union's order is
// a merge: an entry's place is its place in its own list plus the number of entries of the other list that precede
// it, found by bisection.  Dynamic LDS: the old keys (2 x k words), the new ones (2 x padded(Pn) words), and which
// entry holds each place of the union (2 k half-words).  P is the stride of the key arrays.
__device__ __forceinline__ bool key_greater(uint64_t ah, uint64_t al, uint64_t bh, uint64_t bl) { return ah > bh || (ah == bh && al > bl); }

__global__ void __launch_bounds__(kLseThreads) lse_merge_kernel(int k, int P, int Pn, const uint64_t* __restrict__ key_hi,
                                                                const uint64_t* __restrict__ key_lo, const int32_t* __restrict__ best_idx,
                                                                const int32_t* __restrict__ old_count, float* __restrict__ new_score,
                                                                int32_t* __restrict__ new_count, int32_t* __restrict__ source)
{
    extern __shared__ uint64_t words[];
    uint64_t* oh = words;
    uint64_t* ol = oh + k;
    uint64_t* hi = ol + k;
    uint64_t* lo = hi + padded(Pn);
    uint16_t* who = reinterpret_cast<uint16_t*>(lo + padded(Pn));
    __shared__ uint32_t wave_tot[kLseThreads / kWave];
    const int s = blockIdx.x;
    const int64_t col0 = (int64_t)s * k;
    const int n_old = old_count[s] < 0 ? 0 : old_count[s] > k ? k : old_count[s];
    const int m = n_old + k;
    for (int i = threadIdx.x; i < n_old; i += kLseThreads) {
        oh[i] = key_hi[(int64_t)s * P + i];
        ol[i] = key_lo[(int64_t)s * P + i];
    }
    for (int i = threadIdx.x; i < Pn; i += kLseThreads) {
        hi[pad(i)] = i < k ? key_hi[(int64_t)s * P + n_old + i] : 0ull;   // padding sorts last: every real entry has a non-zero key
        lo[pad(i)] = i < k ? key_lo[(int64_t)s * P + n_old + i] : 0ull;
    }
    // bitonic sort, largest (hi, lo) first; one round trip through LDS performs up to three consecutive strides
    // (a thread takes the 8, 4 or 2 entries those strides permute among themselves and exchanges them in registers)
    for (int size = 2; size <= Pn; size <<= 1) {
        int stride = size >> 1;
        while (stride > 0) {
            __syncthreads();
            if (stride >= 4) {
                const int st = stride >> 2;
                for (int g = threadIdx.x; g < (Pn >> 3); g += kLseThreads) sort_group<3>(hi, lo, g, st, size);
                stride >>= 3;
            } else if (stride == 2) {
                for (int g = threadIdx.x; g < (Pn >> 2); g += kLseThreads) sort_group<2>(hi, lo, g, 1, size);
                stride = 0;
            } else {
                for (int g = threadIdx.x; g < (Pn >> 1); g += kLseThreads) sort_group<1>(hi, lo, g, 1, size);
                stride = 0;
            }
        }
    }
    __syncthreads();
    // places in the union (all 128-bit keys differ: they carry the position)
    for (int i = threadIdx.x; i < m; i += kLseThreads) {
        const bool is_old = i < n_old;
        const int j = is_old ? i : i - n_old;
        const uint64_t xh = is_old ? oh[j] : hi[pad(j)], xl = is_old ? ol[j] : lo[pad(j)];
        int a = 0, e = is_old ? k : n_old;   // entries of the other list that are greater
        while (a < e) {
            const int mid = (a + e) >> 1;
            const bool g = is_old ? key_greater(hi[pad(mid)], lo[pad(mid)], xh, xl) : key_greater(oh[mid], ol[mid], xh, xl);
            if (g) a = mid + 1; else e = mid;
        }
        who[j + a] = (uint16_t)(is_old ? j : k + j);
    }
    __syncthreads();
    // a copy has the key and the hash of its predecessor; number the rest.  A thread takes kPer neighbouring places, so
    // that one scan over the workgroup numbers a whole sweep of kPer * kLseThreads places (all 2 k of them as a rule).
    constexpr int kPer = 8;
    uint32_t carry = 0;
    for (int base = 0; base < m; base += kPer * kLseThreads) {
        const int first = base + (int)threadIdx.x * kPer;
        uint64_t mh[kPer], ml[kPer];
        uint32_t keep = 0;   // bit j: place first + j stays
        uint64_t ph = 0, pl = 0;
        if (first > 0 && first < m) {
            const int pid = who[first - 1];
            ph = pid < k ? oh[pid] : hi[pad(pid - k)];
            pl = pid < k ? ol[pid] : lo[pad(pid - k)];
        }
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            mh[j] = ml[j] = 0;
            if (first + j < m) {
                const int id = who[first + j];
                mh[j] = id < k ? oh[id] : hi[pad(id - k)];
                ml[j] = id < k ? ol[id] : lo[pad(id - k)];
                const bool same = first + j > 0 && mh[j] == ph && (ml[j] >> 32) == (pl >> 32);
                keep |= same ? 0u : 1u << j;
                ph = mh[j], pl = ml[j];
            }
        }
        // exclusive scan of the kept counts over the workgroup
        const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
        const uint32_t mine = (uint32_t)__popc(keep);
        const uint32_t incl = wave_inclusive_sum(mine);
        __syncthreads();
        if (lane == kWave - 1) wave_tot[wave] = incl;
        __syncthreads();
        uint32_t before = 0, all = 0;
        for (int w2 = 0; w2 < kLseThreads / kWave; ++w2) {
            const uint32_t t = wave_tot[w2];
            before += w2 < wave ? t : 0u;
            all += t;
        }
        uint32_t rank = carry + before + incl - mine;
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            if ((keep >> j) & 1u) {
                if (rank < (uint32_t)k) {
                    const uint32_t pos = 0xFFFFFFFFu - (uint32_t)ml[j];
                    new_score[col0 + rank] = lse_score_of((uint32_t)(mh[j] >> 32));
                    source[col0 + rank] = pos < (uint32_t)n_old ? -1 - (int32_t)pos : best_idx[col0 + (pos - n_old)];
                }
                ++rank;
            }
        }
        carry += all;
    }
    const uint32_t count = carry < (uint32_t)k ? carry : (uint32_t)k;
    for (int r = count + threadIdx.x; r < k; r += kLseThreads) {
        new_score[col0 + r] = -__builtin_inff();
        source[col0 + r] = kNoSource;
    }
    if (threadIdx.x == 0) new_count[s] = (int32_t)count;
}

// The tile factors of the new S_spec; rows a subgraph does not own and entries past the count are cleared.  A second
// copy holds each schedule's factors side by side (32 x uint16 = 64 bytes): the mutation reads a parent from there
// with four loads instead of one per factor.
__global__ void __launch_bounds__(256) lse_copy_kernel(const LseSeg* __restrict__ segs, int n_sg, int k, int rows, const uint16_t* __restrict__ tiles,
                                                       int64_t pitch, const uint16_t* __restrict__ old_tiles, int64_t spec_pitch,
                                                       const int32_t* __restrict__ source, uint16_t* __restrict__ new_tiles,
                                                       uint4* __restrict__ new_aos)
{
    const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (c >= (int64_t)n_sg * k) return;
    const int s = (int)(c / k);
    const int n_slots = segs[s].n_slots;
    const int32_t src = source[c];
    uint32_t packed[kAosSlots / 2];
#pragma unroll
    for (int i = 0; i < kAosSlots / 2; ++i) packed[i] = 0u;
#pragma unroll
    for (int row = 0; row < PRUNER_MAX_SLOTS; ++row) {
        uint16_t v = 0;
        if (row < n_slots && src != kNoSource) v = src < 0 ? old_tiles[row * spec_pitch + (int64_t)s * k + (-1 - src)] : tiles[row * pitch + src];
        if (row < rows) new_tiles[row * spec_pitch + c] = v;
        packed[row >> 1] |= (uint32_t)v << (16 * (row & 1));
    }
#pragma unroll
    for (int q = 0; q < kAosSlots / 8; ++q) new_aos[c * (kAosSlots / 8) + q] = make_uint4(packed[4 * q], packed[4 * q + 1], packed[4 * q + 2], packed[4 * q + 3]);
}

// The segment of child j: the last one that begins at or before j (empty ones are skipped over).
__device__ __forceinline__ int lse_segment_of(const LseSeg* __restrict__ segs, int n_sg, int64_t j)
{
    int lo = 0, hi = n_sg - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (segs[mid].begin <= j) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// VEC children of one subgraph, neighbours in the population, and their stores (one per row when VEC > 1)
template <int VEC, int NP>
__device__ __forceinline__ void lse_children(const LseSeg& seg, int sub, int count, int k, uint64_t z0, const uint4* __restrict__ spec_aos,
                                             uint32_t mutate_q16, uint16_t* __restrict__ tiles, int64_t pitch, int64_t j0)
{
    uint32_t f[VEC][kAosWords];
#pragma unroll
    for (int e = 0; e < VEC; ++e) lse_child<NP>(seg, sub, count, k, z0 + (uint64_t)(2 * e) * kGamma, spec_aos, mutate_q16, f[e]);
#pragma unroll
    for (int row = 0; row < 8 * NP && row < PRUNER_MAX_SLOTS; ++row) {
        if (row < seg.n_slots) {
            if constexpr (VEC == 1) {
                tiles[row * pitch + j0] = (uint16_t)(f[0][row >> 1] >> (16 * (row & 1)));
            } else {
                // the row's factor of each child: the low or the high halves of two children's words at a time
                const uint32_t half = row & 1 ? 0x07060302u : 0x05040100u;
                const uint32_t w01 = __builtin_amdgcn_perm(f[1 % VEC][row >> 1], f[0][row >> 1], half);
                if constexpr (VEC == 4) {
                    const uint32_t w23 = __builtin_amdgcn_perm(f[3 % VEC][row >> 1], f[2 % VEC][row >> 1], half);
                    *reinterpret_cast<uint2*>(tiles + row * pitch + j0) = make_uint2(w01, w23);
                } else {
                    *reinterpret_cast<uint32_t*>(tiles + row * pitch + j0) = w01;
                }
            }
        }
    }
}
template <int VEC>
__device__ __forceinline__ void lse_children(const LseSeg& seg, int sub, int count, int k, uint64_t z0, const uint4* __restrict__ spec_aos,
                                             uint32_t mutate_q16, uint16_t* __restrict__ tiles, int64_t pitch, int64_t j0)
{
    switch ((seg.n_slots + 7) >> 3) {   // (the same for a whole wavefront but at a border between subgraphs)
        case 0:
        case 1: lse_children<VEC, 1>(seg, sub, count, k, z0, spec_aos, mutate_q16, tiles, pitch, j0); break;
        case 2: lse_children<VEC, 2>(seg, sub, count, k, z0, spec_aos, mutate_q16, tiles, pitch, j0); break;
        case 3: lse_children<VEC, 3>(seg, sub, count, k, z0, spec_aos, mutate_q16, tiles, pitch, j0); break;
        default: lse_children<VEC, 4>(seg, sub, count, k, z0, spec_aos, mutate_q16, tiles, pitch, j0); break;
    }
}

// VEC children per thread (neighbours in the population), stored VEC at a time.
// VEC > 1 needs a pitch that is a multiple of VEC and a population aligned to 2 VEC bytes.
template <int VEC>
__global__ void __launch_bounds__(256) lse_mutate_kernel(const LseSeg* __restrict__ segs, int n_sg, int k, int64_t n, uint16_t* __restrict__ tiles,
                                                         int64_t pitch, const uint4* __restrict__ spec_aos,
                                                         const int32_t* __restrict__ spec_count, uint64_t seed, uint64_t step,
                                                         uint32_t mutate_q16)
{
    const int64_t j0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * VEC;
    if (j0 >= n) return;
    const int sub = lse_segment_of(segs, n_sg, j0);
    const LseSeg seg = segs[sub];
    const uint64_t z0 = lse_child_state(seed, step, j0);
    if (VEC > 1 && j0 + VEC <= seg.end) {
        // all of this thread's children belong to one subgraph: one store per row
        const int count = spec_count[sub];
        if (count < 1) return;
        lse_children<VEC>(seg, sub, count, k, z0, spec_aos, mutate_q16, tiles, pitch, j0);
        return;
    }
    // a thread at a border between subgraphs (or VEC = 1): child by child
    for (int e = 0; e < VEC; ++e) {
        const int64_t j = j0 + e;
        if (j >= n) return;
        const int sj = e == 0 ? sub : lse_segment_of(segs, n_sg, j);
        const LseSeg sg = segs[sj];
        const int count = spec_count[sj];
        if (count < 1 || j >= sg.end) continue;
        lse_children<1>(sg, sj, count, k, z0 + (uint64_t)(2 * e) * kGamma, spec_aos, mutate_q16, tiles, pitch, j);
    }
}

struct LseLayout {
    size_t filter, table, best_idx, best_val, alt_tiles, alt_score, alt_count, zero_count, source, key_hi, key_lo, aos, total;
};

LseLayout lse_layout(int64_t n, int32_t n_sg, int32_t k, int32_t rows)
{
    LseLayout L;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += round_up(bytes, 256);
        return at;
    };
    const size_t cols = (size_t)n_sg * (size_t)k;
    L.filter = take(prior_filter_workspace_bytes(n, n_sg, k));
    L.table = take((size_t)n_sg * sizeof(LseSeg));
    L.best_idx = take(cols * sizeof(int32_t));
    L.best_val = take(cols * sizeof(float));
    L.alt_tiles = take((size_t)rows * cols * sizeof(uint16_t));
    L.alt_score = take(cols * sizeof(float));
    L.alt_count = take((size_t)n_sg * sizeof(int32_t));
    L.zero_count = take((size_t)n_sg * sizeof(int32_t));
    L.source = take(cols * sizeof(int32_t));
    L.key_hi = take(4 * cols * sizeof(uint64_t));   // P < 4k entries per subgraph (2k rounded up to a power of two)
    L.key_lo = take(4 * cols * sizeof(uint64_t));
    L.aos = take(cols * kAosSlots * sizeof(uint16_t));
    L.total = off;
    return L;
}

PerDeviceFlag g_merge_ready;   // the merge kernel's allowance of dynamic LDS has been raised

}  // namespace

size_t lse_workspace_bytes(int64_t n, int32_t n_sg, int32_t k, int32_t rows)
{
    if (n < 0) n = 0;
    if (n_sg < 1) n_sg = 1;
    if (k < 1) k = 1;
    if (rows < 1) rows = 1;
    return lse_layout(n, n_sg, k, rows).total;
}

}  // namespace pruner

using namespace pruner;

extern "C" int pruner_lse(const pruner_subgraph* sg, int32_t n_sg, const int64_t* seg_off, uint16_t* tiles, int64_t tiles_pitch,
                          int32_t tile_rows, int32_t flags, int32_t k, int32_t n_steps, uint64_t seed, uint32_t mutate_q16, float* score,
                          uint16_t* spec_tiles, float* spec_score, int32_t* spec_count, void* workspace, size_t workspace_bytes,
                          void* stream)
{
    if (!sg || !seg_off || n_sg < 1 || n_sg > PRUNER_MAX_SUBGRAPHS) return PRUNER_EINVAL;
    if (n_steps < 1 || mutate_q16 > 65536 || k < 1 || k > PRUNER_MAX_K || tile_rows < 1 || tile_rows > PRUNER_MAX_SLOTS) return PRUNER_EINVAL;
    if (!spec_tiles || !spec_score || !spec_count || !aligned(spec_tiles, 2) || !aligned(spec_score, 4) || !aligned(spec_count, 4))
        return PRUNER_EINVAL;
    if (!workspace || !aligned(workspace, 256)) return PRUNER_EWORKSPACE;
    const int64_t n = seg_off[n_sg];
    if (n < 0 || n > 0x7FFFFFFFll) return PRUNER_EINVAL;
    const LseLayout L = lse_layout(n, n_sg, k, tile_rows);
    if (workspace_bytes < L.total) return PRUNER_EWORKSPACE;
    char* ws = static_cast<char*>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);

    // everything the draft and selection stages refuse, before the first launch
    const size_t draft_bytes = round_up(draft_workspace_bytes(n_sg), 256);
    int rc = draft_check(sg, n_sg, seg_off, tiles, tiles_pitch, flags, score, nullptr, ws + L.filter, draft_bytes);
    if (rc) return rc;
    std::vector<LseSeg> table(n_sg);
    for (int32_t s = 0; s < n_sg; ++s) {
        if (seg_off[s + 1] - seg_off[s] < k) return PRUNER_EINVAL;
        const int32_t n_slots = sg[s].n_sp * 4 + sg[s].n_rd * sg[s].rd_levels;
        if (n_slots > tile_rows) return PRUNER_EINVAL;
        const bool frag = sg[s].frag[0] != 0 || sg[s].frag[1] != 0 || sg[s].frag[2] != 0;
        table[s] = LseSeg{seg_off[s], seg_off[s + 1], sg[s].n_sp, sg[s].n_rd, sg[s].rd_levels, n_slots,
                          {frag ? sg[s].frag[0] : 0, frag ? sg[s].frag[1] : 0, frag ? sg[s].frag[2] : 0}, 0};
    }

    int P = 2;
    while (P < 2 * k) P <<= 1;
    int Pn = 2;
    while (Pn < k) Pn <<= 1;
    const size_t merge_lds = (size_t)k * 16 + (size_t)padded(Pn) * 16 + (size_t)k * 4;
    const int dev = current_device(nullptr);
    if (dev < 0) return PRUNER_EHIP;
    if (!g_merge_ready.get(dev)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&lse_merge_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)(PRUNER_MAX_K * 20 + padded(PRUNER_MAX_K) * 16)) != hipSuccess)
            return PRUNER_EHIP;
        g_merge_ready.mark(dev);
    }

    LseSeg* d_table = reinterpret_cast<LseSeg*>(ws + L.table);
    int32_t* best_idx = reinterpret_cast<int32_t*>(ws + L.best_idx);
    float* best_val = reinterpret_cast<float*>(ws + L.best_val);
    int32_t* source = reinterpret_cast<int32_t*>(ws + L.source);
    int32_t* zero_count = reinterpret_cast<int32_t*>(ws + L.zero_count);
    uint64_t* key_hi = reinterpret_cast<uint64_t*>(ws + L.key_hi);
    uint64_t* key_lo = reinterpret_cast<uint64_t*>(ws + L.key_lo);
    uint4* aos = reinterpret_cast<uint4*>(ws + L.aos);
    // S_spec alternates between the caller's arrays and the workspace's, ending in the caller's
    uint16_t* spec_t[2] = {spec_tiles, reinterpret_cast<uint16_t*>(ws + L.alt_tiles)};
    float* spec_s[2] = {spec_score, reinterpret_cast<float*>(ws + L.alt_score)};
    int32_t* spec_n[2] = {spec_count, reinterpret_cast<int32_t*>(ws + L.alt_count)};
    const int64_t spec_pitch = (int64_t)n_sg * k;

    // the table, and the "no S_spec yet" counts of the first step, in one launch
    rc = put_table(d_table, table.data(), table.size() * sizeof(LseSeg), st, zero_count, round_up((size_t)n_sg * sizeof(int32_t), 4));
    if (rc) return rc;

    const size_t filter_bytes = L.table - L.filter;
    auto mutate = [&](int32_t t, const int32_t* count) {   // SchMutation of step t, in place (parents come from S_spec, not from S_x)
        if (tiles_pitch % 4 == 0 && aligned(tiles, 8))
            hipLaunchKernelGGL(lse_mutate_kernel<4>, dim3((unsigned)((n + 1023) / 1024)), dim3(256), 0, st, d_table, n_sg, k, n, tiles, tiles_pitch,
                               aos, count, seed, (uint64_t)t, mutate_q16);
        else
            hipLaunchKernelGGL(lse_mutate_kernel<1>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, d_table, n_sg, k, n, tiles, tiles_pitch,
                               aos, count, seed, (uint64_t)t, mutate_q16);
    };
    // The mutation of step t - 1 is owed when step t begins: the draft kernels of step t make, store and score the
    // children in one pass if their launch shape allows it (large populations), else it runs as a launch of its own
    // first.  Which of the two is decided by the first step's launches (the shape does not change between steps).
    bool fuses = false;
    for (int32_t t = 0; t < n_steps; ++t) {
        const int now = (n_steps - 1 - t) & 1, before = now ^ 1;   // the last step writes the caller's arrays (index 0)
        // C_SA over S_x and its k best: the launches of pruner_prior_filter
        TopkCtx ctx;
        Upload pending;
        rc = topk_prepare(seg_off, n_sg, k, ws + L.filter + draft_bytes, filter_bytes - draft_bytes, st, &ctx, &pending);
        if (rc) return rc;
        const MutArgs owed{d_table, aos, spec_n[before], seed, (uint64_t)(t - 1), mutate_q16, k};
        if (t > 0 && !fuses) {
            mutate(t - 1, spec_n[before]);
            PRUNER_LAUNCH_CHECK();
        }
        bool counted = false, mutated = false;
        rc = draft_launch(sg, n_sg, seg_off, tiles, tiles_pitch, flags, score, nullptr, ws + L.filter, draft_bytes, st,
                          ctx.large ? ctx.d_hist : nullptr, ctx.large ? ctx.d_block_max : nullptr, ctx.copies, &counted, &pending,
                          t > 0 && fuses ? &owed : nullptr, &mutated);
        if (rc) return rc;
        if (t == 0) fuses = ctx.large && counted && draft_launches_by_class(n);
        else if (fuses != mutated) return PRUNER_EHIP;   // (the shape is the same in every step)
        rc = topk_finish(ctx, score, seg_off, best_idx, best_val, ctx.large && counted, st);
        if (rc) return rc;
        // PriorFilter over the union, then the new S_spec's tile factors
        const int32_t* old_n = t == 0 ? zero_count : spec_n[before];
        hipLaunchKernelGGL(lse_keys_kernel, dim3((unsigned)((P + kKeysThreads - 1) / kKeysThreads), (unsigned)n_sg), dim3(kKeysThreads), 0, st, d_table, k, P, tiles, tiles_pitch,
                           best_idx, best_val, spec_t[before], spec_s[before], old_n, spec_pitch, key_hi, key_lo);
        PRUNER_LAUNCH_CHECK();
        hipLaunchKernelGGL(lse_merge_kernel, dim3(n_sg), dim3(kLseThreads), merge_lds, st, k, P, Pn, key_hi, key_lo, best_idx, old_n, spec_s[now],
                           spec_n[now], source);
        PRUNER_LAUNCH_CHECK();
        hipLaunchKernelGGL(lse_copy_kernel, dim3((unsigned)((spec_pitch + 255) / 256)), dim3(256), 0, st, d_table, n_sg, k, tile_rows, tiles,
                           tiles_pitch, spec_t[before], spec_pitch, source, spec_t[now], aos);
        PRUNER_LAUNCH_CHECK();
    }
    // the last step's mutation: S_x as the caller receives it
    mutate(n_steps - 1, spec_n[0]);
    PRUNER_LAUNCH_CHECK();
    return PRUNER_OK;
}
