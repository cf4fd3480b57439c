// The mutation of Alg. 2's SchMutation as a device function, for the kernel that mutates a population in place and for
// the draft kernel that produces and scores the children in one pass.
#pragma once
#include "common.h"

namespace pruner {

struct alignas(8) LseSeg {
    int64_t begin, end;
    int32_t n_sp, n_rd, rd_levels, n_slots;
    int32_t frag[3];     // 0 outside fragment mode
    int32_t pad;
};

// A member of S_spec as one record: its tile factors side by side (32 x uint16 = 64 bytes), so that a parent is read
// with a few 16-byte loads instead of one load per factor.
constexpr int kAosSlots = 32;
static_assert(PRUNER_MAX_SLOTS <= kAosSlots, "a schedule fits one 64-byte record");

// SplitMix64's output function on a state z = seed + c * gamma.
constexpr uint64_t kGamma = 0x9E3779B97F4A7C15ull;
__device__ __forceinline__ uint64_t splitmix64_mix(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
// floor(x * n / 256) for an 8-bit field x and n < 2^16: one full-rate multiply
__device__ __forceinline__ int pick8(uint32_t x, uint32_t n) { return (int)(__umul24(x & 0xFFu, n) >> 8); }

// Whether p divides x, for 0 < p, x < 2^16; q is then x / p.  x * (1/p) in binary32 is off by less than 0.03 from the
// true quotient, so rounding gives the quotient exactly when there is one, and q * p == x holds for no q otherwise.
__device__ __forceinline__ bool divides(uint32_t p, uint32_t x, uint32_t& q)
{
    q = (uint32_t)__builtin_rintf((float)x * __builtin_amdgcn_rcpf((float)p));
    return __umul24(q, p) == x;
}

constexpr int kAosWords = kAosSlots / 2;

// One child of subgraph `sub` (its S_spec holds `count` >= 1 schedules) from the generator state z1 of its first draw
// (the second draw follows it): `packed` receives its tile factors, two per word, as the parent's record holds them.
// The two slots a mutation touches are read from the record directly, and the child differs from the record by XOR
// masks on their two words: no slot is looked up in registers by a computed index.
template <int NP>   // NP: the 16-byte pieces of a record that the subgraph's slots reach; words past them stay 0
__device__ __forceinline__ void lse_child(const LseSeg& seg, int sub, int count, int k, uint64_t z1, const uint4* __restrict__ spec_aos,
                                          uint32_t mutate_q16, uint32_t (&packed)[kAosWords])
{
    const uint64_t u1 = splitmix64_mix(z1);
    const uint4* parent = spec_aos + ((int64_t)sub * k + (int64_t)__umulhi((uint32_t)u1, (uint32_t)count)) * (kAosSlots / 8);
#pragma unroll
    for (int q = 0; q < kAosSlots / 8; ++q) {
        uint4 w4 = make_uint4(0u, 0u, 0u, 0u);
        if (q < NP) w4 = parent[q];
        packed[4 * q] = w4.x, packed[4 * q + 1] = w4.y, packed[4 * q + 2] = w4.z, packed[4 * q + 3] = w4.w;
    }
    int word_src = -1, word_dst = -1;
    uint32_t mask_src = 0, mask_dst = 0;
    if (((uint32_t)(u1 >> 32) & 0xFFFFu) < mutate_q16) {
        const uint32_t u2 = (uint32_t)splitmix64_mix(z1 + kGamma);
        const int n_axes = seg.n_sp + seg.n_rd;
        const int axis = pick8(u2, (uint32_t)n_axes);
        const int levels = axis < seg.n_sp ? 4 : seg.rd_levels;
        const int base = axis < seg.n_sp ? axis * 4 : seg.n_sp * 4 + (axis - seg.n_sp) * seg.rd_levels;
        const int src = pick8(u2 >> 8, (uint32_t)levels);
        int dst = pick8(u2 >> 16, (uint32_t)(levels - 1));
        if (dst >= src) ++dst;
        const uint16_t* slots = reinterpret_cast<const uint16_t*>(parent);
        const uint32_t v = slots[base + src], at_dst_value = slots[base + dst];
        // distinct prime factors of v in ascending order (at most six below 2^16), 16 bits each, the last found lowest
        uint64_t primes_lo = 0;
        uint32_t primes_hi = 0;
        int n_primes = 0;
        uint32_t rest = v;
        if (rest > 1 && (rest & 1u) == 0) {   // the factor 2 by shifts: tile factors are mostly powers of two
            primes_lo = 2, n_primes = 1;
            rest >>= __builtin_ctz(rest);
        }
        for (uint32_t p = 3; p * p <= rest; p += 2) {
            uint32_t q;
            if (divides(p, rest, q)) {
                primes_hi = (primes_hi << 16) | (uint32_t)(primes_lo >> 48), primes_lo = (primes_lo << 16) | p, ++n_primes;
                do rest = q; while (divides(p, rest, q));
            }
        }
        if (rest > 1) primes_hi = (primes_hi << 16) | (uint32_t)(primes_lo >> 48), primes_lo = (primes_lo << 16) | rest, ++n_primes;
        if (n_primes > 0) {
            const int back = n_primes - 1 - pick8(u2 >> 24, (uint32_t)n_primes);   // the draw picks one of them
            const uint32_t p = (back < 4 ? (uint32_t)(primes_lo >> (16 * (back & 3))) : primes_hi >> (16 * (back & 1))) & 0xFFFFu;
            uint32_t smaller = v >> 1;
            if (p != 2) divides(p, v, smaller);
            bool ok = true;
            if (seg.frag[0] > 0 && src == levels - 1) {
                int frag = 0;
                if (axis == seg.n_sp - 2) frag = seg.frag[0];
                if (axis == seg.n_sp - 1) frag = seg.frag[1];
                if (axis == n_axes - 1) frag = seg.frag[2];
                uint32_t q;
                if (frag > 0 && ((frag & (frag - 1)) == 0 ? (smaller & (uint32_t)(frag - 1)) != 0 : frag > 0xFFFF || !divides((uint32_t)frag, smaller, q)))
                    ok = false;
            }
            if (ok) {
                const int at_src = base + src, at_dst = base + dst;
                word_src = at_src >> 1, word_dst = at_dst >> 1;
                mask_src = ((smaller ^ v) & 0xFFFFu) << (16 * (at_src & 1));
                mask_dst = (((at_dst_value * p) ^ at_dst_value) & 0xFFFFu) << (16 * (at_dst & 1));
            }
        }
    }
#pragma unroll
    for (int w = 0; w < 4 * NP; ++w) packed[w] ^= (w == word_src ? mask_src : 0u) ^ (w == word_dst ? mask_dst : 0u);
}

// The generator state of child j's first draw in step `step`: child j draws outputs c + 1 and c + 2, c = step * 2^41 + 2 j.
__device__ __forceinline__ uint64_t lse_child_state(uint64_t seed, uint64_t step, int64_t j) { return seed + ((step << 41) + 2 * (uint64_t)j + 1) * kGamma; }

// What the mutation reads beside the segment table.
struct MutArgs {
    const LseSeg* segs;        // by subgraph
    const uint4* spec_aos;     // S_spec as records, [n_sg * k][kAosSlots / 8]
    const int32_t* spec_count; // members per subgraph
    uint64_t seed, step;
    uint32_t mutate_q16;
    int32_t k;
};

}  // namespace pruner
