// RandomInitSch (Alg. 1: S_draft = S_spec U RandomInitSch(p0); Alg. 2: the initial S_x): a population of schedules
// drawn uniformly from each subgraph's schedule space, written in the layout the other entry points read.
//
// A schedule is one ordered factorisation of every axis extent into the axis's levels, all axes independent; in
// fragment mode the innermost factor of the last two spatial axes and of the last reduction axis is a multiple of
// the fragment size g (factorise extent / g, multiply the innermost factor by g).  The ordered L-factorisations of
// b = p1^e1 p2^e2 ... (primes ascending) are numbered R = r_1 + C_1 (r_2 + C_2 (...)), where r_i is the lexicographic
// rank of the weak composition of e_i into L parts (part l = exponent of p_i in the factor of level l, outermost
// first) and C_i = binom(e_i + L - 1, L - 1).  Candidate c (global index), axis a takes R = floor(u * count / 2^64),
// u = draw number 8 c + a + 1 of SplitMix64 (Steele/Lea/Flood, OOPSLA 2014) started from the seed.
//
// Two launches: ri_table_kernel writes, for every distinct axis space of the call, the table R -> factors (a few
// hundred rows as a rule); ri_fill_kernel gives every candidate one draw, one multiply-high and one 8-byte table
// read per axis, and stores the factors of four neighbouring candidates at a time.  The fill is bound by its stores
// (2 bytes per slot and candidate).
#include "common.h"

#include <string.h>

#include <vector>

namespace pruner {
namespace {

constexpr int kMaxPrimes = 6;    // 2*3*5*7*11*13*17 > 65535
constexpr int kFillThreads = 256;

struct alignas(16) RiSpace {     // one distinct (levels, extent / fragment, fragment)
    uint32_t table_off;          // first row of its table
    uint32_t count;              // rows = ordered factorisations
    int32_t levels, frag, n_primes;
    uint32_t p[kMaxPrimes], e[kMaxPrimes], C[kMaxPrimes];
    uint32_t pad[3];
};
static_assert(sizeof(RiSpace) % 16 == 0, "tables are uploaded 16 bytes at a time");

struct alignas(16) RiAxis {
    uint32_t table_off, count;
    int32_t levels, pad;
};

struct alignas(16) RiSeg {
    int64_t begin, end;
    int32_t n_axes, first_axis, n_slots, pad;
};

constexpr uint64_t kRiGamma = 0x9E3779B97F4A7C15ull;
__device__ __forceinline__ uint64_t ri_splitmix64_mix(uint64_t z)   // SplitMix64's output function on the state seed + c * gamma
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// weak compositions of m into `parts` parts, parts <= 3: binom(m + parts - 1, parts - 1)
__device__ __forceinline__ uint32_t compositions(int m, int parts)
{
    return parts == 1 ? 1u : parts == 2 ? (uint32_t)(m + 1) : (uint32_t)((m + 2) * (m + 1) / 2);
}

// Row R of a space's table: the factors of the R-th ordered factorisation, level 0 in the low half of .x
__global__ void __launch_bounds__(256) ri_table_kernel(const RiSpace* __restrict__ spaces, uint2* __restrict__ table)
{
    const RiSpace sp = spaces[blockIdx.y];
    uint32_t R = blockIdx.x * 256 + threadIdx.x;
    if (R >= sp.count) return;
    const uint32_t row = sp.table_off + R;
    uint32_t f[4] = {1u, 1u, 1u, 1u};
    for (int i = 0; i < sp.n_primes; ++i) {
        uint32_t r = R % sp.C[i];
        R /= sp.C[i];
        // the composition of e into `levels` parts with lexicographic rank r
        int rest = (int)sp.e[i];
        for (int l = 0; l < sp.levels; ++l) {
            int v = rest;   // the last part takes what is left
            if (l < sp.levels - 1) {
                const int after = sp.levels - l - 1;   // parts after this one
                for (v = 0;; ++v) {
                    const uint32_t cnt = compositions(rest - v, after);
                    if (r < cnt) break;
                    r -= cnt;
                }
            }
            for (int j = 0; j < v; ++j) f[l] *= sp.p[i];
            rest -= v;
        }
    }
    f[sp.levels - 1] *= (uint32_t)sp.frag;
    for (int l = sp.levels; l < 4; ++l) f[l] = 0u;
    table[row] = make_uint2(f[0] | (f[1] << 16), f[2] | (f[3] << 16));
}

// VEC neighbouring candidates per thread, stored VEC at a time (the stores are what this kernel costs); blockIdx.y =
// subgraph.  VEC > 1 needs a pitch that is a multiple of VEC and a population aligned to 2 VEC bytes; a thread's
// candidates start at a multiple of VEC, and the threads at a segment's ragged ends store one by one.
template <int VEC>
__global__ void __launch_bounds__(kFillThreads) ri_fill_kernel(const RiSeg* __restrict__ segs, const RiAxis* __restrict__ axes,
                                                               const uint2* __restrict__ table, uint16_t* __restrict__ tiles, int64_t pitch,
                                                               int rows, uint64_t seed)
{
    const RiSeg seg = segs[blockIdx.y];
    const int64_t c0 = seg.begin / VEC * VEC + ((int64_t)blockIdx.x * kFillThreads + threadIdx.x) * VEC;
    if (c0 >= seg.end) return;
    const bool whole = VEC > 1 && c0 >= seg.begin && c0 + VEC <= seg.end;
    // candidate c draws output 8 c + a + 1 of the generator for its axis a: the state advances by additions
    uint64_t z[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) z[e] = seed + (8ull * (uint64_t)(c0 + e) + 1ull) * kRiGamma;
    int slot = 0;
    for (int a = 0; a < seg.n_axes; ++a) {
        const RiAxis ax = axes[seg.first_axis + a];
        uint2 f[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const uint64_t u = ri_splitmix64_mix(z[e]);
            z[e] += kRiGamma;
            f[e] = table[ax.table_off + (uint32_t)__umul64hi(u, (uint64_t)ax.count)];
        }
#pragma unroll
        for (int l = 0; l < 4; ++l) {
            if (l < ax.levels) {
                uint16_t v[VEC];
#pragma unroll
                for (int e = 0; e < VEC; ++e) v[e] = (uint16_t)((l < 2 ? f[e].x : f[e].y) >> (16 * (l & 1)));
                uint16_t* at = tiles + (int64_t)(slot + l) * pitch + c0;
                if (whole) {
                    uint64_t w = 0;
#pragma unroll
                    for (int e = 0; e < VEC; ++e) w |= (uint64_t)v[e] << (16 * e);
                    if constexpr (VEC == 4) *reinterpret_cast<uint64_t*>(at) = w;
                    else if constexpr (VEC == 2) *reinterpret_cast<uint32_t*>(at) = (uint32_t)w;
                } else {
#pragma unroll
                    for (int e = 0; e < VEC; ++e)
                        if (c0 + e >= seg.begin && c0 + e < seg.end) at[e] = v[e];
                }
            }
        }
        slot += ax.levels;
    }
    for (; slot < rows; ++slot) {   // rows the subgraph does not own
        uint16_t* at = tiles + (int64_t)slot * pitch + c0;
        if (whole) {
            if constexpr (VEC == 4) *reinterpret_cast<uint64_t*>(at) = 0ull;
            else if constexpr (VEC == 2) *reinterpret_cast<uint32_t*>(at) = 0u;
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e)
                if (c0 + e >= seg.begin && c0 + e < seg.end) at[e] = 0;
        }
    }
}

struct Plan {
    std::vector<RiSpace> spaces;
    std::vector<RiAxis> axes;
    std::vector<RiSeg> segs;
    uint64_t table_rows = 0;
    int32_t max_slots = 0;
    uint32_t max_count = 0;
};

int fragment_of(const pruner_subgraph& g, int axis)
{
    if (g.frag[0] == 0 && g.frag[1] == 0 && g.frag[2] == 0) return 1;
    if (axis == g.n_sp - 2) return g.frag[0];
    if (axis == g.n_sp - 1) return g.frag[1];
    if (axis == g.n_sp + g.n_rd - 1) return g.frag[2];
    return 1;
}

uint64_t binom(int n, int k)
{
    uint64_t r = 1;
    for (int i = 1; i <= k; ++i) r = r * (uint64_t)(n - k + i) / (uint64_t)i;
    return r;
}

// the spaces (distinct ones once), per-axis and per-subgraph tables of a call; seg_off may be null (sizes only)
int make_plan(const pruner_subgraph* sg, int32_t n_sg, const int64_t* seg_off, Plan* plan)
{
    for (int32_t s = 0; s < n_sg; ++s) {
        const pruner_subgraph& g = sg[s];
        if (g.n_sp < 1 || g.n_sp > PRUNER_MAX_SP || g.n_rd < 0 || g.n_rd > PRUNER_MAX_RD || g.sp_levels != 4 ||
            (g.n_rd > 0 && g.rd_levels != 2 && g.rd_levels != 3))
            return PRUNER_EINVAL;
        const bool fragments = g.frag[0] != 0 || g.frag[1] != 0 || g.frag[2] != 0;
        if (fragments && (g.n_sp < 2 || g.n_rd < 1 || g.frag[0] < 1 || g.frag[1] < 1 || g.frag[2] < 1)) return PRUNER_EINVAL;
        const int n_axes = g.n_sp + g.n_rd;
        RiSeg seg;
        memset(&seg, 0, sizeof seg);
        seg.begin = seg_off ? seg_off[s] : 0;
        seg.end = seg_off ? seg_off[s + 1] : 0;
        seg.n_axes = n_axes;
        seg.first_axis = (int32_t)plan->axes.size();
        seg.n_slots = g.n_sp * 4 + g.n_rd * g.rd_levels;
        if (seg.n_slots > plan->max_slots) plan->max_slots = seg.n_slots;
        for (int a = 0; a < n_axes; ++a) {
            const int levels = a < g.n_sp ? 4 : g.rd_levels;
            const int frag = fragment_of(g, a);
            if (g.extent[a] < 1 || g.extent[a] > 65535 || g.extent[a] % frag != 0) return PRUNER_EINVAL;
            RiSpace sp;
            memset(&sp, 0, sizeof sp);
            sp.levels = levels;
            sp.frag = frag;
            uint32_t rest = (uint32_t)(g.extent[a] / frag);
            uint64_t count = 1;
            for (uint32_t p = 2; rest > 1; ++p) {
                if (p * p > rest) p = rest;   // what is left is prime
                uint32_t e = 0;
                while (rest % p == 0) rest /= p, ++e;
                if (!e) continue;
                sp.p[sp.n_primes] = p;
                sp.e[sp.n_primes] = e;
                sp.C[sp.n_primes] = (uint32_t)binom((int)e + levels - 1, levels - 1);
                count *= sp.C[sp.n_primes];
                ++sp.n_primes;
            }
            sp.count = (uint32_t)count;   // at most a few ten thousand for extents below 65536
            // an equal space met before shares its table
            size_t hit = plan->spaces.size();
            for (size_t i = 0; i < plan->spaces.size(); ++i) {
                const RiSpace& o = plan->spaces[i];
                if (o.levels == sp.levels && o.frag == sp.frag && o.n_primes == sp.n_primes && memcmp(o.p, sp.p, sizeof sp.p) == 0 &&
                    memcmp(o.e, sp.e, sizeof sp.e) == 0) {
                    hit = i;
                    break;
                }
            }
            if (hit == plan->spaces.size()) {
                sp.table_off = (uint32_t)plan->table_rows;
                plan->table_rows += sp.count;
                if (plan->table_rows > 0x7FFFFFFFull) return PRUNER_ERANGE;
                if (sp.count > plan->max_count) plan->max_count = sp.count;
                plan->spaces.push_back(sp);
            }
            plan->axes.push_back(RiAxis{plan->spaces[hit].table_off, plan->spaces[hit].count, levels, 0});
        }
        plan->segs.push_back(seg);
    }
    if (plan->spaces.size() > 65535) return PRUNER_ERANGE;   // one grid row per space
    return PRUNER_OK;
}

struct Layout {
    size_t spaces, axes, segs, table, total;
};

Layout layout(const Plan& plan)
{
    Layout L;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += round_up(bytes, 256);
        return at;
    };
    L.spaces = take(plan.spaces.size() * sizeof(RiSpace));
    L.axes = take(plan.axes.size() * sizeof(RiAxis));
    L.segs = take(plan.segs.size() * sizeof(RiSeg));
    L.table = take((size_t)plan.table_rows * sizeof(uint2));
    L.total = off;
    return L;
}

}  // namespace
}  // namespace pruner

using namespace pruner;

extern "C" size_t pruner_random_init_workspace_bytes(const pruner_subgraph* sg, int32_t n_sg)
{
    if (!sg || n_sg < 1 || n_sg > PRUNER_MAX_SUBGRAPHS) return 0;
    Plan plan;
    if (make_plan(sg, n_sg, nullptr, &plan) != PRUNER_OK) return 0;
    return layout(plan).total;
}

extern "C" int pruner_random_init(const pruner_subgraph* sg, int32_t n_sg, const int64_t* seg_off, uint16_t* tiles, int64_t tiles_pitch,
                                  int32_t tile_rows, uint64_t seed, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!sg || !seg_off || n_sg < 1 || n_sg > PRUNER_MAX_SUBGRAPHS) return PRUNER_EINVAL;
    if (seg_off[0] != 0) return PRUNER_EINVAL;
    for (int32_t s = 0; s < n_sg; ++s)
        if (seg_off[s + 1] < seg_off[s]) return PRUNER_EINVAL;
    const int64_t n = seg_off[n_sg];
    if (n > 0x7FFFFFFFll || tile_rows < 1 || tile_rows > PRUNER_MAX_SLOTS) return PRUNER_EINVAL;
    Plan plan;
    int rc = make_plan(sg, n_sg, seg_off, &plan);
    if (rc) return rc;
    if (plan.max_slots > tile_rows) return PRUNER_EINVAL;
    if (n == 0) return PRUNER_OK;
    if (!tiles || !aligned(tiles, 2) || tiles_pitch < n) return PRUNER_EINVAL;
    if (!workspace || !aligned(workspace, 256)) return PRUNER_EWORKSPACE;
    const Layout L = layout(plan);
    if (workspace_bytes < L.total) return PRUNER_EWORKSPACE;

    hipStream_t st = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    rc = put_table(ws + L.spaces, plan.spaces.data(), plan.spaces.size() * sizeof(RiSpace), st);
    if (rc) return rc;
    rc = put_table(ws + L.axes, plan.axes.data(), plan.axes.size() * sizeof(RiAxis), st);
    if (rc) return rc;
    rc = put_table(ws + L.segs, plan.segs.data(), plan.segs.size() * sizeof(RiSeg), st);
    if (rc) return rc;
    uint2* table = reinterpret_cast<uint2*>(ws + L.table);
    hipLaunchKernelGGL(ri_table_kernel, dim3((plan.max_count + 255) / 256, (unsigned)plan.spaces.size()), dim3(256), 0, st,
                       reinterpret_cast<const RiSpace*>(ws + L.spaces), table);
    PRUNER_LAUNCH_CHECK();
    int64_t longest = 0;
    for (int32_t s = 0; s < n_sg; ++s)
        if (seg_off[s + 1] - seg_off[s] > longest) longest = seg_off[s + 1] - seg_off[s];
    // (a segment that does not begin at a multiple of the vector width needs one thread more)
    if (tiles_pitch % 4 == 0 && aligned(tiles, 8))
        hipLaunchKernelGGL(ri_fill_kernel<4>, dim3((unsigned)((longest + 4 + 4 * kFillThreads - 1) / (4 * kFillThreads)), (unsigned)n_sg),
                           dim3(kFillThreads), 0, st, reinterpret_cast<const RiSeg*>(ws + L.segs), reinterpret_cast<const RiAxis*>(ws + L.axes), table,
                           tiles, tiles_pitch, (int)tile_rows, seed);
    else
        hipLaunchKernelGGL(ri_fill_kernel<1>, dim3((unsigned)((longest + kFillThreads - 1) / kFillThreads), (unsigned)n_sg), dim3(kFillThreads), 0, st,
                           reinterpret_cast<const RiSeg*>(ws + L.segs), reinterpret_cast<const RiAxis*>(ws + L.axes), table, tiles, tiles_pitch,
                           (int)tile_rows, seed);
    PRUNER_LAUNCH_CHECK();
    return PRUNER_OK;
}
