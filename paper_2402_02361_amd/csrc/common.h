// Internal helpers shared by the entry points of the HIP library (not part of the C boundary).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "pruner.h"

namespace pruner {

constexpr int kWave = 64;  // gfx950 wavefront

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Inclusive prefix sum over the 64 lanes of a wavefront (every lane active).  Data-parallel-primitive adds: shifts by
// 1, 2, 4 and 8 lanes inside each row of 16 lanes, then lane 15 of rows 0 and 2 into rows 1 and 3, then lane 31 into
// rows 2 and 3; a lane without a source adds 0.  Six full-rate vector instructions where shuffles through LDS
// hardware take six round trips.
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t v)
{
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1, 3
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2, 3
    return v;
}

// Inclusive running maximum over the active lanes of a wavefront, by the same moves: the last active lane ends up
// with the maximum of all active lanes when these are lanes 0..m (a lane without a source, or whose source is switched
// off, keeps its own value).
__device__ __forceinline__ uint32_t wave_inclusive_max(uint32_t v)
{
    auto step = [](uint32_t x, uint32_t y) { return x > y ? x : y; };
    v = step(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x111, 0xf, 0xf, false));
    v = step(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x112, 0xf, 0xf, false));
    v = step(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x114, 0xf, 0xf, false));
    v = step(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x118, 0xf, 0xf, false));
    v = step(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x142, 0xa, 0xf, false));
    v = step(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x143, 0xc, 0xf, false));
    return v;
}

// After a launch: PRUNER_EHIP if the runtime reports an error.  hipGetLastError returns (and clears) the last error
// of the calling thread, so an error left by an earlier, unrelated runtime call is reported here as well; launches that
// came before in the same call stay enqueued.
#define PRUNER_LAUNCH_CHECK()                      \
    do {                                           \
        if (hipGetLastError() != hipSuccess) return PRUNER_EHIP; \
    } while (0)

// Facts about the current device that entry points look up once per device: the number of its compute units, and
// whether a kernel's attribute has been set on it (function attributes belong to the device the call was made on).
// Devices are told apart by their ordinal; the tables hold kMaxDevices of them, later ordinals are looked up every time.
constexpr int kMaxDevices = 64;
int current_device(int* compute_units);   // the ordinal (and the count), or -1 if the runtime reports an error
struct PerDeviceFlag {
    bool set[kMaxDevices] = {};
    bool get(int dev) const { return dev >= 0 && dev < kMaxDevices && set[dev]; }
    void mark(int dev) { if (dev >= 0 && dev < kMaxDevices) set[dev] = true; }
};

// Stream-ordered copy of a small host table into device memory without staging buffers: the bytes travel as
// kernel arguments (copied by the runtime at launch), so the host copy may be freed as soon as the call returns
// and the launch can be captured into a graph.
constexpr int kPutBytes = 3584;
struct PutPayload {
    uint4 q[kPutBytes / 16];
};
// Optionally the same launch clears zero_bytes of device scratch at zero_device.
int put_table(void* dst_device, const void* src_host, size_t bytes, hipStream_t stream, void* zero_device = nullptr,
              size_t zero_bytes = 0);

// A table upload that has been prepared but not launched: a later upload into the same workspace takes it along
// (one launch instead of two).
struct Upload {
    std::vector<char> bytes;
    void* dst = nullptr;
    void* zero = nullptr;
    size_t zero_bytes = 0;
};

// Selection in two steps, so that a caller inside the library can produce the first-digit histograms itself
// between them (the draft kernel does, while the scores are still in registers).
struct TopkCtx {
    bool large;            // segments too long for the one-workgroup route
    int32_t n_sg, k;
    int64_t n, span;
    int32_t blocks;        // workgroups of a sweep launch
    int copies;            // copies of the first digit's histogram
    bool wide;             // set by topk_finish
    void *d_segs, *d_state, *d_stage;
    uint32_t* d_hist;      // [copies][n_sg][2048] first digit, then one copy each for the second and third
    uint32_t* d_block_max; // largest key of every 256 neighbouring entries (block_max_slot), or null: the workspace holds none
    char inline_segs[4096];  // small route: the segment table when it travels as a kernel argument
    bool inline_ok;
};
// validates, uploads the segment table, clears the histograms (large route)
// (defer: do not launch the upload, describe it there instead)
int topk_prepare(const int64_t* seg_off, int32_t n_sg, int32_t k, void* workspace, size_t workspace_bytes, hipStream_t stream, TopkCtx* ctx,
                 Upload* defer = nullptr, bool with_block_max = true);
// the remaining launches; have_first_digit: d_hist already holds the first digit's counts of every segment
int topk_finish(const TopkCtx& ctx, const float* score, const int64_t* seg_off, int32_t* idx_out, float* val_out, bool have_first_digit,
                hipStream_t stream);

// Everything pruner_draft_score refuses, without enqueuing anything.
int draft_check(const pruner_subgraph* sg, int32_t n_sg, const int64_t* seg_off, const uint16_t* tiles, int64_t tiles_pitch, int32_t flags,
                const float* score, const int64_t* symbols, const void* workspace, size_t workspace_bytes);
struct MutArgs;   // lse_child.h
// whether a population of n candidates is scored by one launch per loop-nest class (given the full load width)
bool draft_launches_by_class(int64_t n);
// (also: an upload prepared by someone else whose destination lies in the same allocation shortly after this call's own tables)
// Draft scores; when first_digit is not null and the launch shape allows it (*counted says so), the kernel also adds
// every score's first selection digit to first_digit ([copies][n_sg][2048], cleared by the caller) and, when block_max is
// not null, writes the largest key of every 256 neighbouring candidates of a segment there (block_max_slot).
// mut: the explorer loop's mutation is due on this population; when the launch shape allows it (*mutated says so) the
// kernels make the children from S_spec, store them over `tiles` (which is then written) and score them in one pass;
// otherwise nothing of the kind happens and the caller mutates the population before calling.
int draft_launch(const pruner_subgraph* sg, int32_t n_sg, const int64_t* seg_off, const uint16_t* tiles, int64_t tiles_pitch,
                 int32_t flags, float* score, int64_t* symbols, void* workspace, size_t workspace_bytes, hipStream_t stream,
                 uint32_t* first_digit, uint32_t* block_max, int copies, bool* counted, const Upload* also = nullptr,
                 const MutArgs* mut = nullptr, bool* mutated = nullptr);

// workspace needs of the entry points (each defined next to its kernels)
size_t draft_workspace_bytes(int32_t n_sg);
size_t topk_workspace_bytes(int64_t n, int32_t n_sg, int32_t k);
size_t verify_workspace_bytes(int64_t n_d);
size_t prior_filter_workspace_bytes(int64_t n, int32_t n_sg, int32_t k);
size_t lse_workspace_bytes(int64_t n, int32_t n_sg, int32_t k, int32_t rows);
size_t pacm_workspace_bytes(int64_t n_d);

}  // namespace pruner
