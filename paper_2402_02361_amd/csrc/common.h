// Internal helpers shared by the entry points of the HIP library (not part of the C boundary).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "pruner.h"

namespace pruner {

constexpr int kWave = 64;  // gfx950 wavefront

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// A launch is refused if the runtime reports an error for it; earlier sticky errors are not cleared here.
#define PRUNER_LAUNCH_CHECK()                      \
    do {                                           \
        if (hipGetLastError() != hipSuccess) return PRUNER_EHIP; \
    } while (0)

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

// workspace needs of the three entry points (each defined next to its kernels)
size_t draft_workspace_bytes(int32_t n_sg);
size_t topk_workspace_bytes(int64_t n, int32_t n_sg, int32_t k);
size_t verify_workspace_bytes(int64_t n_d);

}  // namespace pruner
