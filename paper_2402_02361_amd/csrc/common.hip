// Pieces used by every entry point: error strings, workspace sizes, small-table upload.
#include "common.h"

#include <string.h>

namespace pruner {

// Block 0 stores the payload; every block clears its 4096-word share of an optional scratch region (counters and
// histograms that must start at zero: a fill kernel, not a memset node, so that captured launches replay correctly).
__global__ void __launch_bounds__(256) put_kernel(uint4* __restrict__ dst, PutPayload payload, int n16, uint32_t* __restrict__ zero,
                                                  int64_t zero_words)
{
    if (blockIdx.x == 0 && (int)threadIdx.x < n16) dst[threadIdx.x] = payload.q[threadIdx.x];
    const int64_t lo = (int64_t)blockIdx.x * 4096;
#pragma unroll 4
    for (int j = 0; j < 16; ++j) {
        const int64_t i = lo + j * 256 + threadIdx.x;
        if (i < zero_words) zero[i] = 0u;
    }
}

int current_device(int* compute_units)
{
    static int cus_of[kMaxDevices];   // 0: not looked up yet
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) return -1;
    int cus = dev < kMaxDevices ? cus_of[dev] : 0;
    if (cus == 0) {
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) return -1;
        if (dev < kMaxDevices) cus_of[dev] = cus;
    }
    if (compute_units) *compute_units = cus;
    return dev;
}

int put_table(void* dst_device, const void* src_host, size_t bytes, hipStream_t stream, void* zero_device, size_t zero_bytes)
{
    // dst is 16-byte aligned and has room for bytes rounded up to 16 (callers size their tables that way);
    // zero_device is 4-byte aligned, zero_bytes a multiple of 4
    const char* src = static_cast<const char*>(src_host);
    char* dst = static_cast<char*>(dst_device);
    const int64_t zero_words = zero_device ? (int64_t)(zero_bytes / 4) : 0;
    bool first = true;
    for (size_t off = 0; off < bytes || first; off += kPutBytes) {
        const size_t left = off < bytes ? bytes - off : 0;
        const size_t chunk = left < (size_t)kPutBytes ? left : (size_t)kPutBytes;
        PutPayload p;
        memset(&p, 0, sizeof p);
        memcpy(&p, src + off, chunk);
        const int n16 = (int)((chunk + 15) / 16);
        const int64_t zw = first ? zero_words : 0;
        const unsigned grid = (unsigned)(zw > 4096 ? (zw + 4095) / 4096 : 1);
        hipLaunchKernelGGL(put_kernel, dim3(grid), dim3(256), 0, stream, reinterpret_cast<uint4*>(dst + off), p, n16,
                           static_cast<uint32_t*>(zero_device), zw);
        PRUNER_LAUNCH_CHECK();
        first = false;
    }
    return PRUNER_OK;
}

}  // namespace pruner

extern "C" const char* pruner_strerror(int code)
{
    switch (code) {
        case PRUNER_OK: return "ok";
        case PRUNER_EINVAL: return "invalid argument";
        case PRUNER_EWORKSPACE: return "workspace missing or too small";
        case PRUNER_ERANGE: return "a symbol of this subgraph can exceed the integer range of the kernels";
        case PRUNER_EHIP: return "the HIP runtime refused a launch";
        default: return "unknown error code";
    }
}

extern "C" size_t pruner_workspace_bytes(int32_t which, int64_t n, int32_t n_sg, int32_t k)
{
    switch (which) {
        case PRUNER_WS_DRAFT: return pruner::draft_workspace_bytes(n_sg);
        case PRUNER_WS_TOPK: return pruner::topk_workspace_bytes(n, n_sg, k);
        case PRUNER_WS_VERIFY: return pruner::verify_workspace_bytes(n);
        case PRUNER_WS_PRIOR_FILTER: return pruner::prior_filter_workspace_bytes(n, n_sg, k);
        case PRUNER_WS_LSE: return pruner::lse_workspace_bytes(n, n_sg, k, PRUNER_MAX_SLOTS);
        case PRUNER_WS_PACM: return pruner::pacm_workspace_bytes(n);
        default: return 0;
    }
}
