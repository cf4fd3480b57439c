// Pieces used by every entry point: error strings, workspace sizes, small-table upload.
#include "common.h"

#include <string.h>

namespace pruner {

__global__ void __launch_bounds__(256) put_kernel(uint4* __restrict__ dst, PutPayload payload, int n16)
{
    const int i = threadIdx.x;
    if (i < n16) dst[i] = payload.q[i];
}

int put_table(void* dst_device, const void* src_host, size_t bytes, hipStream_t stream)
{
    // dst is 16-byte aligned and has room for bytes rounded up to 16 (callers size their tables that way)
    const char* src = static_cast<const char*>(src_host);
    char* dst = static_cast<char*>(dst_device);
    for (size_t off = 0; off < bytes; off += kPutBytes) {
        const size_t chunk = bytes - off < (size_t)kPutBytes ? bytes - off : (size_t)kPutBytes;
        PutPayload p;
        memset(&p, 0, sizeof p);
        memcpy(&p, src + off, chunk);
        const int n16 = (int)((chunk + 15) / 16);
        hipLaunchKernelGGL(put_kernel, dim3(1), dim3(256), 0, stream, reinterpret_cast<uint4*>(dst + off), p, n16);
        PRUNER_LAUNCH_CHECK();
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
        default: return 0;
    }
}
