// Version and status strings of the C ABI, and the fill kernel the other translation units share.
#include "common.h"

namespace ziplm {

static __global__ __launch_bounds__(256) void zero_fill_kernel(uint4 *__restrict__ p, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) p[i] = uint4{0u, 0u, 0u, 0u};
}

int zero_fill(void *p, size_t bytes, hipStream_t stream) {
    if (bytes == 0) return ZIPLM_OK;
    if (!p || bytes % 16 || reinterpret_cast<uintptr_t>(p) % 16) return ZIPLM_ERR_INVALID_ARG;
    const size_t n16 = bytes / 16;
    const size_t blocks = (n16 + 255) / 256;
    hipLaunchKernelGGL(zero_fill_kernel, dim3((unsigned)(blocks < 2048 ? blocks : 2048)), dim3(256), 0, stream,
                       static_cast<uint4 *>(p), n16);
    ZIPLM_HIP_TRY(hipGetLastError());
    return ZIPLM_OK;
}

}  // namespace ziplm

extern "C" int ziplm_version(void) { return 100; }

extern "C" const char *ziplm_status_string(int status) {
    switch (status) {
        case ZIPLM_OK: return "ok";
        case ZIPLM_ERR_INVALID_ARG: return "invalid argument";
        case ZIPLM_ERR_NOT_PD: return "matrix not positive definite";
        case ZIPLM_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case ZIPLM_ERR_DEVICE: return "device error";
        case ZIPLM_ERR_UNSUPPORTED: return "unsupported request";
        default: return "unknown status";
    }
}
