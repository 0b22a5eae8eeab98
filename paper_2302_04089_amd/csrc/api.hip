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

// Ping-pong of one tagged 64-bit word between workgroup 0 and workgroup `partner` of a small cooperative launch:
// device-scope store, device-scope polling load, the two operations every step of the greedy loop waits on.
// Every wait is bounded (0.5 s); on a time-out out[1] is set and both sides leave.
static __global__ __launch_bounds__(64) void handoff_kernel(unsigned long long *words, int partner, int rounds,
                                                            unsigned long long *out) {
    if (threadIdx.x != 0) return;
    const int b = blockIdx.x;
    unsigned long long *ping = words, *pong = words + 32;          // 256 bytes apart
    const unsigned long long limit = 50000000ull;
    if (b == 0) {
        const unsigned long long t0 = wall_clock64();
        for (int i = 1; i <= rounds; ++i) {
            __hip_atomic_store(ping, (unsigned long long)i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const unsigned long long s = wall_clock64();
            while (__hip_atomic_load(pong, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != (unsigned long long)i)
                if (wall_clock64() - s > limit) { out[1] = 1; return; }
        }
        out[0] = wall_clock64() - t0;
    } else if (b == partner) {
        for (int i = 1; i <= rounds; ++i) {
            const unsigned long long s = wall_clock64();
            while (__hip_atomic_load(ping, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != (unsigned long long)i)
                if (wall_clock64() - s > limit) { out[1] = 2; return; }
            __hip_atomic_store(pong, (unsigned long long)i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

}  // namespace ziplm

extern "C" int ziplm_selftest_handoff_latency(int rounds, int partner, double *us_out_host, void *workspace,
                                              size_t workspace_bytes, void *stream) {
    using namespace ziplm;
    constexpr int kWorkgroups = 16;              // workgroup i lands on XCD i % 8
    if (rounds < 1 || rounds > 1000000 || partner < 1 || partner >= kWorkgroups || !us_out_host) return ZIPLM_ERR_INVALID_ARG;
    if (!workspace_ok(workspace, workspace_bytes, 1024)) return ZIPLM_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (zero_fill(workspace, 1024, st) != ZIPLM_OK) return ZIPLM_ERR_DEVICE;
    unsigned long long *words = static_cast<unsigned long long *>(workspace);
    unsigned long long *out = words + 96;
    void *args[] = {&words, &partner, &rounds, &out};
    ZIPLM_HIP_TRY(hipLaunchCooperativeKernel(reinterpret_cast<void *>(handoff_kernel), dim3(kWorkgroups), dim3(64), args, 0, st));
    unsigned long long h[2] = {0, 0};
    ZIPLM_HIP_TRY(hipStreamSynchronize(st));
    ZIPLM_HIP_TRY(hipMemcpy(h, out, sizeof(h), hipMemcpyDeviceToHost));
    if (h[1] != 0) return ZIPLM_ERR_DEVICE;
    *us_out_host = (double)h[0] / 100.0 / (2.0 * rounds);       // 100 MHz clock; two hand-offs per round
    return ZIPLM_OK;
}

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
