// Whole-module error and the prior of the sparsity search.
//
//   ziplm_module_error:  tr(W (H + lambda I) W^T), the layer-wise error (Eq. 1 in the quadratic form of
//       Eq. 2) of dropping every column of the layer at once -- "Pruned structures" in Section 3.1 lists
//       whole attention / feed-forward modules as a structure type -- and the squared denominator of the
//       prior p_s of Section 3.2 ("Structured SPDY search").
//   ziplm_prior:  p_s after each removal of a greedy run, sqrt(running sum of the per-step errors /
//       whole-module error).
//
// The trace is one pass of the fp32 matrix-core product T = W H whose tiles are never stored: each
// workgroup multiplies its tile of T (plus lambda W) element-wise with the same tile of W, sums in fp64 and
// leaves one partial per tile; a single thread then adds the partials in tile order, so the result is
// reproducible from run to run.
#include <atomic>

#include "common.h"
#include "mfma_gemm.h"

namespace ziplm {

// Scratch of ziplm_module_error_static: the per-tile partial sums, for callers that cannot pass a workspace.
// One copy per GPU the library runs on, held until the process ends; 4096 tiles of 128 x 128 cover layers of up
// to 67 million weights (for instance 8192 x 8192).
constexpr int STATIC_SCRATCH_TILES = 4096;
static __device__ __align__(256) double scratch[STATIC_SCRATCH_TILES];

// Device address of `scratch` on the current device.  In host code the array's name is a stand-in for the symbol,
// not an address a kernel could use: the address comes from the runtime, once per device (concurrent first calls
// store the same value), and is what the kernels are given.
static int static_scratch(double **out) {
    constexpr int kMaxDevices = 64;
    static std::atomic<double *> cached[kMaxDevices];
    int dev = 0;
    ZIPLM_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return ZIPLM_ERR_DEVICE;
    double *p = cached[dev].load(std::memory_order_acquire);
    if (!p) {
        void *q = nullptr;
        ZIPLM_HIP_TRY(hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)));
        if (!q) return ZIPLM_ERR_DEVICE;
        p = static_cast<double *>(q);
        cached[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return ZIPLM_OK;
}

static __global__ void sum_partials_kernel(const double *__restrict__ partial, int n, double *__restrict__ out) {
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        double s = 0.0;
        for (int q = 0; q < n; ++q) s += partial[q];
        *out = s;
    }
}

constexpr int PRIOR_THREADS = 1024;

// One workgroup: thread q owns the contiguous chunk [q * chunk, (q + 1) * chunk) of the steps.
static __global__ __launch_bounds__(PRIOR_THREADS) void prior_kernel(const double *__restrict__ err, int n,
                                                                     const double *__restrict__ total,
                                                                     double *__restrict__ prior) {
    __shared__ double chunk_sum[PRIOR_THREADS];
    const int tid = threadIdx.x;
    const int chunk = (n + PRIOR_THREADS - 1) / PRIOR_THREADS;
    const int t0 = tid * chunk, t1 = min(n, t0 + chunk);
    double s = 0.0;
    for (int t = t0; t < t1; ++t) s += err[t];
    chunk_sum[tid] = s;
    __syncthreads();
    if (tid == 0) {          // exclusive prefix over the chunks, in order
        double run = 0.0;
        for (int q = 0; q < PRIOR_THREADS; ++q) {
            const double c = chunk_sum[q];
            chunk_sum[q] = run;
            run += c;
        }
    }
    __syncthreads();
    double run = chunk_sum[tid];
    const double denom = *total;
    // a whole-module error that is not positive and finite makes every prior NaN: the caller sees it at once
    const bool usable = denom > 0.0 && denom < __builtin_inf();
    for (int t = t0; t < t1; ++t) {
        run += err[t];
        prior[t] = usable ? sqrt(run / denom) : __builtin_nan("");
    }
}

static int module_error_tiles(int d_row, int d_col) {
    return ((d_row + gemm::BM - 1) / gemm::BM) * ((d_col + gemm::BN - 1) / gemm::BN);
}

}  // namespace ziplm

extern "C" size_t ziplm_module_error_workspace_bytes(int d_row, int d_col) {
    if (d_row <= 0 || d_col <= 0) return 0;
    return ziplm::align_up(sizeof(double) * (size_t)ziplm::module_error_tiles(d_row, d_col));
}

namespace ziplm {

// The two launches of the whole-module error with the per-tile partial sums in `partials` (one double per tile).
static int launch_module_error(const float *W, const float *H, int d_row, int d_col, float lambda, double *err_out,
                               double *partials, hipStream_t st) {
    // T[i][n] = sum_k W[i][k] H[n][k]  (= (W H)[i][n]: H is symmetric), both operands with k contiguous
    gemm::Args g = {};
    g.A = W; g.B = H; g.C = const_cast<float *>(W);     // the DOT variant only reads C
    g.M = d_row; g.N = d_col; g.K = d_col;
    g.lda = d_col; g.ldb = d_col; g.ldc = d_col;
    g.alpha = 1.f; g.beta = 0.f;
    g.flags = 0;
    g.dot_partial = partials;
    g.dot_lambda = lambda;
    const bool vec = (d_col % 4 == 0) && (reinterpret_cast<uintptr_t>(W) % 16 == 0) &&
                     (reinterpret_cast<uintptr_t>(H) % 16 == 0);
    if (vec) ZIPLM_HIP_TRY((gemm::launch<gemm::K_CONTIG, gemm::K_CONTIG, true, true, true>(g, 1, st)));
    else ZIPLM_HIP_TRY((gemm::launch<gemm::K_CONTIG, gemm::K_CONTIG, false, true, true>(g, 1, st)));
    hipLaunchKernelGGL(sum_partials_kernel, dim3(1), dim3(64), 0, st, static_cast<const double *>(partials),
                       module_error_tiles(d_row, d_col), err_out);
    ZIPLM_HIP_TRY(hipGetLastError());
    return ZIPLM_OK;
}

}  // namespace ziplm

extern "C" int ziplm_module_error(const float *W, const float *H, int d_row, int d_col, float lambda,
                                  double *err_out, void *workspace, size_t workspace_bytes, void *stream) {
    using namespace ziplm;
    if (!W || !H || !err_out || d_row <= 0 || d_col <= 0 || !(lambda >= 0.f)) return ZIPLM_ERR_INVALID_ARG;
    if (!workspace_ok(workspace, workspace_bytes, ziplm_module_error_workspace_bytes(d_row, d_col)))
        return ZIPLM_ERR_WORKSPACE;
    return launch_module_error(W, H, d_row, d_col, lambda, err_out, static_cast<double *>(workspace),
                               static_cast<hipStream_t>(stream));
}

extern "C" int ziplm_module_error_static_max_tiles(void) { return ziplm::STATIC_SCRATCH_TILES; }

extern "C" int ziplm_module_error_static(const float *W, const float *H, int d_row, int d_col, float lambda,
                                         double *err_out, void *stream) {
    using namespace ziplm;
    if (!W || !H || !err_out || d_row <= 0 || d_col <= 0 || !(lambda >= 0.f)) return ZIPLM_ERR_INVALID_ARG;
    if (module_error_tiles(d_row, d_col) > STATIC_SCRATCH_TILES) return ZIPLM_ERR_UNSUPPORTED;     // beyond the built-in scratch
    double *partials = nullptr;
    const int rc = static_scratch(&partials);
    if (rc != ZIPLM_OK) return rc;
    // every partial the second launch reads is written by the first one of this call: nothing to clear
    return launch_module_error(W, H, d_row, d_col, lambda, err_out, partials, static_cast<hipStream_t>(stream));
}

extern "C" int ziplm_prior(const double *err, int n, const double *total, double *prior_out, void *stream) {
    using namespace ziplm;
    if (n < 0 || !total || (n > 0 && (!err || !prior_out))) return ZIPLM_ERR_INVALID_ARG;
    if (n == 0) return ZIPLM_OK;
    hipLaunchKernelGGL(prior_kernel, dim3(1), dim3(PRIOR_THREADS), 0, static_cast<hipStream_t>(stream), err, n, total,
                       prior_out);
    ZIPLM_HIP_TRY(hipGetLastError());
    return ZIPLM_OK;
}
