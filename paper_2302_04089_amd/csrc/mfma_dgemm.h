// Residual of an approximate inverse on the fp64 matrix cores (gfx950):
//
//   R = I - (A + lambda I) X        A, X symmetric n x n in fp32, n a multiple of 128; R in fp32
//
// Every product a_ik x_kj of two fp32 values is exact in fp64 and the sum over k is accumulated in fp64
// (v_mfma_f64_16x16x4_f64), so R -- whose entries are what is left after the cancellation of O(1) terms -- comes
// out with a relative error of 1e-7 or better even when its entries are 1e-4 or smaller.  That is what one Newton
// step X <- X + X R needs to square the error of an fp32 inverse (caption of Algorithm 1: the method is "given" the
// inverse Hessian; the greedy loop's removal order is sensitive to errors of 1e-6 in it).
//
// One workgroup of 256 threads (four wavefronts, 2 x 2) computes a 128 x 128 tile of R; each wavefront owns 64 x 64
// as 4 x 4 accumulator tiles of 16 x 16.  Operands are staged through LDS in fp32 (half the LDS traffic of fp64
// staging) in slices of 32 values of k with two buffers, exactly like the fp32 product kernel, and converted to
// fp64 in registers.  Matrix-instruction layout (wave64): lane l supplies A[row l % 16][k l / 16] and
// B[k l / 16][col l % 16]; accumulator v of lane l is D[row 4 v + l / 16][col l % 16].  The k index inside a slice is
// permuted identically for both operands (the instruction e of a half slice takes k = e, 4 + e, 8 + e, 12 + e), which
// leaves the contraction unchanged and lets a lane fetch its four values with one 128-bit LDS read.
// By symmetry of X the product (A X)_ij = sum_k A[i][k] X[j][k]: both operands are read along their rows.
#pragma once
#include "mfma_gemm.h"

namespace ziplm {
namespace dgemm {

typedef double doublex4 __attribute__((ext_vector_type(4)));

struct ResidualArgs {
    const float *A;        // n x n, leading dimension lda (without the dampening)
    const float *X;        // n x n, leading dimension ldx
    float *R;              // n x n, leading dimension ldr
    const double *lambda;  // device scalar
    int n;
    int64_t lda, ldx, ldr;
};

__global__ __launch_bounds__(gemm::THREADS, 2) void residual_kernel(ResidualArgs g) {
    using gemm::floatx4;
    __shared__ __attribute__((aligned(16))) float lds[2][2][gemm::SLAB];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int cl16 = lane & 15, q4 = lane >> 4;
    const int tiles_n = g.n / gemm::BN;
    // workgroups go to the eight XCDs round-robin; each XCD takes a contiguous eighth of the row-major tile list,
    // so the tiles in flight on one L2 share their row slabs of A
    const int nt = gridDim.x, x = blockIdx.x % 8;
    const int tile = x * (nt / 8) + min(x, nt % 8) + blockIdx.x / 8;
    const int tm = tile / tiles_n, tn = tile % tiles_n;

    doublex4 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = doublex4{0.0, 0.0, 0.0, 0.0};

    gemm::Slab<gemm::K_CONTIG, true, false> ra, rb;
    const int nslices = g.n / gemm::BK;
    ra.load_inside(g.A, g.lda, tm * gemm::BM, 0, tid);
    rb.load_inside(g.X, g.ldx, tn * gemm::BN, 0, tid);
    ra.store(lds[0][0], tid);
    rb.store(lds[0][1], tid);
    __syncthreads();
    int cur = 0;
    for (int s = 0; s < nslices; ++s) {
        const bool more = s + 1 < nslices;
        if (more) {
            ra.load_inside(g.A, g.lda, tm * gemm::BM, (int64_t)(s + 1) * gemm::BK, tid);
            rb.load_inside(g.X, g.ldx, tn * gemm::BN, (int64_t)(s + 1) * gemm::BK, tid);
        }
        const float *sA = lds[cur][0] + (wm * 64 + cl16) * gemm::PITCH_K + 4 * q4;
        const float *sB = lds[cur][1] + (wn * 64 + cl16) * gemm::PITCH_K + 4 * q4;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            floatx4 a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = *reinterpret_cast<const floatx4 *>(sA + i * 16 * gemm::PITCH_K + 16 * h);
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = *reinterpret_cast<const floatx4 *>(sB + j * 16 * gemm::PITCH_K + 16 * h);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                double ad[4], bd[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) { ad[i] = (double)a[i][e]; bd[i] = (double)b[i][e]; }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(ad[i], bd[j], acc[i][j], 0, 0, 0);
            }
        }
        if (more) {
            ra.store(lds[cur ^ 1][0], tid);
            rb.store(lds[cur ^ 1][1], tid);
        }
        __syncthreads();
        cur ^= 1;
    }

    const double lam = *g.lambda;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = tn * gemm::BN + wn * 64 + j * 16 + cl16;
            float xv[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = tm * gemm::BM + wm * 64 + i * 16 + 4 * v + q4;
                xv[v] = g.X[(int64_t)row * g.ldx + col];
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = tm * gemm::BM + wm * 64 + i * 16 + 4 * v + q4;
                const double r = ((row == col) ? 1.0 : 0.0) - acc[i][j][v] - lam * (double)xv[v];
                g.R[(int64_t)row * g.ldr + col] = (float)r;
            }
        }
}

inline hipError_t launch_residual(const ResidualArgs &g, hipStream_t stream) {
    const int tiles = (g.n / gemm::BM) * (g.n / gemm::BN);
    hipLaunchKernelGGL(residual_kernel, dim3(tiles), dim3(gemm::THREADS), 0, stream, g);
    return hipGetLastError();
}

}  // namespace dgemm
}  // namespace ziplm
