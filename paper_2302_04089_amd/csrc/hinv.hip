// Dampened inverse  Hinv = (H + lambda I)^-1  through a Cholesky factorisation (caption of
// Algorithm 1; the paper names neither lambda nor the method, see ziplm.h for the reading).
//
//   A  = H + lambda I, embedded in a dp x dp matrix (dp = d_col rounded up to 128) whose padding is
//        the identity, so that every internal product runs on whole tiles;
//   A  = L L^T     right-looking blocked Cholesky, 64-column panels:
//                  diagonal block factored and inverted in the registers of one wavefront,
//                  panel  L21 = A21 inv(L11)^T  and trailing update  A22 -= L21 L21^T  on the
//                  fp32 matrix cores;
//   T  = L^-1      bottom-up pairwise merges  T21 = -T22 (L21 T11), all pairs of a level in one
//                  batched launch;
//   Hinv = T^T T   lower tiles computed, mirrored to the upper triangle.
#include "common.h"
#include "mfma_gemm.h"

namespace ziplm {

constexpr int NB = 64;  // Cholesky panel width

// lambda = damp_rel * mean(diag H), accumulated in fp64 by one workgroup.
__global__ __launch_bounds__(256) void damp_lambda_kernel(const float *__restrict__ H, int d, float damp_rel,
                                                          double *__restrict__ lambda_out, int *__restrict__ info) {
    __shared__ double part[256];
    double s = 0.0;
    for (int i = threadIdx.x; i < d; i += 256) s += (double)H[(int64_t)i * d + i];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) part[threadIdx.x] += part[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        *lambda_out = (double)damp_rel * (part[0] / (double)d);
        *info = 0;
    }
}

// A (dp x dp) = [H + lambda I, 0; 0, I]
__global__ __launch_bounds__(256) void embed_kernel(const float *__restrict__ H, int d, float *__restrict__ A,
                                                    int dp, const double *__restrict__ lambda) {
    const float lam = (float)(*lambda);
    const int64_t total = (int64_t)dp * dp;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
        const int i = (int)(idx / dp), j = (int)(idx % dp);
        float v;
        if (i < d && j < d) v = H[(int64_t)i * d + j] + (i == j ? lam : 0.f);
        else v = (i == j) ? 1.f : 0.f;
        A[idx] = v;
    }
}

// Factor the 64 x 64 diagonal block at (k0, k0) of A in place (lower triangle) and store the
// inverse of the factor, a dense 64 x 64 lower-triangular matrix, in dinv.
// One wavefront, everything in registers: lane i holds row i of the block (64 VGPRs) and, for the
// inverse, lane c holds column c of T = L^-1.  An entry another lane needs is always "register j
// of lane c" with both known at compile time after full unrolling, i.e. one v_readlane.
//   factorisation, right-looking:  L[i][j] = A[i][j] / l_jj ;  A[i][c] -= L[i][j] L[c][j]  (j < c <= i)
//   inverse, forward substitution: T[i][c] = (delta_ic - sum_{k<i} L[i][k] T[k][c]) / L[i][i]
// A non-positive pivot records 1 + its global column in *info (first one wins) and is replaced by 1
// so that the remaining arithmetic stays finite.
__device__ __forceinline__ float lane_bcast(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

__global__ __launch_bounds__(64) void potrf_diag_kernel(float *__restrict__ A, int ld, int k0,
                                                        float *__restrict__ dinv, int *__restrict__ info) {
    const int lane = threadIdx.x;
    float *Ab = A + (int64_t)k0 * ld + k0;
    float a[NB];
#pragma unroll
    for (int c = 0; c < NB; ++c) a[c] = Ab[(int64_t)lane * ld + c];   // upper entries are never used
    float rdiag[NB];                                                  // 1 / l_jj, uniform
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        float piv = lane_bcast(a[j], j);
        if (!(piv > 0.f)) {                  // uniform
            if (lane == 0 && *info == 0) *info = 1 + k0 + j;
            piv = 1.f;
        }
        const float ljj = sqrtf(piv);
        const float r = 1.0f / ljj;
        rdiag[j] = r;
        a[j] = (lane == j) ? ljj : a[j] * r;              // column j of L (rows above j: unused)
#pragma unroll
        for (int c = j + 1; c < NB; ++c) a[c] -= a[j] * lane_bcast(a[j], c);
    }
    // T = L^-1, lane = column
    float t[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        float s = (lane == i) ? 1.f : 0.f;
#pragma unroll
        for (int k = 0; k < i; ++k) s -= lane_bcast(a[k], i) * t[k];
        t[i] = s * rdiag[i];
    }
#pragma unroll
    for (int c = 0; c < NB; ++c)
        if (c <= lane) Ab[(int64_t)lane * ld + c] = a[c];
#pragma unroll
    for (int i = 0; i < NB; ++i) dinv[i * NB + lane] = t[i];          // t[i] = T[i][lane], zero above the diagonal
}

// T (dp x dp) = block diagonal of the inverted 64 x 64 factors, zero elsewhere.
__global__ __launch_bounds__(256) void place_diag_kernel(float *__restrict__ T, int dp, const float *__restrict__ dinv) {
    const int64_t total = (int64_t)dp * dp;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
        const int i = (int)(idx / dp), j = (int)(idx % dp);
        float v = 0.f;
        if (i / NB == j / NB) v = dinv[(int64_t)(i / NB) * NB * NB + (i % NB) * NB + (j % NB)];
        T[idx] = v;
    }
}

struct HinvLayout {
    int dp;
    float *A, *T, *S, *dinv;
    double *lambda;
    int *info;
    size_t bytes;
};

static HinvLayout hinv_layout(int d_col, void *ws) {
    HinvLayout l;
    l.dp = (d_col + 127) / 128 * 128;
    Carver c(ws);
    const size_t n2 = (size_t)l.dp * l.dp;
    l.A = c.take<float>(n2);
    l.T = c.take<float>(n2);
    l.S = c.take<float>(n2);
    l.dinv = c.take<float>((size_t)(l.dp / NB) * NB * NB);
    l.lambda = c.take<double>(1);
    l.info = c.take<int>(1);
    l.bytes = c.off;
    return l;
}

}  // namespace ziplm

extern "C" size_t ziplm_hinv_workspace_bytes(int d_col) {
    if (d_col <= 0) return 0;
    return ziplm::hinv_layout(d_col, nullptr).bytes;
}

extern "C" int ziplm_hinv(const float *H, float *Hinv, int d_col, float damp_rel, float *lambda_out_host,
                          int *info_host, void *workspace, size_t workspace_bytes, void *stream) {
    using namespace ziplm;
    using namespace ziplm::gemm;
    if (!H || !Hinv || d_col <= 0 || !(damp_rel >= 0.f)) return ZIPLM_ERR_INVALID_ARG;
    const size_t need = ziplm_hinv_workspace_bytes(d_col);
    if (!workspace_ok(workspace, workspace_bytes, need)) return ZIPLM_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const HinvLayout l = hinv_layout(d_col, workspace);
    const int dp = l.dp;
    const int fill_blocks = 1024;

    hipLaunchKernelGGL(damp_lambda_kernel, dim3(1), dim3(256), 0, st, H, d_col, damp_rel, l.lambda, l.info);
    hipLaunchKernelGGL(embed_kernel, dim3(fill_blocks), dim3(256), 0, st, H, d_col, l.A, dp, l.lambda);
    ZIPLM_HIP_TRY(hipGetLastError());

    // ---- A = L L^T, right-looking over 64-column panels --------------------------------------
    for (int k0 = 0; k0 < dp; k0 += NB) {
        float *dinv = l.dinv + (size_t)(k0 / NB) * NB * NB;
        hipLaunchKernelGGL(potrf_diag_kernel, dim3(1), dim3(64), 0, st, l.A, dp, k0, dinv, l.info);
        const int rest = dp - k0 - NB;
        if (rest <= 0) break;
        float *A21 = l.A + (int64_t)(k0 + NB) * dp + k0;
        Args p = {};
        // L21 = A21 inv(L11)^T, in place: the single tile column covers all 64 columns of the panel
        // and a workgroup reads only the rows it later writes, all of them before its epilogue.
        p.A = A21; p.lda = dp;
        p.B = dinv; p.ldb = NB;
        p.C = A21; p.ldc = dp;
        p.M = rest; p.N = NB; p.K = NB;
        p.alpha = 1.f; p.beta = 0.f; p.flags = 0;
        ZIPLM_HIP_TRY((launch<K_CONTIG, K_CONTIG, true, false>(p, 1, st)));
        // A22 -= L21 L21^T, lower tiles only
        Args u = {};
        u.A = A21; u.lda = dp;
        u.B = A21; u.ldb = dp;
        u.C = l.A + (int64_t)(k0 + NB) * dp + (k0 + NB); u.ldc = dp;
        u.M = rest; u.N = rest; u.K = NB;
        u.alpha = -1.f; u.beta = 1.f; u.flags = F_TRI_GRID;
        ZIPLM_HIP_TRY((launch<K_CONTIG, K_CONTIG, true, false>(u, 1, st)));
    }

    // ---- T = L^-1: leaves, then pairwise merges -------------------------------------------------
    hipLaunchKernelGGL(place_diag_kernel, dim3(fill_blocks), dim3(256), 0, st, l.T, dp, l.dinv);
    ZIPLM_HIP_TRY(hipGetLastError());
    for (int s = NB; s < dp; s *= 2) {
        const int nfull = dp / (2 * s);
        const int rem = dp - nfull * 2 * s;
        const int64_t stride = (int64_t)2 * s * (dp + 1);
        for (int pass = 0; pass < 2; ++pass) {
            int a, rs, batch;
            if (pass == 0) { a = 0; rs = s; batch = nfull; }
            else { a = nfull * 2 * s; rs = rem - s; batch = 1; }
            if (batch <= 0 || rs <= 0) continue;
            // S21 = L21 T11      (T11 lower triangular: k starts at the tile column)
            Args m1 = {};
            m1.A = l.A + (int64_t)(a + s) * dp + a; m1.lda = dp;
            m1.B = l.T + (int64_t)a * dp + a; m1.ldb = dp;
            m1.C = l.S + (int64_t)(a + s) * dp + a; m1.ldc = dp;
            m1.M = rs; m1.N = s; m1.K = s;
            m1.alpha = 1.f; m1.beta = 0.f; m1.flags = F_KSTART_N;
            m1.strideA = m1.strideB = m1.strideC = stride;
            ZIPLM_HIP_TRY((launch<K_CONTIG, R_CONTIG, true, false>(m1, batch, st)));
            // T21 = -T22 S21     (T22 lower triangular: k ends with the tile row)
            Args m2 = {};
            m2.A = l.T + (int64_t)(a + s) * dp + (a + s); m2.lda = dp;
            m2.B = l.S + (int64_t)(a + s) * dp + a; m2.ldb = dp;
            m2.C = l.T + (int64_t)(a + s) * dp + a; m2.ldc = dp;
            m2.M = rs; m2.N = s; m2.K = rs;
            m2.alpha = -1.f; m2.beta = 0.f; m2.flags = F_KEND_M;
            m2.strideA = m2.strideB = m2.strideC = stride;
            ZIPLM_HIP_TRY((launch<K_CONTIG, R_CONTIG, true, false>(m2, batch, st)));
        }
    }

    // ---- Hinv = T^T T, lower tiles + mirror, written straight into the caller's d_col x d_col ----
    Args f = {};
    f.A = l.T; f.lda = dp;
    f.B = l.T; f.ldb = dp;
    f.C = Hinv; f.ldc = d_col;
    f.M = d_col; f.N = d_col; f.K = dp;
    f.alpha = 1.f; f.beta = 0.f;
    f.flags = F_TRI_GRID | F_MIRROR | F_KSTART_MAXMN;
    ZIPLM_HIP_TRY((launch<R_CONTIG, R_CONTIG, true, false>(f, 1, st)));

    if (lambda_out_host || info_host) {
        double lam = 0.0;
        int info = 0;
        ZIPLM_HIP_TRY(hipStreamSynchronize(st));
        ZIPLM_HIP_TRY(hipMemcpy(&lam, l.lambda, sizeof(double), hipMemcpyDeviceToHost));
        ZIPLM_HIP_TRY(hipMemcpy(&info, l.info, sizeof(int), hipMemcpyDeviceToHost));
        if (lambda_out_host) *lambda_out_host = (float)lam;
        if (info_host) {
            *info_host = info;
            if (info != 0) return ZIPLM_ERR_NOT_PD;
        }
    }
    return ZIPLM_OK;
}
