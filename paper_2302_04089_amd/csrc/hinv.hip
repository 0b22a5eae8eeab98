// Dampened inverse  Hinv = (H + lambda I)^-1  through a Cholesky factorisation (caption of
// Algorithm 1; the paper names neither lambda nor the method, see ziplm.h for the reading).
//
//   A  = H + lambda I, embedded in a dp x dp matrix (dp = d_col rounded up to 128) whose padding is
//        the identity, so that every internal product runs on whole tiles;
//   A  = L L^T     right-looking blocked Cholesky, 64-column panels, two launches per panel (every dependent
//                  launch costs far more than the arithmetic of a panel): one that factors the diagonal
//                  block in the registers of a wavefront and solves the panel L21 = A21 L11^-T by
//                  substitution (one thread per row), one for the trailing update A22 -= L21 L21^T on
//                  the fp32 matrix cores;
//   T  = L^-1      diagonal blocks inverted in one batched launch, then bottom-up pairwise merges  T21 = -T22 (L21 T11), all pairs of a level in one
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

// Factor the 64 x 64 diagonal block at (k0, k0) of A in place (lower triangle), one wavefront, the
// block in registers: lane i holds row i (64 VGPRs).  Right-looking:
//     l_jj = sqrt(a_jj);  L[i][j] = A[i][j] / l_jj;  A[i][c] -= L[i][j] L[c][j]   (j < c <= i).
// "Entry j of row c" is register j of lane c, both known at compile time after full unrolling: one
// v_readlane.  A non-positive pivot records 1 + its global column in *info (first one wins) and is
// replaced by 1 so that the remaining arithmetic stays finite.
__device__ __forceinline__ float lane_bcast(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

constexpr int PANEL_ROWS = 128;     // rows of the panel one workgroup solves
constexpr int PANEL_THREADS = 256;

// One launch per 64-column panel: every workgroup factors the diagonal block at (k0, k0) itself (wavefront
// 0, redundantly: it is cheaper than a second dependent launch), while its other wavefronts stage the
// workgroup's 128 rows of the panel below it in LDS with coalesced reads; then one thread per row solves
//     x L11^T = a:   x_j = (a_j - sum_{k<j} x_k L11[j][k]) / L11[j][j]
// with its 64 entries in registers and L11 read from LDS with 128-bit broadcast reads, and the rows go back
// through LDS with coalesced writes.  Workgroup 0 stores the factor L11 to `Ldiag` (a separate 64 x 64
// buffer: the diagonal block in A is still being read by the other workgroups) and reports a non-positive
// pivot in *info (1 + global column of the first one; it is replaced by 1 so that the arithmetic stays finite).
__global__ __launch_bounds__(PANEL_THREADS) void panel_kernel(float *__restrict__ A, int ld, int k0, int rows,
                                                               float *__restrict__ Ldiag, int *__restrict__ info) {
    __shared__ __attribute__((aligned(16))) float Ls[NB][NB];
    __shared__ float rdiag[NB];
    __shared__ float Xs[PANEL_ROWS][NB + 1];       // pitch 65: a thread's row is conflict-free to walk
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row0 = blockIdx.x * PANEL_ROWS;
    float *Xg = A + (int64_t)(k0 + NB + row0) * ld + k0;     // this workgroup's rows of the panel
    if (wave == 0) {
        const float *Ab = A + (int64_t)k0 * ld + k0;
        float a[NB];
#pragma unroll
        for (int c = 0; c < NB; c += 4) {
            const gemm::floatx4 v = *reinterpret_cast<const gemm::floatx4 *>(Ab + (int64_t)lane * ld + c);
            a[c] = v[0]; a[c + 1] = v[1]; a[c + 2] = v[2]; a[c + 3] = v[3];        // upper entries are never used
        }
        int first_bad = -1;                                   // branch-free bookkeeping: one straight-line block
        float my_rdiag = 1.f;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            float piv = lane_bcast(a[j], j);
            const bool bad = !(piv > 0.f);                    // uniform
            first_bad = (bad && first_bad < 0) ? j : first_bad;
            piv = bad ? 1.f : piv;
            const float r = __builtin_amdgcn_rsqf(piv);       // 1 ulp reciprocal square root
            my_rdiag = (lane == j) ? r : my_rdiag;            // 1 / l_jj
            a[j] = a[j] * r;                                  // column j of L; lane j: piv / sqrt(piv) = l_jj
#pragma unroll
            for (int c = j + 1; c < NB; ++c) {
                a[c] -= a[j] * lane_bcast(a[j], c);
                // bound how many broadcast values (scalar registers) are alive at once
                if ((c & 15) == 15) __builtin_amdgcn_sched_barrier(0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int c = 0; c < NB; c += 4) {
            gemm::floatx4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = (c + e <= lane) ? a[c + e] : 0.f;
            *reinterpret_cast<gemm::floatx4 *>(&Ls[lane][c]) = v;
            if (blockIdx.x == 0) *reinterpret_cast<gemm::floatx4 *>(Ldiag + lane * NB + c) = v;
        }
        rdiag[lane] = my_rdiag;
        if (blockIdx.x == 0 && first_bad >= 0 && lane == 0 && *info == 0) *info = 1 + k0 + first_bad;
    } else {
        // 128 rows x 16 pieces of four floats, 16 consecutive lanes per row
        for (int e = tid - 64; e < PANEL_ROWS * (NB / 4); e += PANEL_THREADS - 64) {
            const int r = e >> 4, c4 = e & 15;
            gemm::floatx4 v = {0.f, 0.f, 0.f, 0.f};
            if (row0 + r < rows) v = *reinterpret_cast<const gemm::floatx4 *>(Xg + (int64_t)r * ld + 4 * c4);
#pragma unroll
            for (int q = 0; q < 4; ++q) Xs[r][4 * c4 + q] = v[q];
        }
    }
    __syncthreads();
    if (tid < PANEL_ROWS && row0 + tid < rows) {
        float x[NB];
#pragma unroll
        for (int c = 0; c < NB; ++c) x[c] = Xs[tid][c];
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            float sum = x[j];
#pragma unroll
            for (int k4 = 0; k4 < (j + 3) / 4; ++k4) {
                const gemm::floatx4 l = *reinterpret_cast<const gemm::floatx4 *>(&Ls[j][4 * k4]);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (4 * k4 + e < j) sum -= x[4 * k4 + e] * l[e];
            }
            x[j] = sum * rdiag[j];
        }
#pragma unroll
        for (int c = 0; c < NB; ++c) Xs[tid][c] = x[c];
    }
    __syncthreads();
    for (int e = tid; e < PANEL_ROWS * (NB / 4); e += PANEL_THREADS) {
        const int r = e >> 4, c4 = e & 15;
        if (row0 + r < rows) {
            gemm::floatx4 v;
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = Xs[r][4 * c4 + q];
            *reinterpret_cast<gemm::floatx4 *>(Xg + (int64_t)r * ld + 4 * c4) = v;
        }
    }
}

// Inverses of all factored 64 x 64 diagonal blocks at once (off the factorisation's critical path):
// one wavefront per block, lane i holds row i of L, lane c builds column c of T = L^-1 by forward
// substitution, T[i][c] = (delta_ic - sum_{k<i} L[i][k] T[k][c]) / L[i][i]; "entry k of row i" is
// register k of lane i, one v_readlane.
__global__ __launch_bounds__(64) void trtri_diag_kernel(const float *__restrict__ Ldiag_all, float *__restrict__ dinv_all) {
    const int lane = threadIdx.x;
    const float *Lb = Ldiag_all + (size_t)blockIdx.x * NB * NB;
    float *dinv = dinv_all + (size_t)blockIdx.x * NB * NB;
    float a[NB];
#pragma unroll
    for (int c = 0; c < NB; c += 4) {
        const gemm::floatx4 v = *reinterpret_cast<const gemm::floatx4 *>(Lb + lane * NB + c);
        a[c] = v[0]; a[c + 1] = v[1]; a[c + 2] = v[2]; a[c + 3] = v[3];
    }
    float t[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        float s = (lane == i) ? 1.f : 0.f;
#pragma unroll
        for (int k = 0; k < i; ++k) s -= lane_bcast(a[k], i) * t[k];
        t[i] = s / lane_bcast(a[i], i);
    }
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
    float *A, *T, *S, *dinv, *ldiag;
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
    l.ldiag = c.take<float>((size_t)(l.dp / NB) * NB * NB);   // factored diagonal blocks
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
        const int rest = dp - k0 - NB;
        // diagonal block factored and the panel below it solved, L21 = A21 inv(L11)^T, in one launch
        const int pblocks = rest > 0 ? (rest + PANEL_ROWS - 1) / PANEL_ROWS : 1;
        hipLaunchKernelGGL(panel_kernel, dim3(pblocks), dim3(PANEL_THREADS), 0, st, l.A, dp, k0, rest,
                           l.ldiag + (size_t)(k0 / NB) * NB * NB, l.info);
        if (rest <= 0) break;
        float *A21 = l.A + (int64_t)(k0 + NB) * dp + k0;
        // A22 -= L21 L21^T, lower tiles only
        Args u = {};
        u.A = A21; u.lda = dp;
        u.B = A21; u.ldb = dp;
        u.C = l.A + (int64_t)(k0 + NB) * dp + (k0 + NB); u.ldc = dp;
        u.M = rest; u.N = rest; u.K = NB;
        u.alpha = -1.f; u.beta = 1.f; u.flags = F_TRI_GRID;
        ZIPLM_HIP_TRY((launch<K_CONTIG, K_CONTIG, true, false>(u, 1, st)));
    }

    // ---- T = L^-1: leaves (all diagonal blocks in one launch), then pairwise merges -------------------
    hipLaunchKernelGGL(trtri_diag_kernel, dim3(dp / NB), dim3(64), 0, st, l.ldiag, l.dinv);
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
