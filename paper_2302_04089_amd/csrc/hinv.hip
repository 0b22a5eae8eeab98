// Dampened inverse  Hinv = (H + lambda I)^-1  through a Cholesky factorisation (caption of
// Algorithm 1; the paper names neither lambda nor the method, see ziplm.h for the reading).
//
//   A  = H + lambda I, embedded in a dp x dp matrix (dp = d_col rounded up to 128) whose padding is
//        the identity, so that every internal product runs on whole tiles;
//   A  = L L^T     right-looking blocked Cholesky, 128-column panels, two launches per panel (every dependent
//                  launch costs far more than the arithmetic of a panel): one that factors the diagonal
//                  block (two 64 x 64 factorisations in the registers of a wavefront) and solves the panel
//                  L21 = A21 L11^-T by substitution (one thread per row), one for the trailing update
//                  A22 -= L21 L21^T on the fp32 matrix cores;
//   T  = L^-1      diagonal blocks inverted in one batched launch, then bottom-up pairwise merges  T21 = -T22 (L21 T11), all pairs of a level in one
//                  batched launch;
//   X0 = T^T T     lower tiles computed, mirrored to the upper triangle: the inverse as fp32 arithmetic gives it,
//                  wrong by 1e-5 to 1e-3 relative when H is as ill conditioned as post-GELU inputs make it;
//   Hinv = X0 + X0 R,  R = I - A X0   one Newton step.  R is formed on the fp64 matrix cores (exact products of the
//                  fp32 operands, fp64 sums), the correction X0 R on the fp32 ones (R is small, so its rounding is
//                  second order).  The step squares the error of X0, which leaves the rounding of the fp32
//                  result: the greedy loop's removal order and late-step errors then follow an fp64 inverse.
//                  A second step follows when the residual says that one was not enough; past what the two can
//                  repair the result is refused (poison_on_failure_kernel).
#include "common.h"
#include "mfma_gemm.h"
#include "mfma_dgemm.h"

namespace ziplm {

int device_cu_count();

constexpr int NB = 64;  // Cholesky panel width

// Newton steps enqueued per call (all but the first gated on the device, see poison_on_failure_kernel)
constexpr int kNewtonSteps = 2;

// lambda = damp_rel * mean(diag H), accumulated in fp64 by one workgroup.
__global__ __launch_bounds__(256) void damp_lambda_kernel(const float *__restrict__ H, int d, float damp_rel,
                                                          double *__restrict__ lambda_out, int *__restrict__ info,
                                                          int *__restrict__ counters, int ncounters) {
    // arrival counters of the split products: zero before the first of them (each leaves them zero again)
    for (int i = threadIdx.x; i < ncounters; i += 256) counters[i] = 0;
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
        info[0] = 0;        // 1 + column of the first non-positive pivot, or -1: refinement refused
        info[1] = 0;        // departure counter of the last kernel
        for (int s = 0; s < kNewtonSteps; ++s) info[2 + s] = 0;     // largest |R_ij| of each Newton step's residual, float bits
    }
}

// A (dp x dp) = [H + lambda I, 0; 0, I]; lambda == nullptr: [H, 0; 0, I].  With a gate: only if *gate > gate_above.
__global__ __launch_bounds__(256) void embed_kernel(const float *__restrict__ H, int d, float *__restrict__ A,
                                                    int dp, const double *__restrict__ lambda,
                                                    const unsigned *__restrict__ gate, unsigned gate_above) {
    if (gemm::gate_closed(gate, gate_above)) return;
    const float lam = lambda ? (float)(*lambda) : 0.f;
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

// In-register factorisation of a 64 x 64 block held one row per lane (a[c] = entry c of the lane's row; entries
// above the diagonal are ignored).  Right-looking; see the comment above lane_bcast.  On return a[c], c <= lane,
// is the factor, *my_rdiag = 1 / l_(lane,lane), and *first_bad the first column with a non-positive pivot (or -1;
// such a pivot is replaced by 1 so that the arithmetic stays finite).  Column j of the factor is also written
// to Lt[j][lane] (LDS): the transposed factor, whose row j the substitution below reads contiguously.
// Branch-free on purpose: one straight-line block.  Every lane needs the whole column j of the factor: it is
// written to LDS anyway (the transposed factor) and read back as broadcast 128-bit words, four entries per read;
// only the entry the next pivot waits for (column j + 1) travels through a register broadcast, so that the chain
// pivot -> reciprocal root -> scaled column -> next pivot never waits for LDS.  (Sixty-three register broadcasts
// per column, the earlier form, cost two thirds of the routine's time.)
// Columns J0 .. J1 - 1 of that factorisation; only columns below J1 are updated (the block of columns from J1 on gets
// the whole rank-(J1 - J0) update from the matrix cores afterwards, see potrf64_in_registers).
template <int J0, int J1>
__device__ __forceinline__ void potrf_columns(float (&a)[NB], int lane, float (*Lt)[NB], float &my_rdiag, int &first_bad) {
    gemm::floatx4 lprev[NB / 4], lcur[NB / 4];      // column j - 1 and column j of the factor, as read back from LDS
    float aprev = 0.f;                              // this lane's entry of column j - 1
#pragma unroll
    for (int j = J0; j < J1; ++j) {
        // the chain: pivot, reciprocal root, scaled column, and the one update the next pivot waits for
        float piv = lane_bcast(a[j], j);
        const bool bad = !(piv > 0.f);                    // uniform
        first_bad = (bad && first_bad < 0) ? j : first_bad;
        piv = bad ? 1.f : piv;
        const float r = __builtin_amdgcn_rsqf(piv);       // 1 ulp reciprocal square root
        my_rdiag = (lane == j) ? r : my_rdiag;            // 1 / l_jj
        a[j] = a[j] * r;                                  // column j of L; lane j: piv / sqrt(piv) = l_jj
        Lt[j][lane] = a[j];
        if (j + 1 < J1) a[j + 1] -= a[j] * lane_bcast(a[j], j + 1);
        // column j back from LDS (in flight during the multiply-adds below) ...
#pragma unroll
        for (int c4 = 0; c4 < J1 / 4; ++c4)
            if (4 * c4 + 3 > j + 1) lcur[c4] = *reinterpret_cast<const gemm::floatx4 *>(&Lt[j][4 * c4]);
        __builtin_amdgcn_sched_barrier(0);
        // ... while column j - 1, asked for one step ago, updates the columns from j + 1 on
        if (j > J0) {
#pragma unroll
            for (int c4 = 0; c4 < J1 / 4; ++c4)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (4 * c4 + e > j) a[4 * c4 + e] -= aprev * lprev[c4][e];
        }
        __builtin_amdgcn_sched_barrier(0);
        aprev = a[j];
#pragma unroll
        for (int c4 = 0; c4 < J1 / 4; ++c4) lprev[c4] = lcur[c4];
    }
    // (column J1 - 1 has nothing left to update)
}

// The 64 x 64 factorisation in two halves of 32 columns.  After the first half the rows 32 .. 63 hold L21 in their
// first 32 entries (and Lt[k][32 + r] = L21[r][k] in LDS); their remaining 32 x 32 block takes the whole update
// L21 L21^T from the matrix cores at once -- sixteen instructions instead of a thousand multiply-adds spread over the
// column steps -- and goes back to the rows' registers through the part of Lt that the second half has not written
// yet (skewed by the row, so that neither the scatter nor the gather meets a bank conflict).
constexpr int HB = NB / 2;
// First half: afterwards columns 0 .. 31 of the factor are final for all 64 rows (in a[], in Lt[0 .. 31][*], and
// *my_rdiag for lanes below 32), so whoever solves rows against this block can start on those columns.
__device__ __forceinline__ void potrf64_first_half(float (&a)[NB], int lane, float (*Lt)[NB], float &my_rdiag, int &first_bad) {
    first_bad = -1;
    my_rdiag = 1.f;
    potrf_columns<0, HB>(a, lane, Lt, my_rdiag, first_bad);
    {
        const int r = lane & 31, half = lane >> 5;
        gemm::floatx16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
        // lane l supplies A[row l % 32][k l / 32] and B[k l / 32][col l % 32]: the same entry of L21 for both
#pragma unroll
        for (int kk = 0; kk < HB; kk += 2) {
            const float f = Lt[kk + half][HB + r];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(f, f, acc, 0, 0, 0);
        }
        // accumulator v: row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32
        float *scratch = &Lt[HB][0];              // 32 rows of 64 floats, free until the second half writes them
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = 8 * (v >> 2) + 4 * half + (v & 3);
            scratch[row * NB + ((r + row) & 31)] = acc[v];
        }
        // the same wavefront reads what it wrote: LDS keeps a wavefront's operations in order
        if (lane >= HB) {
#pragma unroll
            for (int c = 0; c < HB; ++c) a[HB + c] -= scratch[r * NB + ((c + r) & 31)];
        }
    }
}
__device__ __forceinline__ void potrf64_second_half(float (&a)[NB], int lane, float (*Lt)[NB], float &my_rdiag, int &first_bad) {
    potrf_columns<HB, NB>(a, lane, Lt, my_rdiag, first_bad);
}

// x L^T = a for one row held in registers, column by column: x_j = a_j / L[j][j], then a_c -= x_j L[c][j] for
// every c > j (independent multiply-adds).  Lt[j][c] = L[c][j] and the reciprocals of the diagonal are in LDS;
// rows of Lt are read with 128-bit broadcast reads, and the whole row j + 1 is asked for before row j is used:
// with one read in flight at a time (what the compiler makes of the plain loop) every read's latency is exposed,
// five hundred times per row.
// Columns J0 .. J1 - 1 of the substitution (every later entry of the row is updated): the two halves of a block run
// one after the other give the same operations in the same order as one pass, and the first can start as soon as the
// first half of the block's factor exists.
template <int J0, int J1>
__device__ __forceinline__ void solve_row_columns(float (&x)[NB], const float (*Lt)[NB], const float *rdiag) {
    gemm::floatx4 lcur[NB / 4], lnext[NB / 4];
    float rcur = rdiag[J0], rnext = 0.f;
#pragma unroll
    for (int c4 = 0; c4 < NB / 4; ++c4)
        if (4 * c4 + 3 > J0) lcur[c4] = *reinterpret_cast<const gemm::floatx4 *>(&Lt[J0][4 * c4]);
#pragma unroll
    for (int j = J0; j < J1; ++j) {
        if (j + 1 < J1) {
            rnext = rdiag[j + 1];
#pragma unroll
            for (int c4 = 0; c4 < NB / 4; ++c4)
                if (4 * c4 + 3 > j + 1) lnext[c4] = *reinterpret_cast<const gemm::floatx4 *>(&Lt[j + 1][4 * c4]);
        }
        const float xj = x[j] * rcur;
        x[j] = xj;
#pragma unroll
        for (int c4 = 0; c4 < NB / 4; ++c4) {
            if (4 * c4 + 3 > j) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (4 * c4 + e > j) x[4 * c4 + e] -= xj * lcur[c4][e];
            }
        }
        rcur = rnext;
#pragma unroll
        for (int c4 = 0; c4 < NB / 4; ++c4) lcur[c4] = lnext[c4];
    }
}

constexpr int PW = 2 * NB;          // panel width: two 64-column blocks per launch
constexpr int PANEL_ROWS = 128;     // rows of the panel one workgroup solves
constexpr int PANEL_THREADS = 256;
constexpr int PITCH_B = NB + 1;     // 64 x 64 blocks that lanes walk by rows
constexpr int PITCH_X = PW + 1;     // the 128 x 128 row tile

struct PanelLds {
    float Lt1[NB][NB];              // transposed factor of the first diagonal block: Lt1[j][c] = L11[c][j], c >= j
    float Lt2[NB][NB];              // the same for the second one
    float Lm[NB][PITCH_B];          // block below L11 inside the diagonal 128 x 128: A21, then L21 = A21 L11^-T
    float D22[NB][PITCH_B];         // second diagonal block: A22, then A22 - L21 L21^T
    float rd1[NB], rd2[NB];         // reciprocals of the diagonals of L11 and L22
    float Xs[PANEL_ROWS][PITCH_X];  // this workgroup's rows of the panel
};

// acc(32 x 32) = Aop[ra + i][0..63] . Bop[rb + j][0..63]^T on the fp32 matrix cores (lane l supplies
// A[row l % 32][k l / 32] and B[k l / 32][col l % 32]), then Dst[rd + i][cd + j] -= acc.  Accumulator register v
// of lane l holds row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32.
__device__ __forceinline__ void tile_downdate(const float *Aop, int pitch_a, int ra, const float *Bop, int pitch_b, int rb,
                                              float *Dst, int pitch_d, int rd, int cd, int lane) {
    const int r = lane & 31, half = lane >> 5;
    gemm::floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    const float *ap = Aop + (ra + r) * pitch_a + half;
    const float *bp = Bop + (rb + r) * pitch_b + half;
#pragma unroll 8
    for (int kk = 0; kk < NB; kk += 2) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(ap[kk], bp[kk], acc, 0, 0, 0);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int row = 8 * (v >> 2) + 4 * half + (v & 3);
        Dst[(rd + row) * pitch_d + cd + r] -= acc[v];
    }
}

// One launch per 128-column panel (two 64-column blocks): on this machine a dependent launch costs more than
// the arithmetic of a panel, so the whole panel step is one kernel.  Every workgroup factors the 128 x 128
// diagonal block at (k0, k0) itself, redundantly -- L11 in the registers of wavefront 0, L21 = A21 L11^-T by
// substitution, A22 - L21 L21^T on the matrix cores, L22 in registers again -- while the other wavefronts
// stage the workgroup's 128 rows of the panel below it in LDS with coalesced reads and solve them against the
// finished parts: x1 = a1 L11^-T (one thread per row, 64 entries in registers), a2 - x1 L21^T (matrix cores),
// x2 = (.) L22^-T.  Rows go back through LDS with coalesced writes.  Workgroup 0 stores the factor of the
// diagonal block to separate buffers (`Ldiag`: L11 and L22, `Loff`: L21; the block in A is still being read by
// the other workgroups) and reports a non-positive pivot in *info (1 + its global column, first one wins).
__global__ __launch_bounds__(PANEL_THREADS) __attribute__((amdgpu_waves_per_eu(1, 1))) void panel_kernel(float *__restrict__ A, int ld, int k0, int rows,
                                                               float *__restrict__ Ldiag, float *__restrict__ Loff,
                                                               int *__restrict__ info) {
    extern __shared__ __attribute__((aligned(16))) unsigned char panel_smem[];
    PanelLds &S = *reinterpret_cast<PanelLds *>(panel_smem);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row0 = blockIdx.x * PANEL_ROWS;
    const float *Ab = A + (int64_t)k0 * ld + k0;                  // the diagonal 128 x 128 block
    float *Xg = A + (int64_t)(k0 + PW + row0) * ld + k0;          // this workgroup's rows of the panel
    int bad1 = -1, bad2 = -1;

    // Every 64-column factorisation runs in two halves with a workgroup barrier between them: once the first 32
    // columns of a block's factor exist, the wavefronts that solve rows against the block start on those columns
    // while wavefront 0 factors the other 32, and only the second half of the substitution is left behind the
    // factorisation (same operations in the same order as one pass: the results do not change).
    float a[NB];            // wavefront 0: the diagonal block being factored, one row per lane
    float x[NB];            // wavefronts 1-3: the row being solved
    float my_rdiag = 1.f;

    // ---- stage 0: first half of L11 || everything else staged in LDS
    if (wave == 0) {
#pragma unroll
        for (int c = 0; c < NB; c += 4) {
            const gemm::floatx4 v = *reinterpret_cast<const gemm::floatx4 *>(Ab + (int64_t)lane * ld + c);
            a[c] = v[0]; a[c + 1] = v[1]; a[c + 2] = v[2]; a[c + 3] = v[3];
        }
        potrf64_first_half(a, lane, S.Lt1, my_rdiag, bad1);
        S.rd1[lane] = my_rdiag;                 // final for lanes below 32
    } else {
        const int t = tid - 64, nt = PANEL_THREADS - 64;
        // A21 and A22 of the diagonal block: 64 rows x 16 pieces of four floats each
        for (int e = t; e < 2 * NB * (NB / 4); e += nt) {
            const int which = e >> 10, r = (e >> 4) & 63, c4 = e & 15;
            const gemm::floatx4 v = *reinterpret_cast<const gemm::floatx4 *>(Ab + (int64_t)(NB + r) * ld + which * NB + 4 * c4);
            float *dst = which ? &S.D22[r][4 * c4] : &S.Lm[r][4 * c4];
#pragma unroll
            for (int q = 0; q < 4; ++q) dst[q] = v[q];
        }
        // the workgroup's rows: 128 rows x 32 pieces, 32 consecutive lanes per row
        for (int e = t; e < PANEL_ROWS * (PW / 4); e += nt) {
            const int r = e >> 5, c4 = e & 31;
            gemm::floatx4 v = {0.f, 0.f, 0.f, 0.f};
            if (row0 + r < rows) v = *reinterpret_cast<const gemm::floatx4 *>(Xg + (int64_t)r * ld + 4 * c4);
#pragma unroll
            for (int q = 0; q < 4; ++q) S.Xs[r][4 * c4 + q] = v[q];
        }
    }
    __syncthreads();

    // ---- stage 1: second half of L11 || against its first 32 columns: the block below it (wavefront 1) and the first
    // half of the workgroup's rows (wavefronts 2, 3)
    float *rowp1 = (wave == 1) ? &S.Lm[lane][0] : &S.Xs[(tid - 128) & (PANEL_ROWS - 1)][0];
    if (wave == 0) {
        potrf64_second_half(a, lane, S.Lt1, my_rdiag, bad1);
        S.rd1[lane] = my_rdiag;
        if (blockIdx.x == 0) {
#pragma unroll
            for (int c = 0; c < NB; c += 4) {
                gemm::floatx4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (c + e <= lane) ? a[c + e] : 0.f;
                *reinterpret_cast<gemm::floatx4 *>(Ldiag + lane * NB + c) = v;
            }
        }
    } else {
#pragma unroll
        for (int c = 0; c < NB; ++c) x[c] = rowp1[c];
        solve_row_columns<0, HB>(x, S.Lt1, S.rd1);
    }
    __syncthreads();

    // ---- stage 2: against the other 32 columns of L11
    if (wave >= 1) {
        solve_row_columns<HB, NB>(x, S.Lt1, S.rd1);
#pragma unroll
        for (int c = 0; c < NB; ++c) rowp1[c] = x[c];
    }
    __syncthreads();

    // ---- matrix cores: D22 -= L21 L21^T (lower 32 x 32 tiles 0-2) and Xs[:, 64:128] -= Xs[:, 0:64] L21^T (tiles 3-10).
    // Only the first three are needed by the factorisation of D22 that follows: they and one more go first, the other
    // seven are done by wavefronts 1-3 while wavefront 0 factors the first half.
    auto downdate_tile = [&](int tile) {
        if (tile < 3) {
            const int ti = (tile == 0) ? 0 : 1, tj = (tile == 2) ? 1 : 0;
            tile_downdate(&S.Lm[0][0], PITCH_B, 32 * ti, &S.Lm[0][0], PITCH_B, 32 * tj, &S.D22[0][0], PITCH_B, 32 * ti, 32 * tj, lane);
        } else {
            const int q = tile - 3, rt = q >> 1, ct = q & 1;
            tile_downdate(&S.Xs[0][0], PITCH_X, 32 * rt, &S.Lm[0][0], PITCH_B, 32 * ct, &S.Xs[0][0], PITCH_X, 32 * rt, NB + 32 * ct, lane);
        }
    };
    downdate_tile(wave);
    __syncthreads();

    // ---- stage 4: first half of L22 || the remaining coupling tiles
    if (wave != 0) {
        for (int tile = 3 + wave; tile < 11; tile += 3) downdate_tile(tile);
    } else {
#pragma unroll
        for (int c = 0; c < NB; ++c) a[c] = S.D22[lane][c];
        potrf64_first_half(a, lane, S.Lt2, my_rdiag, bad2);
        S.rd2[lane] = my_rdiag;
    }
    __syncthreads();

    // ---- stage 5: second half of L22 || the second half of the workgroup's rows against its first 32 columns
    // (wavefronts 2, 3); workgroup 0 meanwhile stores the block below L11
    float *rowp2 = &S.Xs[(tid - 128) & (PANEL_ROWS - 1)][NB];
    if (wave == 0) {
        potrf64_second_half(a, lane, S.Lt2, my_rdiag, bad2);
        S.rd2[lane] = my_rdiag;
        if (blockIdx.x == 0) {
#pragma unroll
            for (int c = 0; c < NB; c += 4) {
                gemm::floatx4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (c + e <= lane) ? a[c + e] : 0.f;
                *reinterpret_cast<gemm::floatx4 *>(Ldiag + NB * NB + lane * NB + c) = v;
            }
        }
        if (blockIdx.x == 0 && lane == 0 && *info == 0) {
            if (bad1 >= 0) *info = 1 + k0 + bad1;
            else if (bad2 >= 0) *info = 1 + k0 + NB + bad2;
        }
    } else if (wave >= 2) {
#pragma unroll
        for (int c = 0; c < NB; ++c) x[c] = rowp2[c];
        solve_row_columns<0, HB>(x, S.Lt2, S.rd2);
    } else if (blockIdx.x == 0) {
        for (int e = lane; e < NB * NB; e += 64) Loff[e] = S.Lm[e >> 6][e & 63];
    }
    __syncthreads();

    // ---- stage 6: against the other 32 columns of L22
    if (wave >= 2) {
        solve_row_columns<HB, NB>(x, S.Lt2, S.rd2);
#pragma unroll
        for (int c = 0; c < NB; ++c) rowp2[c] = x[c];
    }
    __syncthreads();
    for (int e = tid; e < PANEL_ROWS * (PW / 4); e += PANEL_THREADS) {
        const int r = e >> 5, c4 = e & 31;
        if (row0 + r < rows) {
            gemm::floatx4 v;
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = S.Xs[r][4 * c4 + q];
            *reinterpret_cast<gemm::floatx4 *>(Xg + (int64_t)r * ld + 4 * c4) = v;
        }
    }
}

// Trailing update of one panel, A22 -= L21 L21^T on the lower 64 x 64 tiles of the trailing matrix.  The general
// product kernel takes 18 us for a single 128 x 128 tile of this product, whatever else runs: four k slices fetched one
// behind the other, 6.8 us of matrix instructions on one compute unit, a read-modify-write of the tile behind them.
// Here the k range is the panel width and nothing else: a workgroup asks for its two 64 x 128 operand blocks and its
// tile of A22 in one go, and a quarter of the matrix instructions is left per workgroup.
constexpr int UT = 64;                  // tile edge
constexpr int UPITCH = PW + 1;          // operand rows in LDS: lanes walk rows at a fixed k
struct UpdateLds {
    float As[UT][UPITCH];
    float Bs[UT][UPITCH];
};
__global__ __launch_bounds__(256, 2) void trailing_update_kernel(float *__restrict__ A, int ld, int k0) {
    extern __shared__ __attribute__((aligned(16))) unsigned char update_smem[];
    UpdateLds &S = *reinterpret_cast<UpdateLds *>(update_smem);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // neighbouring entries of the tile list share their row block: each XCD takes a contiguous eighth of the list
    const int n = gridDim.x, x = blockIdx.x % 8;
    int ti, tj;
    gemm::tri_decode(x * (n / 8) + min(x, n % 8) + blockIdx.x / 8, ti, tj);
    const float *L = A + (int64_t)(k0 + PW) * ld + k0;                 // L21: rows of the trailing matrix x panel columns
    float *C = A + (int64_t)(k0 + PW + ti * UT) * ld + (k0 + PW + tj * UT);
    // everything this workgroup reads, requested before any of it is used
    gemm::floatx4 ra[UT * PW / 4 / 256], rb[UT * PW / 4 / 256];
#pragma unroll
    for (int q = 0; q < UT * PW / 4 / 256; ++q) {
        const int e = tid + 256 * q, r = e >> 5, c4 = e & 31;            // 32 pieces of four floats per row
        ra[q] = *reinterpret_cast<const gemm::floatx4 *>(L + (int64_t)(ti * UT + r) * ld + 4 * c4);
        rb[q] = *reinterpret_cast<const gemm::floatx4 *>(L + (int64_t)(tj * UT + r) * ld + 4 * c4);
    }
    const int wm = wave >> 1, wn = wave & 1, r32 = lane & 31, half = lane >> 5;
    float cold[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int row = 32 * wm + 8 * (v >> 2) + 4 * half + (v & 3);
        cold[v] = C[(int64_t)row * ld + 32 * wn + r32];
    }
#pragma unroll
    for (int q = 0; q < UT * PW / 4 / 256; ++q) {
        const int e = tid + 256 * q, r = e >> 5, c4 = e & 31;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            S.As[r][4 * c4 + t] = ra[q][t];
            S.Bs[r][4 * c4 + t] = rb[q][t];
        }
    }
    __syncthreads();
    // lane l supplies A[row l % 32][k l / 32] and B[k l / 32][col l % 32]; accumulator v holds row
    // 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32
    gemm::floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    const float *ap = &S.As[32 * wm + r32][half];
    const float *bp = &S.Bs[32 * wn + r32][half];
#pragma unroll 16
    for (int kk = 0; kk < PW; kk += 2) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(ap[kk], bp[kk], acc, 0, 0, 0);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int row = 32 * wm + 8 * (v >> 2) + 4 * half + (v & 3);
        C[(int64_t)row * ld + 32 * wn + r32] = cold[v] - acc[v];
    }
}

// Puts the blocks L21 of all diagonal 128 x 128 blocks (kept aside by panel_kernel) into the factor:
// A[k0 + 64 + r][k0 + c] = Loff[k0 / 128][r][c].
__global__ __launch_bounds__(256) void place_offdiag_kernel(float *__restrict__ A, int ld, const float *__restrict__ Loff) {
    const int k0 = blockIdx.x * PW;
    const float *src = Loff + (size_t)blockIdx.x * NB * NB;
    for (int e = threadIdx.x; e < NB * NB; e += 256) A[(int64_t)(k0 + NB + (e >> 6)) * ld + k0 + (e & 63)] = src[e];
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

// The diagonal 128 x 128 tiles of T: the two inverted 64 x 64 factors on their diagonal, zeros beside them.  Tiles
// below the diagonal are written by the merges; tiles above it are never read (every product that reads T clips its
// k range to the lower triangle at tile granularity).  One workgroup per tile.
__global__ __launch_bounds__(256) void place_diag_kernel(float *__restrict__ T, int dp, const float *__restrict__ dinv) {
    const int t0 = blockIdx.x * PW;
    for (int e = threadIdx.x; e < PW * PW / 4; e += 256) {
        const int i = e / (PW / 4), j = 4 * (e % (PW / 4));
        gemm::floatx4 v = {0.f, 0.f, 0.f, 0.f};
        if (i / NB == j / NB)
            v = *reinterpret_cast<const gemm::floatx4 *>(dinv + (int64_t)((t0 + i) / NB) * NB * NB + (i % NB) * NB + (j % NB));
        *reinterpret_cast<gemm::floatx4 *>(T + (int64_t)(t0 + i) * dp + t0 + j) = v;
    }
}

// A Newton step X <- X + X (I - A X) squares the error of X only while the residual R = I - A X is small, and its own
// fp32 product leaves about 1e-7.  Measured on rank-deficient Hessians (relative error of the result against the fp64
// inverse, by the largest entry of the residual the step started from): 4.6e-5 -> 6e-8, 4.5e-4 -> 1.4e-6,
// 1.2e-3 -> 6e-6, 8e-3 -> 1.3e-4.  So:
//   * a step whose residual stays below kRepeatAbove is the last one (error below 5e-7; conditioning up to about 1e5
//     gets there with the first step);
//   * above it a second step follows, enqueued by the host every time and gated on the device by the residual of the
//     first (a closed gate costs five empty launches, 25 us);
//   * the result is refused when the residual the LAST executed step started from is above kResidualLimit (error up
//     to about 1e-5), NaN included: the matrix is too ill conditioned for the fp32 factorisation to be refined.
//     That is the case from a condition number of a few 1e6 on -- where the rounding of the fp32 Hessian itself
//     (2e-7 per entry) already moves the exact inverse by tens of per cent, so a third step would refine noise.
constexpr float kRepeatAbove = 2.5e-4f;
constexpr float kResidualLimit = 1.5e-3f;
constexpr int kInfoWords = 2 + kNewtonSteps;      // status, departure counter, one residual maximum per step

// A failed factorisation (info != 0) or a refused refinement must not pass for an inverse with callers that never look
// at info: the diagonal of Hinv becomes NaN, which the greedy loop reports as a non-positive pivot at its first step.
__global__ __launch_bounds__(256) void poison_on_failure_kernel(float *__restrict__ Hinv, int d, int *__restrict__ info) {
    // the residual of the last step that ran: step s + 1 ran iff step s left more than kRepeatAbove
    float last = __uint_as_float((unsigned)info[2]);
    for (int s = 1; s < kNewtonSteps && !(last <= kRepeatAbove); ++s) last = __uint_as_float((unsigned)info[2 + s]);
    const bool refused = !(last <= kResidualLimit);
    if (info[0] == 0 && !refused) return;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < d; i += gridDim.x * 256) Hinv[(int64_t)i * d + i] = __builtin_nanf("");
    // every workgroup reads info[0] before any of them may change it: the flag is raised by the last one to leave
    __syncthreads();
    if (threadIdx.x == 0 && info[0] == 0 && atomicAdd(&info[1], 1) == (int)gridDim.x - 1) info[0] = -1;
}

// The large merges of the triangular inverse have 48 to 256 output tiles for 256 compute units (two workgroups fit on each): their k range
// is shared by several workgroups.  Accumulator sets (one per workgroup) the workspace provides for that:
constexpr int MERGE_PARTIAL_SETS = 512;
static int merge_splits(int M, int N, int64_t K, int batch) {
    const int tiles = ((M + gemm::BM - 1) / gemm::BM) * ((N + gemm::BN - 1) / gemm::BN) * batch;
    if (tiles > 256 || K < 512) return 1;
    int n = MERGE_PARTIAL_SETS / tiles;
    if (n > 8) n = 8;
    if (n > K / 128) n = (int)(K / 128);
    return n < 1 ? 1 : n;
}

struct HinvLayout {
    int dp;
    float *A, *T, *S, *dinv, *ldiag, *loff, *partial;
    int *counters;       // one per (batch, tile) of a split product
    int ncounters;
    double *lambda;
    int *info;
    // Newton step: partial sums of the tiles two workgroups share
    int resid_workgroups;
    double *resid_scratch;
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
    // split-K accumulators of the merges; directly behind S, which is free again when the last product runs
    l.partial = c.take<float>((size_t)MERGE_PARTIAL_SETS * 64 * gemm::THREADS);
    l.dinv = c.take<float>((size_t)(l.dp / NB) * NB * NB);
    l.ldiag = c.take<float>((size_t)(l.dp / NB) * NB * NB);   // factored 64 x 64 diagonal blocks
    l.loff = c.take<float>((size_t)(l.dp / PW) * NB * NB);    // the block below the first one in every 128 x 128
    l.lambda = c.take<double>(1);
    {
        const int tm = l.dp / gemm::BM;
        // the lower tiles of a full-size product, the 256 tiles at most of a split merge, the range boundaries of the residual
        l.ncounters = tm * (tm + 1) / 2 + dgemm::RESIDUAL_MAX_WORKGROUPS;
        l.counters = c.take<int>((size_t)l.ncounters);
    }
    l.info = c.take<int>(kInfoWords);
    l.resid_workgroups = dgemm::residual_workgroups(l.dp, 2 * device_cu_count());     // two workgroups fit a compute unit
    if (l.resid_workgroups > dgemm::RESIDUAL_MAX_WORKGROUPS) l.resid_workgroups = dgemm::RESIDUAL_MAX_WORKGROUPS;
    l.resid_scratch = c.take<double>(dgemm::residual_scratch_doubles(l.resid_workgroups));
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

    hipLaunchKernelGGL(damp_lambda_kernel, dim3(1), dim3(256), 0, st, H, d_col, damp_rel, l.lambda, l.info, l.counters, l.ncounters);
    hipLaunchKernelGGL(embed_kernel, dim3(fill_blocks), dim3(256), 0, st, H, d_col, l.A, dp, l.lambda,
                       static_cast<const unsigned *>(nullptr), 0u);
    ZIPLM_HIP_TRY(hipGetLastError());

    // ---- A = L L^T, right-looking over 128-column panels: one panel launch, one trailing update ----
    // every time: the attribute belongs to the current device's copy of the kernel, and the call costs microseconds
    ZIPLM_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(panel_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                      (int)sizeof(PanelLds)));
    ZIPLM_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(trailing_update_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                      (int)sizeof(UpdateLds)));
    for (int k0 = 0; k0 < dp; k0 += PW) {
        const int rest = dp - k0 - PW;
        const int pblocks = rest > 0 ? (rest + PANEL_ROWS - 1) / PANEL_ROWS : 1;
        hipLaunchKernelGGL(panel_kernel, dim3(pblocks), dim3(PANEL_THREADS), sizeof(PanelLds), st, l.A, dp, k0, rest,
                           l.ldiag + (size_t)(k0 / NB) * NB * NB, l.loff + (size_t)(k0 / PW) * NB * NB, l.info);
        ZIPLM_HIP_TRY(hipGetLastError());
        if (rest <= 0) break;
        // A22 -= L21 L21^T, lower 64 x 64 tiles
        const int nt = rest / UT;
        hipLaunchKernelGGL(trailing_update_kernel, dim3(nt * (nt + 1) / 2), dim3(256), sizeof(UpdateLds), st, l.A, dp, k0);
        ZIPLM_HIP_TRY(hipGetLastError());
    }
    hipLaunchKernelGGL(place_offdiag_kernel, dim3(dp / PW), dim3(256), 0, st, l.A, dp, l.loff);

    // ---- T = L^-1: leaves (all diagonal blocks in one launch), then pairwise merges -------------------
    hipLaunchKernelGGL(trtri_diag_kernel, dim3(dp / NB), dim3(64), 0, st, l.ldiag, l.dinv);
    hipLaunchKernelGGL(place_diag_kernel, dim3(dp / PW), dim3(256), 0, st, l.T, dp, l.dinv);
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
            m1.partial = l.partial;
            m1.tile_counters = l.counters;
            ZIPLM_HIP_TRY((launch_splitk<K_CONTIG, R_CONTIG, true, false>(m1, batch, merge_splits(m1.M, m1.N, m1.K, batch), st)));
            // T21 = -T22 S21     (T22 lower triangular: k ends with the tile row)
            Args m2 = {};
            m2.A = l.T + (int64_t)(a + s) * dp + (a + s); m2.lda = dp;
            m2.B = l.S + (int64_t)(a + s) * dp + a; m2.ldb = dp;
            m2.C = l.T + (int64_t)(a + s) * dp + a; m2.ldc = dp;
            m2.M = rs; m2.N = s; m2.K = rs;
            m2.alpha = -1.f; m2.beta = 0.f; m2.flags = F_KEND_M;
            m2.strideA = m2.strideB = m2.strideC = stride;
            m2.partial = l.partial;
            m2.tile_counters = l.counters;
            ZIPLM_HIP_TRY((launch_splitk<K_CONTIG, R_CONTIG, true, false>(m2, batch, merge_splits(m2.M, m2.N, m2.K, batch), st)));
        }
    }

    // ---- X0 = T^T T, lower tiles + mirror, into the buffer of the factor (not needed any more) ----
    Args f = {};
    f.A = l.T; f.lda = dp;
    f.B = l.T; f.ldb = dp;
    f.C = l.A; f.ldc = dp;
    f.M = dp; f.N = dp; f.K = dp;
    f.alpha = 1.f; f.beta = 0.f;
    f.flags = F_TRI_GRID | F_MIRROR | F_KSTART_MAXMN;
    {
        // All tiles fit the chip at once, so the launch lasts as long as its longest tile: the one at (0, 0) runs
        // over the whole k range.  Every tile's k range is shared by up to four workgroups; their accumulators
        // go to S and the merges' buffer behind it (S is free by now).
        const int tm = dp / BM, tiles = tm * (tm + 1) / 2;
        const size_t sets = ((char *)l.partial - (char *)l.S) / (sizeof(float) * 64 * THREADS) + MERGE_PARTIAL_SETS;
        int nsplit = (int)(sets / (size_t)tiles);
        if (nsplit > 4) nsplit = 4;
        if (dp < 1024) nsplit = 1;
        f.partial = l.S;
        f.tile_counters = l.counters;
        ZIPLM_HIP_TRY((launch_splitk<R_CONTIG, R_CONTIG, true, false>(f, 1, nsplit < 1 ? 1 : nsplit, st)));
    }

    // ---- Newton steps: R = I - (H + lambda I) X in fp64 (into T), Hinv = X + X R (lower tiles + mirror) ----
    // H is copied once into a padded matrix (S, free again) so that the residual runs on whole tiles; the padding of H
    // and of X is the identity, so the padded block of R stays apart from the d_col x d_col one.  From here on the
    // caller's H is not read again (Hinv may be the same memory).  The first step starts from X0 in A; a later one
    // (gated: it runs only if the step before left a residual above kRepeatAbove) copies Hinv back into A first.
    // (A caller's H that is a whole number of tiles already, and is not also the output, is read in place.)
    const bool h_in_place = (d_col == dp) && (static_cast<const void *>(H) != static_cast<const void *>(Hinv)) &&
                            (reinterpret_cast<uintptr_t>(H) % 16 == 0);          // 128-bit loads
    if (!h_in_place)
        hipLaunchKernelGGL(embed_kernel, dim3(fill_blocks), dim3(256), 0, st, H, d_col, l.S, dp,
                           static_cast<const double *>(nullptr), static_cast<const unsigned *>(nullptr), 0u);
    for (int step = 0; step < kNewtonSteps; ++step) {
        const unsigned *gate = step ? reinterpret_cast<const unsigned *>(l.info + 2 + step - 1) : nullptr;
        const unsigned above = __builtin_bit_cast(unsigned, kRepeatAbove);
        if (step)
            hipLaunchKernelGGL(embed_kernel, dim3(fill_blocks), dim3(256), 0, st, Hinv, d_col, l.A, dp,
                               static_cast<const double *>(nullptr), gate, above);
        ZIPLM_HIP_TRY(hipGetLastError());
        {
            dgemm::ResidualArgs r = {};
            r.A = h_in_place ? H : l.S; r.lda = dp;
            r.X = l.A; r.ldx = dp;
            r.R = l.T; r.ldr = dp;
            r.lambda = l.lambda;
            r.n = dp;
            r.scratch = l.resid_scratch;
            r.rmax_bits = reinterpret_cast<unsigned *>(l.info + 2 + step);
            r.n_valid = d_col;
            r.gate = gate; r.gate_above = above;
            r.counters = l.counters;
            ZIPLM_HIP_TRY(dgemm::launch_residual(r, l.resid_workgroups, st));
        }
        Args c = {};
        c.A = l.A; c.lda = dp;          // X, rows along k
        c.B = l.T; c.ldb = dp;          // R[k][n]
        c.C = Hinv; c.ldc = d_col;
        c.D = l.A; c.ldd = dp;
        c.M = d_col; c.N = d_col; c.K = dp;
        c.alpha = 1.f; c.beta = 0.f;
        c.flags = F_TRI_GRID | F_MIRROR;
        c.gate = gate; c.gate_above = above;
        // 300 tiles on 512 slots at 3072 columns: the k range of every tile is shared so that the slots fill up.  The
        // accumulators go where the residual kept its partial tiles (done with them); S keeps H for the next step.
        const int tm = (d_col + BM - 1) / BM, tiles = tm * (tm + 1) / 2;
        const size_t sets = dgemm::residual_scratch_doubles(l.resid_workgroups) * sizeof(double) / (sizeof(float) * 64 * THREADS);
        int nsplit = (int)(sets / (size_t)tiles);
        if (nsplit > 3) nsplit = 3;
        if (dp < 1024 || tiles >= 2 * 2 * device_cu_count()) nsplit = 1;
        c.partial = reinterpret_cast<float *>(l.resid_scratch);
        c.tile_counters = l.counters;
        ZIPLM_HIP_TRY((launch_splitk<K_CONTIG, R_CONTIG, true, false>(c, 1, nsplit < 1 ? 1 : nsplit, st)));
    }
    hipLaunchKernelGGL(poison_on_failure_kernel, dim3((d_col + 255) / 256 < 64 ? (d_col + 255) / 256 : 64), dim3(256), 0, st, Hinv, d_col, l.info);
    ZIPLM_HIP_TRY(hipGetLastError());

    if (lambda_out_host || info_host) {
        double lam = 0.0;
        int info = 0;
        ZIPLM_HIP_TRY(hipStreamSynchronize(st));
        ZIPLM_HIP_TRY(hipMemcpy(&lam, l.lambda, sizeof(double), hipMemcpyDeviceToHost));
        ZIPLM_HIP_TRY(hipMemcpy(&info, l.info, sizeof(int), hipMemcpyDeviceToHost));
        if (lambda_out_host) *lambda_out_host = (float)lam;
        if (info_host) {
            *info_host = info;
            if (info > 0) return ZIPLM_ERR_NOT_PD;
            if (info < 0) return ZIPLM_ERR_UNSUPPORTED;       // too ill conditioned for the fp32 factorisation to be refined
        }
    }
    return ZIPLM_OK;
}
