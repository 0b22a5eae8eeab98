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
    // Work sharing.  The (tile, k slice) pairs are numbered tile by tile and dealt out in equal contiguous
    // ranges to the workgroups of the launch, as many workgroups as the device runs at once, so that nobody
    // waits for a second round of tiles (576 tiles on 512 slots would take two rounds for 1.125 rounds of work).
    // A range that starts or ends inside a tile leaves its part of that tile as partial sums in `scratch` (two sets
    // of accumulators per workgroup: [2 w] for the tail of the tile its range starts in, [2 w + 1] for the head of
    // the tile it ends in).  The launch uses at most one workgroup per tile, so a tile is shared by two workgroups
    // at most: the one of the two that finishes second adds head and tail, always in that order, and writes the tile.
    double *scratch;       // [2 * workgroups][64 accumulators][256 threads]
    // Largest |R_ij| over the n_valid x n_valid block that holds the caller's matrix (the rest is padding), as the
    // bit pattern of a non-negative float, raised with an unsigned atomic maximum; NaN counts as infinity.  One
    // Newton step squares the error only while R is small: the caller refuses the result beyond a limit.
    unsigned *rmax_bits;
    int n_valid;
    // optional gate, as in gemm::Args: nothing happens unless *gate > gate_above
    const unsigned *gate;
    unsigned gate_above;
    // one arrival counter per boundary between two ranges, zero before the launch and zero again after it
    int *counters;
};

__device__ __forceinline__ void residual_note_max(float local, unsigned *rmax_bits) {
    // maximum over the wavefront, then one atomic per wavefront
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) local = fmaxf(local, __shfl_xor(local, o));
    if ((threadIdx.x & 63) == 0) atomicMax(rmax_bits, __float_as_uint(local));
}
__device__ __forceinline__ float residual_magnitude(double r) {
    const float a = fabsf((float)r);
    return (a == a) ? a : __builtin_inff();
}

// The range of units of workgroup w out of G.
__device__ __forceinline__ long long residual_range_begin(long long total, int w, int G) { return total * w / G; }

__global__ __launch_bounds__(gemm::THREADS, 2) void residual_kernel(ResidualArgs g) {
    using gemm::floatx4;
    __shared__ __attribute__((aligned(16))) float lds[2][2][gemm::SLAB];
    if (gemm::gate_closed(g.gate, g.gate_above)) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int cl16 = lane & 15, q4 = lane >> 4;
    const int tiles_n = g.n / gemm::BN;
    const int nslices = g.n / gemm::BK;
    // workgroups go to the eight XCDs round-robin; each XCD takes a contiguous eighth of the ranges, so the tiles in
    // flight on one L2 share their row slabs of A
    const int G = gridDim.x, x = blockIdx.x % 8;
    const int w = x * (G / 8) + min(x, G % 8) + blockIdx.x / 8;
    const long long total = (long long)tiles_n * tiles_n * nslices;
    const long long u0 = residual_range_begin(total, w, G), u1 = residual_range_begin(total, w + 1, G);
    const double lam = *g.lambda;

    for (long long u = u0; u < u1;) {
        const int tile = (int)(u / nslices), k0 = (int)(u % nslices);
        const int k1 = (int)min((long long)nslices, k0 + (u1 - u));
        const int tm = tile / tiles_n, tn = tile % tiles_n;
        u += k1 - k0;

        doublex4 acc[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = doublex4{0.0, 0.0, 0.0, 0.0};

        gemm::Slab<gemm::K_CONTIG, true, false> ra, rb;
        __syncthreads();                 // the previous segment's last slice has been read by every wavefront
        ra.load_inside(g.A, g.lda, tm * gemm::BM, (int64_t)k0 * gemm::BK, tid);
        rb.load_inside(g.X, g.ldx, tn * gemm::BN, (int64_t)k0 * gemm::BK, tid);
        ra.store(lds[0][0], tid);
        rb.store(lds[0][1], tid);
        __syncthreads();
        int cur = 0;
        for (int s = k0; s < k1; ++s) {
            const bool more = s + 1 < k1;
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

        if (k0 > 0 || k1 < nslices) {
            // Part of a tile, which this range shares with a neighbour (a tail continues the tile that range w - 1
            // began, a head begins the tile that range w + 1 continues).  The partial sums are written through to memory
            // and the workgroup counts itself at the boundary; of the two, the one that counts second reads both sets
            // back and finishes the tile: head + tail, in that order whoever is second.  One running pointer, advanced
            // behind an opaque step: sixty-four addresses computed ahead of the stores (their offsets exceed what an
            // instruction can encode) would need more registers than are left.
            const bool is_tail = k0 > 0;
            const int boundary = is_tail ? w - 1 : w;
            double *dst = g.scratch + ((size_t)2 * w + (is_tail ? 0 : 1)) * (64 * gemm::THREADS) + tid;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        __hip_atomic_store(dst, acc[i][j][v], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        dst += gemm::THREADS;
                        asm volatile("" : "+v"(dst));
                    }
            __builtin_amdgcn_s_waitcnt(0);          // acknowledged, for every thread, before the workgroup counts itself
            __syncthreads();
            int *ticket = reinterpret_cast<int *>(&lds[0][0][0]);
            if (tid == 0) *ticket = __hip_atomic_fetch_add(g.counters + boundary, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            if (*ticket != 1) continue;             // uniform: the neighbour will finish the tile
            if (tid == 0) __hip_atomic_store(g.counters + boundary, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const double *head = g.scratch + ((size_t)2 * boundary + 1) * (64 * gemm::THREADS) + tid;
            const double *tail = g.scratch + ((size_t)2 * (boundary + 1)) * (64 * gemm::THREADS) + tid;
            float rmax2 = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int col = tn * gemm::BN + wn * 64 + j * 16 + cl16;
                    double sum[4];
                    float xv[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int row = tm * gemm::BM + wm * 64 + i * 16 + 4 * v + q4;
                        sum[v] = __hip_atomic_load(head, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) +
                                 __hip_atomic_load(tail, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        head += gemm::THREADS;
                        tail += gemm::THREADS;
                        asm volatile("" : "+v"(head), "+v"(tail));
                        xv[v] = g.X[(int64_t)row * g.ldx + col];
                    }
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int row = tm * gemm::BM + wm * 64 + i * 16 + 4 * v + q4;
                        const double r = ((row == col) ? 1.0 : 0.0) - sum[v] - lam * (double)xv[v];
                        g.R[(int64_t)row * g.ldr + col] = (float)r;
                        if (row < g.n_valid && col < g.n_valid) rmax2 = fmaxf(rmax2, residual_magnitude(r));
                    }
                }
            residual_note_max(rmax2, g.rmax_bits);
            continue;
        }

        float rmax = 0.f;
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
                    if (row < g.n_valid && col < g.n_valid) rmax = fmaxf(rmax, residual_magnitude(r));
                }
            }
        residual_note_max(rmax, g.rmax_bits);
    }
}

// Workgroups of the first launch: at most one per tile (a tile is then shared by two workgroups at most), at most
// `slots` (what the device runs at once).
inline int residual_workgroups(int n, int slots) {
    const int tiles = (n / gemm::BM) * (n / gemm::BN);
    return tiles < slots ? tiles : slots;
}
constexpr int RESIDUAL_MAX_WORKGROUPS = 1024;
inline size_t residual_scratch_doubles(int workgroups) { return (size_t)2 * workgroups * 64 * gemm::THREADS; }

inline hipError_t launch_residual(const ResidualArgs &g, int workgroups, hipStream_t stream) {
    if (!g.counters) return hipErrorInvalidValue;
    hipLaunchKernelGGL(residual_kernel, dim3(workgroups), dim3(gemm::THREADS), 0, stream, g);
    return hipGetLastError();
}

}  // namespace dgemm
}  // namespace ziplm
