// fp32 matrix-core GEMM building block for gfx950 (CDNA4), used by the Hessian accumulation and by
// the blocked Cholesky / triangular inverse.
//
//   C[M x N] = alpha * opA(A) * opB(B) + beta * C
//
// One workgroup of 256 threads (4 wavefronts of 64 lanes, arranged 2 x 2) computes a 128 x 128 tile
// of C; each wavefront owns a 64 x 64 sub-tile as 2 x 2 accumulators of v_mfma_f32_32x32x2_f32.
// The K loop advances in slices of 32, staged through LDS with two buffers so that the global loads
// of slice k+1 overlap the matrix instructions of slice k (one barrier per slice).
//
// Operand storage ("mode") is described from the point of view of the tile an operand contributes,
// a (128 rows) x (32 k) slab whose rows are the M index for A and the N index for B:
//   K_CONTIG : element (r, k) at base[r * ld + k]   (row-major operand, k fastest)
//   R_CONTIG : element (r, k) at base[k * ld + r]   (the operand's transpose is row-major)
// so  NT = (A K_CONTIG, B K_CONTIG)  computes A B^T for row-major A [M][K], B [N][K];
//     NN = (A K_CONTIG, B R_CONTIG)  computes A B   for row-major B [K][N];
//     TN = (A R_CONTIG, B R_CONTIG)  computes A^T B for row-major A [K][M], B [K][N].
//
// Matrix-instruction operand layout (32x32x2, wave64): lane l supplies A[row = l % 32][k = l / 32] and
// B[k = l / 32][col = l % 32]; accumulator register v of lane l holds
// C[row = 8 * (v / 4) + 4 * (l / 32) + (v % 4)][col = l % 32].
// The k index inside a slice is permuted identically for A and B (lanes 0-31 take k = 8j..8j+3,
// lanes 32-63 take k = 8j+4..8j+7, over four consecutive instructions), which leaves the
// contraction unchanged and lets a K_CONTIG operand be fetched with one 128-bit LDS read.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ziplm {
namespace gemm {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128;      // tile rows
constexpr int BN = 128;      // tile cols
constexpr int BK = 32;       // k slice
constexpr int THREADS = 256;
constexpr int PITCH_K = 36;  // floats per row of a K_CONTIG slab in LDS ([128][36]); 36 = 4 (mod 32)
constexpr int PITCH_R = 128; // floats per k-row of an R_CONTIG slab in LDS ([32][128])
constexpr int SLAB = BM * PITCH_K;  // floats reserved per operand per buffer (>= 32 * 128)

enum Mode { K_CONTIG = 0, R_CONTIG = 1 };

enum Flags : unsigned {
    F_LOWER_ONLY = 1u,     // compute only tiles with tile_col <= tile_row (square output)
    F_MIRROR = 2u,         // also write the transpose of every strictly-lower tile (symmetric output)
    F_KSTART_N = 4u,       // k starts at tile_col * 128 (B is lower triangular: B(k, n) = 0 for k < n)
    F_KSTART_MAXMN = 8u,   // k starts at max(tile_row, tile_col) * 128 (T^T T with T lower triangular)
    F_KEND_M = 16u,        // k ends at (tile_row + 1) * 128 (A is lower triangular: A(m, k) = 0 for k > m)
    F_TRI_GRID = 32u,      // blockIdx.x enumerates the lower-triangular tile list instead of a 2-D grid
    F_PARTIAL = 64u,       // split-K: write raw accumulators to `partial`, no epilogue
    F_SPLIT_TILE_RANGE = 128u,   // with F_PARTIAL: the splits share each tile's own k range (after the flags above)
};
// The DOT variant of the kernel writes no output matrix: it sums (alpha * acc + dot_lambda * C) * C over the tile,
// C read-only, in fp64, into dot_partial[tile].

struct Args {
    const float *A;
    const float *B;
    float *C;
    int M, N;
    int64_t K;
    int64_t lda, ldb, ldc;
    float alpha, beta;
    unsigned flags;
    // batching (blockIdx.z) -- element offsets added per batch index
    int64_t strideA, strideB, strideC;
    // split-K (blockIdx.y when F_PARTIAL): k range of split s is [s * k_chunk, min(K, (s+1) * k_chunk))
    int64_t k_chunk;
    float *partial;   // [split][tile][64 regs][256 threads]
    int tiles_n;      // number of tile columns (2-D grid decoding)
    // DOT variant
    double *dot_partial;   // [tiles]
    float dot_lambda;
    // optional addend: with D set the result is alpha * acc + D (beta and the old C are ignored); with F_MIRROR the
    // transposed element receives the same value (tiles on the diagonal mirror their lower half), so C is exactly
    // symmetric.  Not batched.
    const float *D;
    int64_t ldd;
    // optional gate: with gate set, the launch does nothing unless *gate > gate_above (a word written by an earlier
    // kernel on the stream), so that the host can enqueue work whose need only the device knows
    const unsigned *gate;
    unsigned gate_above;
    // FUSED split-K: one arrival counter per (batch, tile), zero before the launch and zero again after it
    int *tile_counters;
};

__device__ __forceinline__ bool gate_closed(const unsigned *gate, unsigned above) {
    return gate && __builtin_nontemporal_load(gate) <= above;
}

// ---------------------------------------------------------------------------------------------
// Global -> register -> LDS staging of one 128 x 32 slab.
// ---------------------------------------------------------------------------------------------
template <int MODE, bool VEC, bool KGUARD>
struct Slab {
    floatx4 r[4];

    __device__ __forceinline__ void load(const float *__restrict__ base, int64_t ld, int row0,
                                         int rows, int64_t k0, int64_t kend, int tid) {
        if (MODE == K_CONTIG) {
            const int c4 = tid & 7;         // which group of 4 k
            const int rr = tid >> 3;        // 0..31
            const int64_t k = k0 + 4 * c4;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int row = row0 + rr + 32 * q;
                floatx4 v = {0.f, 0.f, 0.f, 0.f};
                if (row < rows) {
                    const float *p = base + (int64_t)row * ld + k;
                    if (VEC && (!KGUARD || k + 3 < kend)) {
                        v = *reinterpret_cast<const floatx4 *>(p);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (!KGUARD || k + e < kend) v[e] = p[e];
                    }
                }
                r[q] = v;
            }
        } else {
            const int i4 = tid & 31;        // which group of 4 rows
            const int kr = tid >> 5;        // 0..7
            const int row = row0 + 4 * i4;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int64_t k = k0 + kr + 8 * q;
                floatx4 v = {0.f, 0.f, 0.f, 0.f};
                if (!KGUARD || k < kend) {
                    const float *p = base + k * ld + row;
                    if (VEC && row + 3 < rows) {
                        v = *reinterpret_cast<const floatx4 *>(p);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (row + e < rows) v[e] = p[e];
                    }
                }
                r[q] = v;
            }
        }
    }

    // The same for a slab that lies wholly inside the operand (all 128 rows, all 32 k) and is 16-byte aligned:
    // four plain 128-bit loads.  The guarded form costs some four hundred instructions per slice and wavefront,
    // issued ahead of the matrix instructions of the slice.
    __device__ __forceinline__ void load_inside(const float *__restrict__ base, int64_t ld, int row0, int64_t k0, int tid) {
        if (MODE == K_CONTIG) {
            const float *p = base + (int64_t)(row0 + (tid >> 3)) * ld + k0 + 4 * (tid & 7);
#pragma unroll
            for (int q = 0; q < 4; ++q) r[q] = *reinterpret_cast<const floatx4 *>(p + (int64_t)32 * q * ld);
        } else {
            const float *p = base + (k0 + (tid >> 5)) * ld + row0 + 4 * (tid & 31);
#pragma unroll
            for (int q = 0; q < 4; ++q) r[q] = *reinterpret_cast<const floatx4 *>(p + (int64_t)8 * q * ld);
        }
    }

    __device__ __forceinline__ void store(float *__restrict__ s, int tid) const {
        if (MODE == K_CONTIG) {
            const int c4 = tid & 7, rr = tid >> 3;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *reinterpret_cast<floatx4 *>(s + (rr + 32 * q) * PITCH_K + 4 * c4) = r[q];
        } else {
            const int i4 = tid & 31, kr = tid >> 5;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *reinterpret_cast<floatx4 *>(s + (kr + 8 * q) * PITCH_R + 4 * i4) = r[q];
        }
    }
};

// Four k-values of one 32-row fragment for the calling lane: k = kk + 4 * half + {0,1,2,3}.
template <int MODE>
__device__ __forceinline__ floatx4 fragment(const float *__restrict__ s, int row, int kk, int half) {
    if (MODE == K_CONTIG) {
        return *reinterpret_cast<const floatx4 *>(s + row * PITCH_K + kk + 4 * half);
    } else {
        floatx4 v;
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = s[(kk + 4 * half + q) * PITCH_R + row];
        return v;
    }
}

// One k slice of 32 for the calling wavefront's 64 x 64 sub-tile.
template <int AMODE, int BMODE>
__device__ __forceinline__ void mma_slice(const float *__restrict__ sA, const float *__restrict__ sB,
                                          floatx16 (&acc)[2][2], int wm, int wn, int lane) {
    const int r = lane & 31, half = lane >> 5;
#pragma unroll
    for (int kk = 0; kk < BK; kk += 8) {
        floatx4 a[2], b[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) a[i] = fragment<AMODE>(sA, wm * 64 + i * 32 + r, kk, half);
#pragma unroll
        for (int j = 0; j < 2; ++j) b[j] = fragment<BMODE>(sB, wn * 64 + j * 32 + r, kk, half);
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][q], b[j][q], acc[i][j], 0, 0, 0);
    }
}

// Decodes index t of the lower-triangular tile list (0,0),(1,0),(1,1),(2,0),... into (row, col).
__device__ __forceinline__ void tri_decode(int t, int &tm, int &tn) {
    int m = (int)((sqrtf(8.0f * (float)t + 1.0f) - 1.0f) * 0.5f);
    while ((m + 1) * (m + 2) / 2 <= t) ++m;
    while (m * (m + 1) / 2 > t) --m;
    tm = m;
    tn = t - m * (m + 1) / 2;
}

// Epilogue for one accumulator set: C = alpha * acc + beta * C, optional mirrored copy.  With beta != 0 the
// old values of a 32 x 32 block are all loaded before the first store, so that their latencies overlap
// (a load issued after a store to the same array would otherwise have to wait for it).
template <int V0 = 0, int V1 = 16>
__device__ __forceinline__ void epilogue(const floatx16 (&acc)[2][2], float *__restrict__ C, int64_t ldc,
                                         int M, int N, int tm, int tn, float alpha, float beta,
                                         bool mirror, int wm, int wn, int lane,
                                         const float *__restrict__ D = nullptr, int64_t ldd = 0, bool sym_diag = false) {
    const int r = lane & 31, half = lane >> 5;
    if (D) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int col = tn * BN + wn * 64 + j * 32 + r;
                const int row_base = tm * BM + wm * 64 + i * 32 + 4 * half;
                float add[V1 - V0];
#pragma unroll
                for (int v = V0; v < V1; ++v) {
                    const int row = row_base + 8 * (v >> 2) + (v & 3);
                    add[v - V0] = (row < M && col < N) ? D[(int64_t)row * ldd + col] : 0.f;
                }
#pragma unroll
                for (int v = V0; v < V1; ++v) {
                    const int row = row_base + 8 * (v >> 2) + (v & 3);
                    // a tile on the diagonal of a symmetric output keeps its lower half and mirrors it: the
                    // product need not be symmetric to the last bit, the output must be
                    if (row < M && col < N && (!sym_diag || row >= col)) {
                        const float val = alpha * acc[i][j][v] + add[v - V0];
                        C[(int64_t)row * ldc + col] = val;
                        if (mirror || sym_diag) C[(int64_t)col * ldc + row] = val;
                    }
                }
            }
        return;
    }
    // All old values of the thread's four 32 x 32 blocks are requested before the first store: stores to C and
    // loads from C cannot be reordered by the compiler, and block by block this was four memory round trips
    // at the end of every workgroup (a quarter of a K = 128 trailing update).
    float old[2][2][V1 - V0], old_t[2][2][V1 - V0];
    if (beta != 0.f) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int col = tn * BN + wn * 64 + j * 32 + r;
                const int row_base = tm * BM + wm * 64 + i * 32 + 4 * half;
#pragma unroll
                for (int v = V0; v < V1; ++v) {
                    const int row = row_base + 8 * (v >> 2) + (v & 3);
                    const bool ok = row < M && col < N;
                    old[i][j][v - V0] = ok ? C[(int64_t)row * ldc + col] : 0.f;
                    old_t[i][j][v - V0] = (ok && mirror) ? C[(int64_t)col * ldc + row] : 0.f;
                }
            }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = tn * BN + wn * 64 + j * 32 + r;
            const int row_base = tm * BM + wm * 64 + i * 32 + 4 * half;
#pragma unroll
            for (int v = V0; v < V1; ++v) {
                const int row = row_base + 8 * (v >> 2) + (v & 3);
                if (row < M && col < N) {
                    float val = alpha * acc[i][j][v];
                    float vt = val;
                    if (beta != 0.f) { val += beta * old[i][j][v - V0]; vt += beta * old_t[i][j][v - V0]; }
                    C[(int64_t)row * ldc + col] = val;
                    // symmetric output (M == N): transposed element of a strictly-lower tile
                    if (mirror) C[(int64_t)col * ldc + row] = vt;
                }
            }
        }
}

// CHUNK > 0: two-level accumulation.  A chain of matrix instructions rounds its running sum to fp32 at every link,
// so the error of a long k range grows like sqrt(links) * 2^-24 of the sum (1e-6 after 3000 tokens, which the
// greedy loop downstream turns into removal-order differences).  With CHUNK the accumulators are added to a
// second fp32 set and reset every CHUNK slices (32 * CHUNK values of k): a chain restarts from zero after
// 16 * CHUNK links, and the second set takes one rounding per chunk instead of one per link, so the error is
// about (sqrt(16 CHUNK / chunks) + sqrt(chunks)) * 2^-25 of the sum -- 1e-7 for a dozen chunks of 256.  A
// second set in fp64 does not fit the register file at two workgroups per compute unit; callers bound the
// number of chunks per launch through the k range they give a workgroup.  The products are unchanged.
// FUSED (the instantiation that F_PARTIAL launches use): no second launch for the sum over the splits.  Every workgroup
// writes its accumulators through to memory and counts itself at its tile; the one that counts last reads all the sets
// back, adds them in split order (the same order, hence the same bits, whoever is last) and applies the epilogue.
template <int AMODE, int BMODE, bool VEC, bool KGUARD, bool DOT = false, int CHUNK = 0, bool FUSED = false>
__global__ __launch_bounds__(THREADS, 2) void gemm_kernel(Args g) {
    __shared__ __attribute__((aligned(16))) float lds[2][2][SLAB];
    if (gate_closed(g.gate, g.gate_above)) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    int tm, tn, split = 0, tile_linear;
    if (g.flags & F_TRI_GRID) {
        // Workgroups are dealt to the 8 XCDs round-robin by blockIdx.x.  Neighbouring entries of the tile
        // list share their row slab of A, so each XCD takes a contiguous eighth of the list and finds
        // that slab in its own L2.
        // (Not when the k range shrinks with the tile row: an eighth of the list would then be an eighth of the tiles
        // and far from an eighth of the work.  Dealt one by one, every XCD gets long and short tiles alike, and the
        // longest go out first.)
        const int n = gridDim.x, x = blockIdx.x % 8;
        tile_linear = (g.flags & F_KSTART_MAXMN) ? (int)blockIdx.x : x * (n / 8) + min(x, n % 8) + blockIdx.x / 8;
        tri_decode(tile_linear, tm, tn);
    } else {
        tile_linear = blockIdx.x;
        tm = blockIdx.x / g.tiles_n;
        tn = blockIdx.x % g.tiles_n;
        if ((g.flags & F_LOWER_ONLY) && tn > tm) return;
    }
    if (g.flags & F_PARTIAL) split = blockIdx.y;

    const float *A = g.A + (int64_t)blockIdx.z * g.strideA;
    const float *B = g.B + (int64_t)blockIdx.z * g.strideB;
    float *C = g.C + (int64_t)blockIdx.z * g.strideC;

    int64_t kb = 0, ke = g.K;
    if (g.flags & F_KSTART_N) kb = (int64_t)tn * BN;
    if (g.flags & F_KSTART_MAXMN) kb = (int64_t)(tm > tn ? tm : tn) * BM;
    if (g.flags & F_KEND_M) { int64_t e = (int64_t)(tm + 1) * BM; ke = e < ke ? e : ke; }
    if (g.flags & F_SPLIT_TILE_RANGE) {
        // whole slices per split; the last splits of a short range may get nothing and write zeros
        const int64_t slices = ke > kb ? (ke - kb + BK - 1) / BK : 0;
        const int64_t per = (slices + gridDim.y - 1) / gridDim.y * BK;
        const int64_t b2 = kb + split * per, e2 = b2 + per;
        kb = b2 < ke ? b2 : ke;
        ke = e2 < ke ? e2 : ke;
    } else if (g.flags & F_PARTIAL) {
        kb = (int64_t)split * g.k_chunk;
        int64_t e = kb + g.k_chunk;
        ke = e < g.K ? e : g.K;
    }

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    float acc2[CHUNK > 0 ? 64 : 1];
#pragma unroll
    for (int e = 0; e < (CHUNK > 0 ? 64 : 1); ++e) acc2[e] = 0.f;
    int in_chunk = 0;

    const int64_t nslices = ke > kb ? (ke - kb + BK - 1) / BK : 0;
    Slab<AMODE, VEC, KGUARD> ra;
    Slab<BMODE, VEC, KGUARD> rb;
    // tile rows and k range wholly inside both operands: unguarded loads (uniform over the workgroup)
    const bool inside = VEC && (tm + 1) * BM <= g.M && (tn + 1) * BN <= g.N && (ke - kb) % BK == 0;
    if (nslices > 0) {
        if (inside) {
            ra.load_inside(A, g.lda, tm * BM, kb, tid);
            rb.load_inside(B, g.ldb, tn * BN, kb, tid);
        } else {
            ra.load(A, g.lda, tm * BM, g.M, kb, ke, tid);
            rb.load(B, g.ldb, tn * BN, g.N, kb, ke, tid);
        }
        ra.store(lds[0][0], tid);
        rb.store(lds[0][1], tid);
    }
    __syncthreads();
    int cur = 0;
    for (int64_t s = 0; s < nslices; ++s) {
        const bool more = (s + 1 < nslices);
        if (more) {
            if (inside) {
                ra.load_inside(A, g.lda, tm * BM, kb + (s + 1) * BK, tid);
                rb.load_inside(B, g.ldb, tn * BN, kb + (s + 1) * BK, tid);
            } else {
                ra.load(A, g.lda, tm * BM, g.M, kb + (s + 1) * BK, ke, tid);
                rb.load(B, g.ldb, tn * BN, g.N, kb + (s + 1) * BK, ke, tid);
            }
        }
        mma_slice<AMODE, BMODE>(lds[cur][0], lds[cur][1], acc, wm, wn, lane);
        if (more) {
            ra.store(lds[cur ^ 1][0], tid);
            rb.store(lds[cur ^ 1][1], tid);
        }
        if (CHUNK > 0 && (++in_chunk == CHUNK || !more)) {      // uniform over the workgroup
            in_chunk = 0;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        acc2[(i * 2 + j) * 16 + v] += acc[i][j][v];
                        acc[i][j][v] = 0.f;
                    }
        }
        __syncthreads();
        cur ^= 1;
    }
    if (CHUNK > 0) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = acc2[(i * 2 + j) * 16 + v];
    }

    if (FUSED && (g.flags & F_PARTIAL)) {
        const int nsplit = gridDim.y;
        float *sets = g.partial + ((int64_t)blockIdx.z * nsplit * gridDim.x + tile_linear) * (64 * THREADS);
        const int64_t set_stride = (int64_t)gridDim.x * (64 * THREADS);
        float *dst = sets + split * set_stride;
        // written through to memory (the reader may sit on another XCD) ...
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    __hip_atomic_store(dst + ((i * 2 + j) * 16 + v) * THREADS + tid, acc[i][j][v], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // ... and acknowledged, for every thread of the workgroup, before the workgroup counts itself
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        int *ticket = reinterpret_cast<int *>(&lds[0][0][0]);      // every wavefront is past the last slice's barrier
        if (tid == 0)
            *ticket = __hip_atomic_fetch_add(g.tile_counters + (int64_t)blockIdx.z * gridDim.x + tile_linear, 1, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (*ticket != nsplit - 1) return;                          // uniform
        if (tid == 0)
            __hip_atomic_store(g.tile_counters + (int64_t)blockIdx.z * gridDim.x + tile_linear, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // the last one: all sets in split order, its own included (read back, so that the sum does not depend on who is last)
        for (int s2 = 0; s2 < nsplit; ++s2) {
            const float *src = sets + s2 * set_stride;
            float part[64];
#pragma unroll
            for (int e = 0; e < 64; ++e) part[e] = __hip_atomic_load(src + e * THREADS + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const float pv = part[(i * 2 + j) * 16 + v];
                        acc[i][j][v] = (s2 == 0) ? (0.f + pv) : acc[i][j][v] + pv;
                    }
        }
    }
    if (DOT) {
        // every thread sums its 64 products in fp64, then the 256 partial sums are added in thread order
        const int r = lane & 31, half = lane >> 5;
        double sum = 0.0;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int col = tn * BN + wn * 64 + j * 32 + r;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = tm * BM + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                    if (row < g.M && col < g.N) {
                        const float c = C[(int64_t)row * g.ldc + col];
                        sum += ((double)(g.alpha * acc[i][j][v]) + (double)g.dot_lambda * (double)c) * (double)c;
                    }
                }
            }
        double *red = reinterpret_cast<double *>(&lds[0][0][0]);   // all waves are past the last slice's barrier
        red[tid] = sum;
        __syncthreads();
        if (tid == 0) {
            double total = 0.0;
            for (int q = 0; q < THREADS; ++q) total += red[q];
            g.dot_partial[tile_linear] = total;
        }
        return;
    }
    const bool mirror = (g.flags & F_MIRROR) && (tm != tn);
    epilogue(acc, C, g.ldc, g.M, g.N, tm, tn, g.alpha, g.beta, mirror, wm, wn, lane,
             g.D ? g.D + (int64_t)blockIdx.z * g.strideC : nullptr, g.ldd, (g.flags & F_MIRROR) && tm == tn);
}

// Host-side launch of a full (non split-K) product.  `batch` >= 1.
template <int AMODE, int BMODE, bool VEC, bool KGUARD, bool DOT = false>
inline hipError_t launch(Args g, int batch, hipStream_t stream) {
    if (g.M <= 0 || g.N <= 0 || batch <= 0) return hipSuccess;
    const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    g.tiles_n = tiles_n;
    dim3 grid;
    if (g.flags & F_TRI_GRID) grid = dim3(tiles_m * (tiles_m + 1) / 2, 1, batch);
    else grid = dim3(tiles_m * tiles_n, 1, batch);
    hipLaunchKernelGGL((gemm_kernel<AMODE, BMODE, VEC, KGUARD, DOT>), grid, dim3(THREADS), 0, stream, g);
    return hipGetLastError();
}

// A product whose tile list alone cannot fill the chip: `nsplit` workgroups share every tile's k range and the last of
// them to finish adds their accumulators in split order and applies the epilogue (FUSED above).  `partial` must hold
// nsplit * tiles * batch accumulator sets of 64 * THREADS floats, `tile_counters` tiles * batch zeros.
template <int AMODE, int BMODE, bool VEC, bool KGUARD>
inline hipError_t launch_splitk(Args g, int batch, int nsplit, hipStream_t stream) {
    if (nsplit <= 1) return launch<AMODE, BMODE, VEC, KGUARD>(g, batch, stream);
    if (g.M <= 0 || g.N <= 0 || batch <= 0) return hipSuccess;
    if (!g.partial || !g.tile_counters) return hipErrorInvalidValue;
    const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    g.tiles_n = tiles_n;
    const int tiles = (g.flags & F_TRI_GRID) ? tiles_m * (tiles_m + 1) / 2 : tiles_m * tiles_n;
    g.flags |= F_PARTIAL | F_SPLIT_TILE_RANGE;
    hipLaunchKernelGGL((gemm_kernel<AMODE, BMODE, VEC, KGUARD, false, 0, true>), dim3(tiles, nsplit, batch), dim3(THREADS), 0, stream, g);
    return hipGetLastError();
}

}  // namespace gemm
}  // namespace ziplm
