// Greedy structured OBS pruning (Algorithm 1; Eq. 2 score, Eq. 3 weight update, Eq. 4 elimination
// of the removed structure from the inverse Hessian).
//
// State inside a call: Hd = the inverse Hessian in fp64 (workspace copy of the caller's fp32 Hinv;
// fp32 storage of this matrix loses the 1e-4 agreement with exact arithmetic over thousands of
// eliminations when H is ill conditioned), W in fp32 in place, score reductions in fp64.
//
// Single columns (group_size == 1): one persistent cooperative kernel runs all n_remove steps; the
// steps are separated by device-wide barriers, the host is not involved.  Per step
//     candidates -> barrier -> argmin (every workgroup redundantly) + update -> barrier.
// The update pass over W also produces the partial squared column norms the next step's scores need
// and the pass over Hd refreshes a compact copy of its diagonal, so a step reads the state once.
// Rows of Hd that belong to removed columns are skipped; removed columns are masked per lane.
//
// Larger structures (2 <= group_size <= 64): two ordinary launches per step,
//     score  (eight workgroups per live structure: block inverse and Gram contraction of an eighth of the
//             rows, both on the fp64 matrix cores)
//     update (every workgroup picks the cheapest structure itself from the scores and forms the coefficients
//             C_H = Hd[:,S] B, C_W = W[:,S] B of its own rows on the fly; both products on the fp64 matrix cores),
// because on this machine a dependent launch costs more than the arithmetic of a step.
#include <hip/hip_cooperative_groups.h>

#include <type_traits>

#include "common.h"

namespace ziplm {

int device_cu_count();
bool lazy_columns_feasible(int d_row, int d_col);
size_t lazy_columns_workspace_bytes(int d_row, int d_col, int n_snap);
int lazy_columns_pack(int n_layers, int d_row, int d_col);
size_t lazy_columns_pack_workspace_bytes(int pack, int d_row, int d_col, int n_snap);
size_t lazy_columns_pack_exchange_bytes(int pack, int d_row, int d_col);
int lazy_columns_launch(float *W, float *Hinv, int pack, int64_t stride_w, int64_t stride_hinv, int d_row, int d_col,
                        int n_remove, int32_t *order_out, double *err_out, const uint8_t *alive_in, int n_snap,
                        const int32_t *snap_steps_host, float *W_snap, void *workspace, void *exchange,
                        hipStream_t st, int **status_dev_out, int stall_wg);

// Single columns go to the deferred-update kernel whenever its per-workgroup state fits LDS; the eager kernel
// below (one full read-modify-write of the state per step) covers the other shapes and has an entry point of its own.
static bool use_lazy_columns(int d_row, int d_col) { return lazy_columns_feasible(d_row, d_col); }

// What the device's status word means to the caller.
static int status_to_return_code(int status) {
    if (status > 0) return ZIPLM_ERR_NOT_PD;          // 1 + step with a non-positive pivot
    if (status == -1) return ZIPLM_ERR_DEVICE;        // a bounded wait gave up
    if (status < -1) return ZIPLM_ERR_INVALID_ARG;    // -(2 + step): no live structure left at that step
    return ZIPLM_OK;
}

constexpr int PT = 512;        // threads per workgroup of the persistent kernel (= columns per tile)
constexpr int H_ROWS = 8;      // rows of Hd per tile
constexpr int W_ROWS = 32;     // rows of W per tile (one partial norm per tile and column)
constexpr unsigned long long kBarrierTimeoutTicks = 400000000ull;  // 4 s of the 100 MHz wall clock

struct PruneState {
    float *W;
    float *Hinv;
    double *Hd;
    int m, d, g, G, n_remove;
    int32_t *order;
    double *err;
    const uint8_t *alive_in;
    uint8_t *alive;      // per structure
    double *Pn;          // [nrc][d] partial squared column norms (g == 1)
    double *diag;        // [d] compact diagonal of Hd (g == 1)
    double *cand_score;  // [ncc]
    int *cand_idx;       // [ncc]
    int nrc, ncc;
    const int *snap_of_step;  // [n_remove + 1] first snapshot taken after that many removals, or -1
    const int *snap_next;     // [n_snap] next snapshot at the same step, or -1
    float *W_snap;
    unsigned *bar;       // barrier arrival counter
    int *status;         // 0 ok, >0: 1 + step with a non-positive pivot, -1: barrier timed out, < -1: -(2 + step) with nothing left alive
    // group path
    double *score;       // [G][SCORE_PARTS]
    double *Binv;        // [G][g*g]
    int *dead_step;      // [G] step at which the structure was removed; kNever while alive, -1 if it came in removed
};

// Several layers of one shape in one launch (grid dimension y = layer): layer l uses the state of layer 0
// with every workspace pointer moved by l * ws_bytes and the caller's arrays by their own strides.  The
// snapshot schedule is shared.  All strides are 0 for a single layer.
struct BatchShift {
    size_t ws_bytes;
    long long w, hinv, order, err, snap;    // elements
};

__device__ __forceinline__ PruneState layer_state(PruneState P, const BatchShift &B, int l) {
    if (l == 0) return P;
    const size_t o = (size_t)l * B.ws_bytes;
    auto mv = [o](auto *&ptr) { if (ptr) ptr = reinterpret_cast<std::remove_reference_t<decltype(ptr)>>(reinterpret_cast<char *>(ptr) + o); };
    mv(P.Hd); mv(P.alive); mv(P.bar); mv(P.status); mv(P.score); mv(P.Binv); mv(P.dead_step);
    P.W += (long long)l * B.w;
    P.Hinv += (long long)l * B.hinv;
    P.order += (long long)l * B.order;
    P.err += (long long)l * B.err;
    if (P.W_snap) P.W_snap += (long long)l * B.snap;
    return P;
}

// ---------------------------------------------------------------------------------------------
// helpers
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ bool better(double s1, int i1, double s2, int i2) {
    // strict order: smaller score first, lower index on equal scores; index -1 = "none"
    if (i2 < 0) return i1 >= 0;
    if (i1 < 0) return false;
    return (s1 < s2) || (s1 == s2 && i1 < i2);
}

// Workgroup barrier that orders LDS traffic only: __syncthreads() also waits for every global load in flight,
// which would serialise loads issued ahead of the barrier with the work behind it.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int NT>
__device__ __forceinline__ void block_argmin(double &s, int &i, double *sh_s, int *sh_i) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const double so = __shfl_down(s, o);
        const int io = __shfl_down(i, o);
        if (better(so, io, s, i)) { s = so; i = io; }
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { sh_s[wave] = s; sh_i[wave] = i; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double bs = sh_s[0];
        int bi = sh_i[0];
        for (int w = 1; w < NT / 64; ++w)
            if (better(sh_s[w], sh_i[w], bs, bi)) { bs = sh_s[w]; bi = sh_i[w]; }
        sh_s[0] = bs;
        sh_i[0] = bi;
    }
    __syncthreads();
    s = sh_s[0];
    i = sh_i[0];
    __syncthreads();
}

// Device-wide barrier for a cooperative launch (all workgroups resident).  A monotonically
// increasing arrival counter; `epoch` counts the barriers this workgroup has passed.  Waiting is
// bounded: after kBarrierTimeoutTicks the waiter raises status = -1, which every waiter polls, so
// that all workgroups leave their loops and the grid drains.  Returns false on abort.
__device__ __forceinline__ bool grid_barrier(unsigned *counter, unsigned &epoch, unsigned nblocks, int *status) {
    __shared__ int ok_flag;
    __syncthreads();
    if (threadIdx.x == 0) {
        epoch += 1;
        __threadfence();
        atomicAdd(counter, 1u);
        const unsigned target = epoch * nblocks;
        const unsigned long long t0 = wall_clock64();
        int ok = 1;
        unsigned spins = 0;
        while (__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            __builtin_amdgcn_s_sleep(1);
            if ((++spins & 63u) == 0u) {
                if (__hip_atomic_load(status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == -1) { ok = 0; break; }
                if (wall_clock64() - t0 > kBarrierTimeoutTicks) {
                    __hip_atomic_store(status, -1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    ok = 0;
                    break;
                }
            }
        }
        __threadfence();
        ok_flag = ok;
    }
    __syncthreads();
    const bool ok = ok_flag != 0;
    __syncthreads();
    return ok;
}

__device__ __forceinline__ void snapshot_copy(const PruneState &P, int removed, int gtid, int gthreads) {
    int q = P.snap_of_step ? P.snap_of_step[removed] : -1;
    while (q >= 0) {
        float *dst = P.W_snap + (size_t)q * P.m * P.d;
        const size_t total = (size_t)P.m * P.d;
        for (size_t idx = gtid; idx < total; idx += gthreads) {
            const int j = (int)(idx % P.d);
            const bool live = P.dead_step ? (P.dead_step[j / P.g] >= removed) : (P.alive[j / P.g] != 0);
            dst[idx] = live ? P.W[idx] : 0.f;
        }
        q = P.snap_next[q];
    }
}

// ---------------------------------------------------------------------------------------------
// group_size == 1: persistent cooperative kernel
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(PT) void prune_columns_kernel(PruneState P) {
    __shared__ double sh_s[PT / 64];
    __shared__ int sh_i[PT / 64];
    const int nb = gridDim.x, b = blockIdx.x, tid = threadIdx.x;
    const int gtid = b * PT + tid, gthreads = nb * PT;
    const int d = P.d, m = P.m;
    unsigned epoch = 0;

    // ---- set-up: fp64 copy of the inverse Hessian, alive flags, diagonal, partial column norms ----
    {
        const size_t total = (size_t)d * d;
        for (size_t idx = gtid; idx < total; idx += gthreads) P.Hd[idx] = (double)P.Hinv[idx];
        for (int j = gtid; j < d; j += gthreads) {
            P.alive[j] = P.alive_in ? (P.alive_in[j] != 0) : 1;
            P.diag[j] = (double)P.Hinv[(size_t)j * d + j];
        }
        for (int tile = b; tile < P.nrc * P.ncc; tile += nb) {
            const int rc = tile / P.ncc, j = (tile % P.ncc) * PT + tid;
            if (j < d) {
                double s = 0.0;
                const int i1 = min(m, (rc + 1) * W_ROWS);
                for (int i = rc * W_ROWS; i < i1; ++i) {
                    const double w = (double)P.W[(size_t)i * d + j];
                    s += w * w;
                }
                P.Pn[(size_t)rc * d + j] = s;
            }
        }
    }
    bool ok = grid_barrier(P.bar, epoch, nb, P.status);

    const int n_h_tiles = ((d + H_ROWS - 1) / H_ROWS) * P.ncc;
    const int n_w_tiles = P.nrc * P.ncc;
    int t = 0;
    for (; ok && t < P.n_remove; ++t) {
        snapshot_copy(P, t, gtid, gthreads);

        // ---- candidates: Eq. 2 for single columns, ||W[:,j]||^2 / Hd[j][j], per chunk of PT columns
        for (int cc = b; cc < P.ncc; cc += nb) {
            const int j = cc * PT + tid;
            double s = 0.0;
            int idx = -1;
            if (j < d && P.alive[j]) {
                double nrm = 0.0;
                for (int rc = 0; rc < P.nrc; ++rc) nrm += P.Pn[(size_t)rc * d + j];
                const double dj = P.diag[j];
                if (dj > 0.0) { s = nrm / dj; idx = j; }
                else __hip_atomic_store(P.status, 1 + t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            block_argmin<PT>(s, idx, sh_s, sh_i);
            if (tid == 0) { P.cand_score[cc] = s; P.cand_idx[cc] = idx; }
        }
        ok = grid_barrier(P.bar, epoch, nb, P.status);
        if (!ok) break;

        // ---- argmin over the candidates, redundantly in every workgroup (same inputs, same result)
        double best = 0.0;
        int p = -1;
        for (int cc = 0; cc < P.ncc; ++cc) {
            const double s = P.cand_score[cc];
            const int i = P.cand_idx[cc];
            if (better(s, i, best, p)) { best = s; p = i; }
        }
        const int st = __hip_atomic_load(P.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (p < 0 || st != 0) {     // uniform over the grid: status was written before the barrier
            if (gtid == 0 && st == 0) *P.status = -(2 + t);      // nothing alive: more removals asked for than live columns
            break;
        }
        if (gtid == 0) {
            P.order[t] = p;
            P.err[t] = best;
            P.alive[p] = 0;   // readers of this step treat p as removed either way
        }

        // ---- Eq. 3 and Eq. 4 with the pre-step row p of Hd (row and column p are not written) ----
        const double *R = P.Hd + (size_t)p * d;
        const double inv = 1.0 / R[p];
        for (int tile = b; tile < n_h_tiles + n_w_tiles; tile += nb) {
            if (tile < n_h_tiles) {
                const int rt = tile / P.ncc, j = (tile % P.ncc) * PT + tid;
                const bool live = (j < d) && (j != p) && P.alive[j];
                const double rj = live ? R[j] : 0.0;
                const int i1 = min(d, (rt + 1) * H_ROWS);
                for (int i = rt * H_ROWS; i < i1; ++i) {
                    if (i == p || !P.alive[i]) continue;
                    const double ci = R[i] * inv;
                    if (live) {
                        double *h = P.Hd + (size_t)i * d + j;
                        const double v = *h - ci * rj;
                        *h = v;
                        if (i == j) P.diag[j] = v;
                    }
                }
            } else {
                const int wt = tile - n_h_tiles;
                const int rc = wt / P.ncc, j = (wt % P.ncc) * PT + tid;
                const bool live = (j < d) && (j != p) && P.alive[j];
                const double rj = live ? R[j] : 0.0;
                const int i1 = min(m, (rc + 1) * W_ROWS);
                double s = 0.0;
                for (int i = rc * W_ROWS; i < i1; ++i) {
                    const double cw = (double)P.W[(size_t)i * d + p] * inv;
                    if (live) {
                        float *w = P.W + (size_t)i * d + j;
                        const float v = (float)((double)(*w) - cw * rj);
                        *w = v;
                        s += (double)v * (double)v;
                    }
                }
                if (live) P.Pn[(size_t)rc * d + j] = s;
            }
        }
        ok = grid_barrier(P.bar, epoch, nb, P.status);
    }

    // ---- final masking (last line of Algorithm 1) and write-back of the surviving inverse -------
    if (ok && t == P.n_remove) snapshot_copy(P, P.n_remove, gtid, gthreads);
    {
        const size_t totalw = (size_t)m * d;
        for (size_t idx = gtid; idx < totalw; idx += gthreads)
            if (!P.alive[idx % d]) P.W[idx] = 0.f;
        const size_t total = (size_t)d * d;
        for (size_t idx = gtid; idx < total; idx += gthreads) {
            const int i = (int)(idx / d), j = (int)(idx % d);
            P.Hinv[idx] = (P.alive[i] && P.alive[j]) ? (float)P.Hd[idx] : 0.f;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// group_size > 1: per-step launches
// ---------------------------------------------------------------------------------------------
constexpr int GMAX = 64;
constexpr int SCORE_PARTS = 8;      // workgroups that share the rows of W when one structure is scored
constexpr int kNever = 0x7fffffff;
// Structure s takes part in step t iff dead_step[s] >= t.  The workgroup that records the removal of step t
// writes t, which a workgroup still choosing step t's structure reads as "alive" just like the old value:
// all workgroups of a launch see the same set whatever the timing.

__global__ __launch_bounds__(256) void group_init_kernel(PruneState P, BatchShift B) {
    P = layer_state(P, B, blockIdx.y);
    const int gtid = blockIdx.x * 256 + threadIdx.x, gthreads = gridDim.x * 256;
    const size_t total = (size_t)P.d * P.d;
    for (size_t idx = gtid; idx < total; idx += gthreads) P.Hd[idx] = (double)P.Hinv[idx];
    for (int s = gtid; s < P.G; s += gthreads) P.dead_step[s] = (P.alive_in && P.alive_in[s] == 0) ? -1 : kNever;
}

typedef double doublex4 __attribute__((ext_vector_type(4)));

// Inverse of a symmetric positive definite 4 x 4 block by 2 x 2 blocks (Schur complement of the leading block).
// Only the upper triangle of p is read.  Returns false if one of the four successive pivots is not positive
// (they are p00, det A / p00, s00, det S / s00 with A the leading block and S the Schur complement).
__device__ __forceinline__ double rcp_newton(double x) {
    double r = __builtin_amdgcn_rcp(x);
    r = __builtin_fma(__builtin_fma(-x, r, 1.0), r, r);
    return __builtin_fma(__builtin_fma(-x, r, 1.0), r, r);
}
__device__ __forceinline__ bool spd4_inverse(const double (&p)[4][4], double (&q)[4][4]) {
    const double det_a = __builtin_fma(p[0][0], p[1][1], -p[0][1] * p[0][1]);
    const double ia = rcp_newton(det_a);
    const double a00 = p[1][1] * ia, a01 = -p[0][1] * ia, a11 = p[0][0] * ia;          // A^-1
    // T = A^-1 B with B = p[0..1][2..3]
    const double t00 = __builtin_fma(a00, p[0][2], a01 * p[1][2]), t01 = __builtin_fma(a00, p[0][3], a01 * p[1][3]);
    const double t10 = __builtin_fma(a01, p[0][2], a11 * p[1][2]), t11 = __builtin_fma(a01, p[0][3], a11 * p[1][3]);
    // S = D - B^T T
    const double s00 = p[2][2] - __builtin_fma(p[0][2], t00, p[1][2] * t10);
    const double s01 = p[2][3] - __builtin_fma(p[0][2], t01, p[1][2] * t11);
    const double s11 = p[3][3] - __builtin_fma(p[0][3], t01, p[1][3] * t11);
    const double det_s = __builtin_fma(s00, s11, -s01 * s01);
    const double is = rcp_newton(det_s);
    const double i00 = s11 * is, i01 = -s01 * is, i11 = s00 * is;                      // S^-1
    q[2][2] = i00; q[2][3] = q[3][2] = i01; q[3][3] = i11;
    q[0][2] = q[2][0] = -__builtin_fma(t00, i00, t01 * i01);                            // -T S^-1
    q[0][3] = q[3][0] = -__builtin_fma(t00, i01, t01 * i11);
    q[1][2] = q[2][1] = -__builtin_fma(t10, i00, t11 * i01);
    q[1][3] = q[3][1] = -__builtin_fma(t10, i01, t11 * i11);
    q[0][0] = a00 - __builtin_fma(q[0][2], t00, q[0][3] * t01);                          // A^-1 + T S^-1 T^T
    q[0][1] = q[1][0] = a01 - __builtin_fma(q[0][2], t10, q[0][3] * t11);
    q[1][1] = a11 - __builtin_fma(q[1][2], t10, q[1][3] * t11);
    return p[0][0] > 0.0 && det_a > 0.0 && s00 > 0.0 && det_s > 0.0;
}

// SCORE_PARTS workgroups per structure s, each with its own share of the rows of W.  Both g x g matrices of a
// workgroup live in the accumulator layout of v_mfma_f64_16x16x4_f64 (lane l supplies A[row l%16][k l/16] and
// B[k l/16][col l%16]; accumulator v holds D[row 4v + l/16][col l%16]): wavefront w holds tile row w, i.e.
// element v of tile tb is entry [16 w + 4 v + l/16][16 tb + l%16].
//   G = W[rows,S]^T W[rows,S]  (fp64) from the rows of W staged in LDS, 128 at a time.  The whole Gram matrix of
//       a 768 x 64 structure is 3072 matrix instructions, 20 us on the four SIMDs of one compute unit: that,
//       not memory, is why the rows are shared out;
//   B = (Hd[S,S])^-1 by the symmetric sweep, four pivots at a time: with K the pivots and Q = M[K,K]^-1,
//           M[K,K] <- -Q,  M[K,j] <- Q M[K,j],  M[i,K] <- (Q M[K,i])^T,  M[i,j] <- M[i,j] - M[i,K] Q M[K,j],
//       which ends at -B after g / 4 steps.  The matrix stays symmetric, so all a step needs from other
//       wavefronts are the four rows K; they go through LDS (the four pivots of a step are exactly the rows
//       one accumulator element of one wavefront holds), every thread inverts the 4 x 4 pivot block itself, and
//       the rank-4 update of a tile is ONE matrix instruction.  An elimination that kept a column per thread
//       and eliminated pivot by pivot was bound by LDS traffic (32 broadcast values per thread and pivot pair).
//       The pivots of a positive definite block are its successive Schur complements, all > 0: no pivoting;
//       a non-positive one is the error path.  Every part repeats the inversion (same inputs, same operations,
//       same B); part 0 stores B for the update launch;
//   score_s[part] = sum_{i in rows} w_i B w_i^T = <B, G>, straight from the two register sets; the update
//       launch adds the parts in index order.
__global__ __launch_bounds__(256) void group_score_kernel(PruneState P, BatchShift B, int step) {
    P = layer_state(P, B, blockIdx.z);
    constexpr int GR = 128;                      // rows of W per pass of the Gram product
    __shared__ __attribute__((aligned(16))) float Wt[GR][GMAX + 4];
    __shared__ __attribute__((aligned(16))) double Rk[2][4][GMAX];     // the four pivot rows of a step, two buffers
    __shared__ double red[256];
    __shared__ int bad;
    const int s = blockIdx.x, tid = threadIdx.x, g = P.g, d = P.d;
    const int lane = tid & 63, wave = tid >> 6, q4 = lane >> 4, cl16 = lane & 15;
    const int part_idx = blockIdx.y;
    const int c0 = s * g;
    // this workgroup's rows of W: a SCORE_PARTS-th of them, in whole groups of four (one matrix-core k step)
    const int rows_per_part = ((P.m + SCORE_PARTS - 1) / SCORE_PARTS + 3) / 4 * 4;
    const int r_begin = min(P.m, part_idx * rows_per_part), r_end = min(P.m, r_begin + rows_per_part);
    // A kernel this short is a chain of memory round trips: the status word, the structure's state, its block
    // of the inverse Hessian and the first rows of W are all asked for before any of them is looked at.
    const int status = *P.status;
    const int ds = P.dead_step[s];
    // The g x g block in accumulator layout; beyond g the matrix is continued by the identity, which the
    // elimination leaves alone.
    doublex4 bacc[4];
#pragma unroll
    for (int tb = 0; tb < 4; ++tb)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int i = 16 * wave + 4 * v + q4, j = 16 * tb + cl16;
            bacc[tb][v] = (i < g && j < g) ? P.Hd[(size_t)(c0 + i) * d + c0 + j] : (i == j ? 1.0 : 0.0);
        }
    float wv[GR / 4];                            // rows wave + 4 q of the pass, column `lane` of the structure
    auto load_rows = [&](int i0) {
#pragma unroll
        for (int q = 0; q < GR / 4; ++q) {
            const int r = i0 + wave + 4 * q;
            wv[q] = (r < r_end && lane < g) ? P.W[(size_t)r * d + c0 + lane] : 0.f;
        }
    };
    load_rows(r_begin);
    if (status != 0) return;
    if (ds < step) {
        if (tid == 0) P.score[s * SCORE_PARTS + part_idx] = 0.0;
        return;
    }
    if (tid == 0) bad = 0;

    // ---- Gram matrix: this wavefront's tile row, tiles (wave, x), x < 4 (g <= 64)
    const int nt = (g + 15) / 16;
    doublex4 acc[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) acc[x] = doublex4{0.0, 0.0, 0.0, 0.0};
    for (int i0 = r_begin; i0 < r_end; i0 += GR) {
        if (i0 != r_begin) {
            lds_barrier();                       // the previous pass has been read
            load_rows(i0);
        }
#pragma unroll
        for (int q = 0; q < GR / 4; ++q) Wt[wave + 4 * q][lane] = wv[q];
        lds_barrier();
        // k groups of four rows, in whole blocks of eight (rows past the end were staged as zeros): a loop around
        // matrix-core instructions is only unrolled when its trip count is known to be a multiple of the factor
        const int nks8 = (min(GR, r_end - i0) + 31) / 32;
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            if (wave < nt && x < nt) {                  // wave-uniform
                const int ta = wave, tb = x;
                for (int k8 = 0; k8 < nks8; ++k8) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int ks = 8 * k8 + e;
                        const double av = (double)Wt[4 * ks + q4][16 * ta + cl16];
                        const double bv = (double)Wt[4 * ks + q4][16 * tb + cl16];
                        acc[x] = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc[x], 0, 0, 0);
                    }
                }
            }
        }
    }
    // ---- -B by the symmetric sweep, four pivots per step
    bool stop = false;
    for (int ta = 0; ta < 4 && !stop; ++ta) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int k0 = 16 * ta + 4 * v;          // pivots k0 .. k0 + 3: element v of tile row ta, one per q4
            if (k0 >= g) { stop = true; break; }
            const int buf = v & 1;
            if (wave == ta) {
#pragma unroll
                for (int tb = 0; tb < 4; ++tb) Rk[buf][q4][16 * tb + cl16] = bacc[tb][v];
            }
            // one barrier per step: a buffer is written again two steps later, behind the barrier of the step in
            // between, which every wavefront reaches after its reads of this one
            lds_barrier();
            double pv[4][4], qv[4][4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int f = 0; f < 4; ++f) pv[e][f] = Rk[buf][e][k0 + f];
            if (!spd4_inverse(pv, qv)) {            // uniform: every thread read the same block
                if (tid == 0) bad = 1;
                stop = true;
                break;
            }
            // row q4 of Q for this lane
            double qrow[4];
#pragma unroll
            for (int f = 0; f < 4; ++f) qrow[f] = (q4 == 0) ? qv[0][f] : (q4 == 1) ? qv[1][f] : (q4 == 2) ? qv[2][f] : qv[3][f];
            // B operands: S = Q M[K,:] restricted to this lane's k (= q4) and columns; for the columns of K minus Q
            const bool col_in_k = (cl16 >> 2) == v;          // within tile column ta
            const int cf = cl16 & 3;
            const double minus_q = -((cf == 0) ? qrow[0] : (cf == 1) ? qrow[1] : (cf == 2) ? qrow[2] : qrow[3]);
            double sop[4];
#pragma unroll
            for (int tb = 0; tb < 4; ++tb) {
                const int j = 16 * tb + cl16;
                double acc_s = qrow[0] * Rk[buf][0][j];
                acc_s = __builtin_fma(qrow[1], Rk[buf][1][j], acc_s);
                acc_s = __builtin_fma(qrow[2], Rk[buf][2][j], acc_s);
                acc_s = __builtin_fma(qrow[3], Rk[buf][3][j], acc_s);
                sop[tb] = (tb == ta && col_in_k) ? minus_q : acc_s;
            }
            // A operand: column K_q4 of this wavefront's rows = row K_q4 at those columns (symmetry)
            const double aop = -Rk[buf][q4][16 * wave + cl16];
#pragma unroll
            for (int tb = 0; tb < 4; ++tb) {
                doublex4 base = bacc[tb];
                if (tb == ta && col_in_k) base = doublex4{0.0, 0.0, 0.0, 0.0};
                base = __builtin_amdgcn_mfma_f64_16x16x4f64(aop, sop[tb], base, 0, 0, 0);
                if (wave == ta) base[v] = sop[tb];          // rows K themselves
                bacc[tb] = base;
            }
        }
    }
    lds_barrier();
    if (bad) {
        if (tid == 0 && part_idx == 0) atomicCAS(P.status, 0, 1 + step);
        return;
    }
    if (part_idx == 0) {
        double *Bout = P.Binv + (size_t)s * g * g;
#pragma unroll
        for (int tb = 0; tb < 4; ++tb)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = 16 * wave + 4 * v + q4, j = 16 * tb + cl16;
                if (i < g && j < g) Bout[i * g + j] = -bacc[tb][v];
            }
    }

    // ---- <B, G>: both in the same layout; G is zero beyond g
    double part = 0.0;
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int v = 0; v < 4; ++v) part -= bacc[x][v] * acc[x][v];
    red[tid] = part;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if (tid < o) red[tid] += red[tid + o];
        __syncthreads();
    }
    if (tid == 0) P.score[s * SCORE_PARTS + part_idx] = red[0];
}

// Second (and last) launch of a step.  Every workgroup finds the cheapest live structure p itself from the
// scores (lowest index on ties; the same inputs give the same answer everywhere; workgroup 0 records it), takes
// B = (Hd[S,S])^-1 of that structure as left by the scoring launch, and for each of its 16-row tiles forms the
// coefficients  C = rows[:, S] B  on the fly before applying
//     Hd[i][j] -= sum_b C_H[i][b] Hd[S_b][j]   and   W[i][j] -= sum_b C_W[i][b] Hd[S_b][j]   (Eq. 4, Eq. 3).
// Rows and columns of the selected structure and of earlier removed ones are left alone (they are zeroed at
// the end), so the rows Hd[S,:] and the columns Hd[:,S] read here are the pre-step ones for every workgroup.
constexpr int G_ROWS = 16;
constexpr int G_CT = 2;             // 16-column tiles per wavefront: a workgroup covers 64 G_CT columns
constexpr int G_COLS = 4 * 16 * G_CT;
__global__ __launch_bounds__(256) void group_update_kernel(PruneState P, BatchShift Bsh, int step) {
    P = layer_state(P, Bsh, blockIdx.y);
    __shared__ double Bs[GMAX][GMAX + 1];     // B of the selected structure, zero beyond g
    __shared__ double As[G_ROWS][GMAX + 1];   // this tile's rows restricted to the columns of S, zero beyond g
    __shared__ double Cs[G_ROWS][GMAX + 1];   // this tile's rows of C_H or C_W
    __shared__ double sh_s[4];
    __shared__ int sh_i[4];
    const int g = P.g, d = P.d, m = P.m, tid = threadIdx.x;
    // A kernel this short is a chain of memory round trips: everything that can be asked for at once is (the
    // status word with the scores here; all operands of the tile once p is known, further down).
    const int status = *P.status;
    double best = 0.0;
    int p = -1;
    if (P.G <= 64) {
        // every wavefront finds the minimum for itself: no barrier
        const int q = tid & 63;
        if (q < P.G) {
            const int ds = P.dead_step[q];
            double v = 0.0;
#pragma unroll
            for (int e = 0; e < SCORE_PARTS; ++e) v += P.score[q * SCORE_PARTS + e];      // fixed order
            if (ds >= step) { best = v; p = q; }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const double so = __shfl_xor(best, o);
            const int io = __shfl_xor(p, o);
            if (better(so, io, best, p)) { best = so; p = io; }
        }
    } else {
        for (int q = tid; q < P.G; q += 256) {
            const int ds = P.dead_step[q];
            double v = 0.0;
#pragma unroll
            for (int e = 0; e < SCORE_PARTS; ++e) v += P.score[q * SCORE_PARTS + e];      // fixed order
            if (ds >= step && better(v, q, best, p)) { best = v; p = q; }
        }
        block_argmin<256>(best, p, sh_s, sh_i);
    }
    if (status != 0) return;
    if (p < 0) {                                   // nothing left to remove: the request was impossible
        if (blockIdx.x == 0 && tid == 0) *P.status = -(2 + step);
        return;
    }
    if (blockIdx.x == 0 && tid == 0) {
        P.order[step] = p;
        P.err[step] = best;
        P.dead_step[p] = step;
    }
    const int c0 = p * g;
    const double *B = P.Binv + (size_t)p * g * g;
    const int lane = tid & 63, wave = tid >> 6, q4 = lane >> 4, cl16 = lane & 15;
    double bload[GMAX / 4];
#pragma unroll
    for (int q = 0; q < GMAX / 4; ++q) {           // element mapping without divisions: column = lane (g <= 64)
        const int i = wave + 4 * q;
        bload[q] = (i < g && lane < g) ? B[i * g + lane] : 0.0;
    }
    bool b_stored = false;
    const int ncc = (d + G_COLS - 1) / G_COLS;
    const int n_h_tiles = ((d + G_ROWS - 1) / G_ROWS) * ncc;
    const int n_w_tiles = ((m + G_ROWS - 1) / G_ROWS) * ncc;
    for (int tile = blockIdx.x; tile < n_h_tiles + n_w_tiles; tile += gridDim.x) {
        const bool is_h = tile < n_h_tiles;
        const int tt = is_h ? tile : tile - n_h_tiles;
        const int i0 = (tt / ncc) * G_ROWS, jw = (tt % ncc) * G_COLS + 16 * G_CT * wave;     // this wavefront's columns
        const int rows = is_h ? d : m;
        double aload[G_ROWS / 4];
#pragma unroll
        for (int q = 0; q < G_ROWS / 4; ++q) {
            const int i = i0 + wave + 4 * q;
            aload[q] = 0.0;
            if (i < rows && lane < g) aload[q] = is_h ? P.Hd[(size_t)i * d + c0 + lane] : (double)P.W[(size_t)i * d + c0 + lane];
        }
        // The column tiles of this wavefront: which columns take part, and the old values of its elements
        // (element v of tile ct: row i0 + 4 v + q4, column jw + 16 ct + cl16), fetched ahead of the products.
        bool live[G_CT];
        double old[G_CT][4];
#pragma unroll
        for (int ct = 0; ct < G_CT; ++ct) {
            const int j = jw + 16 * ct + cl16;
            const int sj = (j < d) ? j / g : 0;
            live[ct] = (j < d) && sj != p && P.dead_step[sj] >= step;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = i0 + 4 * v + q4;
                old[ct][v] = 0.0;
                if (live[ct] && i < rows) old[ct][v] = is_h ? P.Hd[(size_t)i * d + j] : (double)P.W[(size_t)i * d + j];
            }
        }
        // the rows of the selected structure over this wavefront's columns: B operands of the second product
        double rv[G_CT][GMAX / 4];
#pragma unroll
        for (int ct = 0; ct < G_CT; ++ct) {
            const int j = jw + 16 * ct + cl16;
#pragma unroll
            for (int ks = 0; ks < GMAX / 4; ++ks) {
                const int bb = 4 * ks + q4;
                rv[ct][ks] = (live[ct] && bb < g) ? P.Hd[(size_t)(c0 + bb) * d + j] : 0.0;
            }
        }
        lds_barrier();                  // the previous tile's readers of As, Bs and Cs are done
        if (!b_stored) {
#pragma unroll
            for (int q = 0; q < GMAX / 4; ++q) Bs[wave + 4 * q][lane] = bload[q];
            b_stored = true;
        }
#pragma unroll
        for (int q = 0; q < G_ROWS / 4; ++q) As[wave + 4 * q][lane] = aload[q];
        lds_barrier();
        // C = A B, 16 x 64: wavefront w forms columns 16 w .. 16 w + 15 (lane supplies A[row cl16][k q4] and
        // B[k q4][col cl16] of each k group of four; accumulator v is C[row 4 v + q4][col cl16])
        {
            doublex4 c = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
            for (int ks = 0; ks < GMAX / 4; ++ks)
                c = __builtin_amdgcn_mfma_f64_16x16x4f64(As[cl16][4 * ks + q4], Bs[4 * ks + q4][16 * wave + cl16], c, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 4; ++v) Cs[4 * v + q4][16 * wave + cl16] = c[v];
        }
        lds_barrier();
        // acc = C R with R = Hd[S, columns]: sixteen k groups, the A operand shared by the column tiles
        double ca[GMAX / 4];
#pragma unroll
        for (int ks = 0; ks < GMAX / 4; ++ks) ca[ks] = Cs[cl16][4 * ks + q4];
        doublex4 acc[G_CT];
#pragma unroll
        for (int ct = 0; ct < G_CT; ++ct) {
            acc[ct] = doublex4{0.0, 0.0, 0.0, 0.0};
#pragma unroll
            for (int ks = 0; ks < GMAX / 4; ++ks)
                acc[ct] = __builtin_amdgcn_mfma_f64_16x16x4f64(ca[ks], rv[ct][ks], acc[ct], 0, 0, 0);
        }
#pragma unroll
        for (int ct = 0; ct < G_CT; ++ct) {
            if (!live[ct]) continue;
            const int j = jw + 16 * ct + cl16;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = i0 + 4 * v + q4;
                if (i >= rows) continue;
                if (is_h) {
                    const int si = i / g;
                    if (si == p || P.dead_step[si] < step) continue;
                    P.Hd[(size_t)i * d + j] = old[ct][v] - acc[ct][v];
                } else {
                    P.W[(size_t)i * d + j] = (float)(old[ct][v] - acc[ct][v]);
                }
            }
        }
    }
}

__global__ __launch_bounds__(256) void group_snapshot_kernel(PruneState P, BatchShift B, int removed) {
    P = layer_state(P, B, blockIdx.y);
    snapshot_copy(P, removed, blockIdx.x * 256 + threadIdx.x, gridDim.x * 256);
}

__global__ __launch_bounds__(256) void group_final_kernel(PruneState P, BatchShift B) {
    P = layer_state(P, B, blockIdx.y);
    const int gtid = blockIdx.x * 256 + threadIdx.x, gthreads = gridDim.x * 256;
    const int d = P.d, g = P.g;
    const size_t totalw = (size_t)P.m * d;
    for (size_t idx = gtid; idx < totalw; idx += gthreads)
        if (P.dead_step[(idx % d) / g] != kNever) P.W[idx] = 0.f;
    const size_t total = (size_t)d * d;
    for (size_t idx = gtid; idx < total; idx += gthreads) {
        const int i = (int)(idx / d), j = (int)(idx % d);
        P.Hinv[idx] = (P.dead_step[i / g] == kNever && P.dead_step[j / g] == kNever) ? (float)P.Hd[idx] : 0.f;
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
struct PruneLayout {
    PruneState st;
    int *snap_of_step;
    int *snap_next;
    size_t bytes;
};

static PruneLayout prune_layout(int d_row, int d_col, int g, int n_snap, void *ws) {
    PruneLayout l = {};
    PruneState &s = l.st;
    s.m = d_row; s.d = d_col; s.g = g; s.G = d_col / g;
    s.nrc = (d_row + W_ROWS - 1) / W_ROWS;
    s.ncc = (d_col + PT - 1) / PT;
    Carver c(ws);
    s.Hd = c.take<double>((size_t)d_col * d_col);
    s.alive = c.take<uint8_t>((size_t)s.G);
    s.bar = c.take<unsigned>(1);
    s.status = c.take<int>(1);
    l.snap_of_step = c.take<int>((size_t)s.G + 1);
    l.snap_next = c.take<int>((size_t)(n_snap > 0 ? n_snap : 1));
    if (g == 1) {
        s.Pn = c.take<double>((size_t)s.nrc * d_col);
        s.diag = c.take<double>((size_t)d_col);
        s.cand_score = c.take<double>((size_t)s.ncc);
        s.cand_idx = c.take<int>((size_t)s.ncc);
    } else {
        s.score = c.take<double>((size_t)s.G * SCORE_PARTS);
        s.Binv = c.take<double>((size_t)s.G * g * g);
        s.dead_step = c.take<int>((size_t)s.G);
    }
    l.bytes = c.off;
    return l;
}

// Uploads the snapshot schedule (first snapshot per step + chain of further ones at the same step) into the
// tables of `l` and points P at them.  The sources are pageable: the copies have staged them when this returns.
static int upload_snapshot_schedule(PruneLayout &l, PruneState &P, int G, int n_snap, const int32_t *steps_host,
                                    hipStream_t st) {
    if (n_snap <= 0) {
        P.snap_of_step = nullptr;
        P.snap_next = nullptr;
        return ZIPLM_OK;
    }
    int *of_step = new int[(size_t)G + 1];
    int *next = new int[(size_t)n_snap];
    for (int t = 0; t <= G; ++t) of_step[t] = -1;
    for (int q = n_snap - 1; q >= 0; --q) {
        next[q] = of_step[steps_host[q]];
        of_step[steps_host[q]] = q;
    }
    hipError_t e1 = hipMemcpyAsync(l.snap_of_step, of_step, sizeof(int) * ((size_t)G + 1), hipMemcpyHostToDevice, st);
    hipError_t e2 = hipMemcpyAsync(l.snap_next, next, sizeof(int) * (size_t)n_snap, hipMemcpyHostToDevice, st);
    hipError_t e3 = hipStreamSynchronize(st);
    delete[] of_step;
    delete[] next;
    if (e1 != hipSuccess || e2 != hipSuccess || e3 != hipSuccess) return ZIPLM_ERR_DEVICE;
    P.snap_of_step = l.snap_of_step;
    P.snap_next = l.snap_next;
    return ZIPLM_OK;
}

// The launch sequence of the group path for `layers` layers at once (grid dimension y).
static int launch_group_steps(const PruneState &P, const BatchShift &B, int layers, int n_remove, int n_snap,
                              hipStream_t st) {
    const int fill = 1024;
    const int ncc = (P.d + G_COLS - 1) / G_COLS;
    const int tiles = ((P.d + G_ROWS - 1) / G_ROWS + (P.m + G_ROWS - 1) / G_ROWS) * ncc;
    hipLaunchKernelGGL(group_init_kernel, dim3(fill, layers), dim3(256), 0, st, P, B);
    for (int t = 0; t < n_remove; ++t) {
        if (n_snap > 0) hipLaunchKernelGGL(group_snapshot_kernel, dim3(fill, layers), dim3(256), 0, st, P, B, t);
        hipLaunchKernelGGL(group_score_kernel, dim3(P.G, SCORE_PARTS, layers), dim3(256), 0, st, P, B, t);
        hipLaunchKernelGGL(group_update_kernel, dim3(tiles, layers), dim3(256), 0, st, P, B, t);
    }
    if (n_snap > 0) hipLaunchKernelGGL(group_snapshot_kernel, dim3(fill, layers), dim3(256), 0, st, P, B, n_remove);
    hipLaunchKernelGGL(group_final_kernel, dim3(fill, layers), dim3(256), 0, st, P, B);
    ZIPLM_HIP_TRY(hipGetLastError());
    return ZIPLM_OK;
}

}  // namespace ziplm

namespace ziplm {

// Arguments shared by the single-layer entry points, validated before anything is enqueued.
static int check_prune_args(const float *W, const float *Hinv, int d_row, int d_col, int group_size, int n_remove,
                            const int32_t *order_out, const double *err_out, int n_snap,
                            const int32_t *snapshot_steps_host, const float *W_snap) {
    if (!W || !Hinv || d_row <= 0 || d_col <= 0 || group_size <= 0 || d_col % group_size) return ZIPLM_ERR_INVALID_ARG;
    const int G = d_col / group_size;
    if (n_remove < 0 || n_remove > G) return ZIPLM_ERR_INVALID_ARG;
    if (n_remove > 0 && (!order_out || !err_out)) return ZIPLM_ERR_INVALID_ARG;
    if (n_snap < 0 || (n_snap > 0 && (!snapshot_steps_host || !W_snap))) return ZIPLM_ERR_INVALID_ARG;
    for (int q = 0; q < n_snap; ++q)
        if (snapshot_steps_host[q] < 0 || snapshot_steps_host[q] > n_remove) return ZIPLM_ERR_INVALID_ARG;
    if (group_size > GMAX) return ZIPLM_ERR_UNSUPPORTED;
    return ZIPLM_OK;
}

static int report_status(const int *status_dev, int *info_host, hipStream_t st) {
    if (!info_host) return ZIPLM_OK;
    int status = 0;
    ZIPLM_HIP_TRY(hipStreamSynchronize(st));
    ZIPLM_HIP_TRY(hipMemcpy(&status, status_dev, sizeof(int), hipMemcpyDeviceToHost));
    *info_host = status;
    return status_to_return_code(status);
}

// Eager single-column kernel and the two-launch group path on a validated request.
static int launch_eager_or_groups(float *W, float *Hinv, int d_row, int d_col, int group_size, int n_remove,
                                  int32_t *order_out, double *err_out, const uint8_t *alive_in, int n_snap,
                                  const int32_t *snapshot_steps_host, float *W_snap, int *info_host, void *workspace,
                                  hipStream_t st) {
    const int G = d_col / group_size;
    PruneLayout l = prune_layout(d_row, d_col, group_size, n_snap, workspace);
    PruneState &P = l.st;
    P.W = W; P.Hinv = Hinv; P.n_remove = n_remove;
    P.order = order_out; P.err = err_out; P.alive_in = alive_in; P.W_snap = W_snap;
    {
        const int rc = upload_snapshot_schedule(l, P, G, n_snap, snapshot_steps_host, st);
        if (rc != ZIPLM_OK) return rc;
    }
    // bar and status are adjacent 256-byte slots
    if (zero_fill(P.bar, 2 * kAlign, st) != ZIPLM_OK) return ZIPLM_ERR_DEVICE;
    // the device counts removals against the structures that are alive; a request for more than that shows up
    // as "no candidate" -> status = -(2 + step)
    if (group_size == 1) {
        int per_cu = 0;
        ZIPLM_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, prune_columns_kernel, PT, 0));
        if (per_cu < 1) return ZIPLM_ERR_DEVICE;
        const int nblocks = device_cu_count();   // one workgroup per compute unit keeps the barrier short
        void *args[] = {&P};
        ZIPLM_HIP_TRY(hipLaunchCooperativeKernel(reinterpret_cast<void *>(prune_columns_kernel), dim3(nblocks),
                                                 dim3(PT), args, 0, st));
    } else {
        const BatchShift none = {};
        const int rc = launch_group_steps(P, none, 1, n_remove, n_snap, st);
        if (rc != ZIPLM_OK) return rc;
    }
    return report_status(P.status, info_host, st);
}

}  // namespace ziplm

extern "C" size_t ziplm_prune_workspace_bytes(int d_row, int d_col, int group_size, int n_snap) {
    if (d_row <= 0 || d_col <= 0 || group_size <= 0 || d_col % group_size) return 0;
    if (group_size == 1 && ziplm::use_lazy_columns(d_row, d_col))
        return ziplm::lazy_columns_workspace_bytes(d_row, d_col, n_snap);
    return ziplm::prune_layout(d_row, d_col, group_size, n_snap, nullptr).bytes;
}

extern "C" size_t ziplm_prune_exchange_bytes(int n_layers, int d_row, int d_col, int group_size) {
    if (n_layers <= 0 || d_row <= 0 || d_col <= 0 || group_size != 1 || !ziplm::use_lazy_columns(d_row, d_col)) return 0;
    size_t need = 0;
    for (int done = 0; done < n_layers;) {
        const int pack = ziplm::lazy_columns_pack(n_layers - done, d_row, d_col);
        const size_t b = ziplm::lazy_columns_pack_exchange_bytes(pack, d_row, d_col);
        need = b > need ? b : need;
        done += pack;
    }
    return need;
}

extern "C" int ziplm_exchange_alloc(size_t bytes, void **exchange_out) {
    if (!exchange_out || bytes == 0) return ZIPLM_ERR_INVALID_ARG;
    *exchange_out = nullptr;
    void *q = nullptr;
    if (hipExtMallocWithFlags(&q, ziplm::align_up(bytes), hipDeviceMallocUncached) != hipSuccess) {
        (void)hipGetLastError();
        return ZIPLM_ERR_DEVICE;
    }
    *exchange_out = q;
    return ZIPLM_OK;
}

// exchange == NULL: the slots and payloads live in the workspace.  Otherwise it must be aligned and large enough.
static int check_exchange(const void *exchange, size_t exchange_bytes, size_t need) {
    if (!exchange) return ZIPLM_OK;
    return ziplm::workspace_ok(exchange, exchange_bytes, need) ? ZIPLM_OK : ZIPLM_ERR_WORKSPACE;
}

extern "C" int ziplm_structured_obs_prune(float *W, float *Hinv, int d_row, int d_col, int group_size,
                                          int n_remove, int32_t *order_out, double *err_out,
                                          const uint8_t *alive_in, int n_snap,
                                          const int32_t *snapshot_steps_host, float *W_snap, int *info_host,
                                          void *exchange, size_t exchange_bytes,
                                          void *workspace, size_t workspace_bytes, void *stream) {
    using namespace ziplm;
    const int bad = check_prune_args(W, Hinv, d_row, d_col, group_size, n_remove, order_out, err_out, n_snap,
                                     snapshot_steps_host, W_snap);
    if (bad != ZIPLM_OK) return bad;
    const size_t need = ziplm_prune_workspace_bytes(d_row, d_col, group_size, n_snap);
    if (!workspace_ok(workspace, workspace_bytes, need)) return ZIPLM_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);

    if (group_size == 1 && use_lazy_columns(d_row, d_col)) {
        if (check_exchange(exchange, exchange_bytes, lazy_columns_pack_exchange_bytes(1, d_row, d_col)) != ZIPLM_OK)
            return ZIPLM_ERR_WORKSPACE;
        int *status_dev = nullptr;
        const int rc = lazy_columns_launch(W, Hinv, 1, 0, 0, d_row, d_col, n_remove, order_out, err_out, alive_in,
                                           n_snap, snapshot_steps_host, W_snap, workspace, exchange, st, &status_dev, -1);
        if (rc != ZIPLM_OK) return rc;
        return report_status(status_dev, info_host, st);
    }
    return launch_eager_or_groups(W, Hinv, d_row, d_col, group_size, n_remove, order_out, err_out, alive_in, n_snap,
                                  snapshot_steps_host, W_snap, info_host, workspace, st);
}

extern "C" size_t ziplm_prune_eager_workspace_bytes(int d_row, int d_col, int n_snap) {
    if (d_row <= 0 || d_col <= 0) return 0;
    return ziplm::prune_layout(d_row, d_col, 1, n_snap, nullptr).bytes;
}

extern "C" int ziplm_structured_obs_prune_eager(float *W, float *Hinv, int d_row, int d_col, int n_remove,
                                                int32_t *order_out, double *err_out, const uint8_t *alive_in,
                                                int n_snap, const int32_t *snapshot_steps_host, float *W_snap,
                                                int *info_host, void *workspace, size_t workspace_bytes,
                                                void *stream) {
    using namespace ziplm;
    const int bad = check_prune_args(W, Hinv, d_row, d_col, 1, n_remove, order_out, err_out, n_snap,
                                     snapshot_steps_host, W_snap);
    if (bad != ZIPLM_OK) return bad;
    if (!workspace_ok(workspace, workspace_bytes, ziplm_prune_eager_workspace_bytes(d_row, d_col, n_snap)))
        return ZIPLM_ERR_WORKSPACE;
    return launch_eager_or_groups(W, Hinv, d_row, d_col, 1, n_remove, order_out, err_out, alive_in, n_snap,
                                  snapshot_steps_host, W_snap, info_host, workspace, static_cast<hipStream_t>(stream));
}

extern "C" int ziplm_selftest_bounded_wait(float *W, float *Hinv, int d_row, int d_col, int32_t *order_out,
                                           double *err_out, int *info_host, void *workspace,
                                           size_t workspace_bytes, void *stream) {
    using namespace ziplm;
    const int bad = check_prune_args(W, Hinv, d_row, d_col, 1, d_col, order_out, err_out, 0, nullptr, nullptr);
    if (bad != ZIPLM_OK) return bad;
    if (!info_host) return ZIPLM_ERR_INVALID_ARG;
    if (!use_lazy_columns(d_row, d_col)) return ZIPLM_ERR_UNSUPPORTED;
    if (!workspace_ok(workspace, workspace_bytes, ziplm_prune_workspace_bytes(d_row, d_col, 1, 0))) return ZIPLM_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int *status_dev = nullptr;
    const int rc = lazy_columns_launch(W, Hinv, 1, 0, 0, d_row, d_col, d_col, order_out, err_out, nullptr, 0, nullptr,
                                       nullptr, workspace, nullptr, st, &status_dev, 0);
    if (rc != ZIPLM_OK) return rc;
    return report_status(status_dev, info_host, st);
}

extern "C" size_t ziplm_prune_batch_workspace_bytes(int n_layers, int d_row, int d_col, int group_size, int n_snap) {
    if (n_layers <= 0 || d_row <= 0 || d_col <= 0 || group_size < 1 || group_size > ziplm::GMAX || d_col % group_size) return 0;
    if (group_size == 1) {
        // single columns: the launches of a batch run one after the other and share the workspace
        if (!ziplm::use_lazy_columns(d_row, d_col)) return ziplm_prune_workspace_bytes(d_row, d_col, 1, n_snap);
        size_t need = 0;
        for (int done = 0; done < n_layers;) {
            const int pack = ziplm::lazy_columns_pack(n_layers - done, d_row, d_col);
            const size_t b = ziplm::lazy_columns_pack_workspace_bytes(pack, d_row, d_col, n_snap);
            need = b > need ? b : need;
            done += pack;
        }
        return need;
    }
    return (size_t)n_layers * ziplm::prune_layout(d_row, d_col, group_size, n_snap, nullptr).bytes;
}

extern "C" int ziplm_structured_obs_prune_batch(float *W, float *Hinv, int n_layers, int64_t stride_w,
                                                int64_t stride_hinv, int d_row, int d_col, int group_size,
                                                int n_remove, int32_t *order_out, double *err_out, int n_snap,
                                                const int32_t *snapshot_steps_host, float *W_snap, int *info_host,
                                                void *exchange, size_t exchange_bytes,
                                                void *workspace, size_t workspace_bytes, void *stream) {
    using namespace ziplm;
    if (n_layers <= 0) return ZIPLM_ERR_INVALID_ARG;
    const int bad = check_prune_args(W, Hinv, d_row, d_col, group_size, n_remove, order_out, err_out, n_snap,
                                     snapshot_steps_host, W_snap);
    if (bad != ZIPLM_OK) return bad;
    if (stride_w < (int64_t)d_row * d_col || stride_hinv < (int64_t)d_col * d_col) return ZIPLM_ERR_INVALID_ARG;
    const int G = d_col / group_size;
    const size_t need = ziplm_prune_batch_workspace_bytes(n_layers, d_row, d_col, group_size, n_snap);
    if (!workspace_ok(workspace, workspace_bytes, need)) return ZIPLM_ERR_WORKSPACE;
    if (check_exchange(exchange, exchange_bytes, ziplm_prune_exchange_bytes(n_layers, d_row, d_col, group_size)) != ZIPLM_OK)
        return ZIPLM_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);

    // the worst status over the layers: a device failure outranks an impossible request outranks a bad pivot
    auto worse = [](int a, int b) {
        auto rank = [](int rc) { return rc == ZIPLM_ERR_DEVICE ? 3 : rc == ZIPLM_ERR_INVALID_ARG ? 2 : rc == ZIPLM_ERR_NOT_PD ? 1 : 0; };
        return rank(b) > rank(a) ? b : a;
    };

    if (group_size == 1) {
        // Single columns: a few layers per launch, each on its share of the compute units; the launches follow
        // one another on the stream and reuse the workspace.
        int worst = ZIPLM_OK;
        const size_t snap_stride = (size_t)n_snap * d_row * d_col;
        for (int done = 0; done < n_layers;) {
            float *Wl = W + (size_t)done * stride_w, *Hl = Hinv + (size_t)done * stride_hinv;
            int32_t *ol = order_out ? order_out + (size_t)done * n_remove : nullptr;
            double *el = err_out ? err_out + (size_t)done * n_remove : nullptr;
            float *sl = W_snap ? W_snap + (size_t)done * snap_stride : nullptr;
            if (!use_lazy_columns(d_row, d_col)) {
                const int rc = launch_eager_or_groups(Wl, Hl, d_row, d_col, 1, n_remove, ol, el, nullptr, n_snap,
                                                      snapshot_steps_host, sl, info_host ? info_host + done : nullptr,
                                                      workspace, st);
                if (rc != ZIPLM_OK && rc != ZIPLM_ERR_NOT_PD && rc != ZIPLM_ERR_DEVICE && rc != ZIPLM_ERR_INVALID_ARG) return rc;
                worst = worse(worst, rc);
                done += 1;
                continue;
            }
            const int pack = lazy_columns_pack(n_layers - done, d_row, d_col);
            int *status_dev[16] = {};
            const int rc = lazy_columns_launch(Wl, Hl, pack, stride_w, stride_hinv, d_row, d_col, n_remove, ol, el, nullptr,
                                               n_snap, snapshot_steps_host, sl, workspace, exchange, st, status_dev, -1);
            if (rc != ZIPLM_OK) return rc;
            if (info_host) {
                // the next launch reuses the status words
                ZIPLM_HIP_TRY(hipStreamSynchronize(st));
                for (int q = 0; q < pack; ++q) {
                    int status = 0;
                    ZIPLM_HIP_TRY(hipMemcpy(&status, status_dev[q], sizeof(int), hipMemcpyDeviceToHost));
                    info_host[done + q] = status;
                    worst = worse(worst, status_to_return_code(status));
                }
            }
            done += pack;
        }
        return worst;
    }

    PruneLayout l = prune_layout(d_row, d_col, group_size, n_snap, workspace);
    PruneState &P = l.st;
    P.W = W; P.Hinv = Hinv; P.n_remove = n_remove;
    P.order = order_out; P.err = err_out; P.alive_in = nullptr; P.W_snap = W_snap;
    BatchShift B = {};
    B.ws_bytes = l.bytes;
    B.w = stride_w; B.hinv = stride_hinv; B.order = n_remove; B.err = n_remove;
    B.snap = (long long)n_snap * d_row * d_col;
    {
        const int rc = upload_snapshot_schedule(l, P, G, n_snap, snapshot_steps_host, st);
        if (rc != ZIPLM_OK) return rc;
    }
    for (int q = 0; q < n_layers; ++q)     // bar and status of every layer
        if (zero_fill(reinterpret_cast<char *>(P.bar) + (size_t)q * l.bytes, 2 * kAlign, st) != ZIPLM_OK) return ZIPLM_ERR_DEVICE;
    {
        const int rc = launch_group_steps(P, B, n_layers, n_remove, n_snap, st);
        if (rc != ZIPLM_OK) return rc;
    }
    if (info_host) {
        ZIPLM_HIP_TRY(hipStreamSynchronize(st));
        int worst = ZIPLM_OK;
        for (int q = 0; q < n_layers; ++q) {
            int status = 0;
            ZIPLM_HIP_TRY(hipMemcpy(&status, reinterpret_cast<char *>(P.status) + (size_t)q * l.bytes, sizeof(int),
                                    hipMemcpyDeviceToHost));
            info_host[q] = status;
            worst = worse(worst, status_to_return_code(status));
        }
        return worst;
    }
    return ZIPLM_OK;
}
