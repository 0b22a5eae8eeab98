// Greedy structured OBS pruning for single-column structures (Algorithm 1 with |S| = 1), fast path.
//
// Mathematically this is the same sequence as the eager loop: at step t the column with the smallest
// Eq. 2 score  ||W[:,j]||^2 / Hinv[j][j]  is removed, W is compensated (Eq. 3) and the column is
// eliminated from the inverse Hessian (Eq. 4).  What differs is when the O(r^2) elimination is
// applied to memory:
//
//   * Eq. 4 is a rank-1 downdate  Hinv -= u u^T / u[p]  with u = the current row p.  The next step
//     only needs (a) the current diagonal, which each owner keeps up to date from u alone, and (b) the
//     current row of the next pivot, which is  stale_row - sum_k u_k[p'] u_k / piv_k  over the
//     downdates not yet applied.  So the downdates of up to 64 consecutive steps are kept as a list
//     of pivot rows and applied to the stored matrix in one pass ("flush").  The stored fp64 matrix
//     is then read and written once per 64 steps instead of once per step.
//   * W is compensated at every step (Eq. 3 needs no deferral: the scores need the current W).
//
// Work is divided by columns: workgroup b owns `cpb` consecutive columns j, i.e. column j of W (kept
// transposed as a row of `wt`, in LDS when it fits), row j of the fp64 inverse Hessian, its diagonal
// entry, squared norm and score.  One wavefront works on one owned column at a time.  Per step:
//
//   1. every workgroup publishes its best owned column (score, index) and, speculatively, what the
//      others would need if it wins: that column of W, the entries u_k[p] of the pending pivot rows
//      and the current diagonal entry.  All of it is written as 64-bit words carrying 32 bits of
//      data and a 32-bit step tag, so readers can tell a fresh word from an old one without any
//      ordering between stores ("flag in data"); buffers alternate with the step parity.
//   2. every workgroup reads all candidates, takes the argmin (lowest index on ties), reads the
//      winner's payload, forms its slice of the current pivot row, updates its diagonal entries,
//      compensates its columns of W and refreshes their norms and scores.
//
// One exchange per step is the only device-wide synchronisation; every 64 steps one barrier
// precedes the flush.  All waits are bounded: on a time-out the waiter raises status = -1 and
// leaves; the others then time out or see the flag, and the grid drains.
#include "common.h"

namespace ziplm {

int device_cu_count();

namespace lazy {

constexpr int LT = 1024;                 // threads per workgroup (16 wavefronts)
constexpr int NW = LT / 64;
constexpr int BMAX = 64;                 // pending pivot rows between flushes (one lane per row)
constexpr int ROWS_PER_PASS = 16;        // owned rows updated per sweep over the pending rows in a flush
constexpr unsigned long long kTimeoutTicks = 400000000ull;   // 4 s of the 100 MHz wall clock
constexpr int IDX_NONE = -1;             // workgroup has no live column
constexpr int IDX_ERROR = 0x7ffffff0;    // workgroup met a non-positive diagonal entry
constexpr int SLOT_WORDS = 4;

struct State {
    // caller's buffers
    float *W;
    float *Hinv;
    int m, d, n_remove;
    int32_t *order;
    double *err;
    const uint8_t *alive_in;
    // snapshots
    int n_snap;
    const int *snap_steps;   // device copy of the caller's list
    float *W_snap;
    // workspace
    double *Hd;                   // [d][d]   stored (stale between flushes) inverse Hessian
    float *Wt;                    // [d][m]   transposed W when it does not fit LDS, else unused
    double *U;                    // [2][BMAX][d] pending pivot rows of the current / previous block
    unsigned long long *slots;    // [2][nb][SLOT_WORDS]
    unsigned long long *pay;      // [2][nb][pay_words]
    unsigned long long *bar;      // [nb] flush-barrier epochs
    int *status;
    int cpb;                      // columns per workgroup
    int w_in_lds;
    int pay_words;                // m + 2*BMAX + 2
};

__device__ __forceinline__ unsigned long long ll_pack(unsigned data, unsigned tag) {
    return ((unsigned long long)data << 32) | tag;
}
__device__ __forceinline__ void ll_store(unsigned long long *p, unsigned data, unsigned tag) {
    __hip_atomic_store(p, ll_pack(data, tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Spins until the word carries `tag`; returns false on time-out or when another waiter gave up.
__device__ __forceinline__ bool ll_wait(const unsigned long long *p, unsigned tag, unsigned &data, int *status) {
    unsigned spins = 0;
    unsigned long long t0 = 0;
    for (;;) {
        const unsigned long long v = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((unsigned)(v & 0xffffffffu) == tag) { data = (unsigned)(v >> 32); return true; }
        if ((++spins & 255u) == 0u) {
            if (t0 == 0) t0 = wall_clock64();
            if (__hip_atomic_load(status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == -1) return false;
            if (wall_clock64() - t0 > kTimeoutTicks) {
                __hip_atomic_store(status, -1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                return false;
            }
        }
    }
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

__device__ __forceinline__ bool better(double s1, int i1, double s2, int i2) {
    if (i2 < 0) return i1 >= 0;
    if (i1 < 0) return false;
    return (s1 < s2) || (s1 == s2 && i1 < i2);
}

__device__ __forceinline__ unsigned dhi(double x) { return (unsigned)((unsigned long long)__double_as_longlong(x) >> 32); }
__device__ __forceinline__ unsigned dlo(double x) { return (unsigned)((unsigned long long)__double_as_longlong(x) & 0xffffffffu); }
__device__ __forceinline__ double dmake(unsigned hi, unsigned lo) {
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

// LDS carve-up (byte offsets), identical on host and device.
struct Lds {
    size_t uloc, coef, hist, pivs, wcol, norm, diag, score, hstale, alive_own, alive_bits, snap_bits, red_s, red_i, misc, wt, total;
};
__host__ __device__ inline Lds lds_layout(int m, int d, int cpb, bool w_in_lds) {
    Lds l;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t r = o; o += (bytes + 15) / 16 * 16; return r; };
    l.uloc = take(sizeof(double) * BMAX * cpb);          // pending pivot rows, owned slice: [k][jl]
    l.coef = take(sizeof(double) * BMAX * ROWS_PER_PASS);// flush coefficients of one pass: [k][row]
    l.hist = take(sizeof(double) * BMAX);                // u_k[p] of the current pivot
    l.pivs = take(sizeof(double) * BMAX);                // pivots of the pending rows
    l.wcol = take(sizeof(float) * m);                    // column p of W
    l.norm = take(sizeof(double) * cpb);
    l.diag = take(sizeof(double) * cpb);
    l.score = take(sizeof(double) * cpb);
    l.hstale = take(sizeof(double) * cpb);
    l.alive_own = take(sizeof(int) * cpb);
    l.alive_bits = take(sizeof(unsigned) * ((d + 31) / 32));
    l.snap_bits = take(sizeof(unsigned) * ((d + 32) / 32 + 1));
    l.red_s = take(sizeof(double) * NW);
    l.red_i = take(sizeof(int) * NW);
    l.misc = take(96);
    l.wt = take(w_in_lds ? sizeof(float) * (size_t)cpb * m : 0);
    l.total = o;
    return l;
}

__global__ __launch_bounds__(LT) void prune_lazy_kernel(State S) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int b = blockIdx.x, nb = gridDim.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = S.m, d = S.d, cpb = S.cpb;
    const Lds L = lds_layout(m, d, cpb, S.w_in_lds != 0);
    double *uloc = reinterpret_cast<double *>(smem + L.uloc);
    double *coef = reinterpret_cast<double *>(smem + L.coef);
    double *hist = reinterpret_cast<double *>(smem + L.hist);
    double *pivs = reinterpret_cast<double *>(smem + L.pivs);
    float *wcol = reinterpret_cast<float *>(smem + L.wcol);
    double *norm = reinterpret_cast<double *>(smem + L.norm);
    double *diag = reinterpret_cast<double *>(smem + L.diag);
    double *score = reinterpret_cast<double *>(smem + L.score);
    double *hstale = reinterpret_cast<double *>(smem + L.hstale);
    int *alive_own = reinterpret_cast<int *>(smem + L.alive_own);
    unsigned *alive_bits = reinterpret_cast<unsigned *>(smem + L.alive_bits);
    double *red_s = reinterpret_cast<double *>(smem + L.red_s);
    int *red_i = reinterpret_cast<int *>(smem + L.red_i);
    unsigned *snap_bits = reinterpret_cast<unsigned *>(smem + L.snap_bits);
    int *misc = reinterpret_cast<int *>(smem + L.misc);   // [0] fail flag, [1] winner, [2] error seen, [3] local candidate
    double *misc_d = reinterpret_cast<double *>(smem + L.misc + 32);  // [0] best score, [1] pivot

    const int j0 = b * cpb;
    const int nown = max(0, min(cpb, d - j0));
    // generic pointer: LDS or this workgroup's private rows of the transposed copy in global memory
    float *wt = S.w_in_lds ? reinterpret_cast<float *>(smem + L.wt) : (S.Wt + (size_t)j0 * m);

    // ------------------------------------------------------------------ set-up (own data only)
    for (int w = tid; w < (d + 31) / 32; w += LT) {
        unsigned bits = 0;
        for (int e = 0; e < 32; ++e) {
            const int c = w * 32 + e;
            if (c < d && (S.alive_in ? S.alive_in[c] != 0 : true)) bits |= 1u << e;
        }
        alive_bits[w] = bits;
    }
    if (tid == 0) { misc[0] = 0; misc[2] = 0; }
    for (int w = tid; w < (d + 32) / 32 + 1; w += LT) snap_bits[w] = 0;
    __syncthreads();
    for (int q = tid; q < S.n_snap; q += LT) {
        const int sstep = S.snap_steps[q];
        atomicOr(&snap_bits[sstep >> 5], 1u << (sstep & 31));
    }
    for (int jl = 0; jl < nown; ++jl) {
        const size_t row = (size_t)(j0 + jl) * d;
        for (int c = tid; c < d; c += LT) S.Hd[row + c] = (double)S.Hinv[row + c];
    }
    for (int jl = wave; jl < nown; jl += NW) {
        const int j = j0 + jl;
        double s = 0.0;
        for (int i = lane; i < m; i += 64) {
            const float w = S.W[(size_t)i * d + j];
            wt[(size_t)jl * m + i] = w;
            s += (double)w * (double)w;
        }
        s = wave_sum(s);
        if (lane == 0) {
            const double dj = (double)S.Hinv[(size_t)j * d + j];
            const int alive = S.alive_in ? (S.alive_in[j] != 0) : 1;
            norm[jl] = s;
            diag[jl] = dj;
            alive_own[jl] = alive;
            score[jl] = s / dj;
        }
    }
    __syncthreads();

    unsigned long long bar_epoch = 0;
    int k = 0;          // pending pivot rows
    int ublk = 0;       // which half of U the current block of steps writes
    int t = 0;
    bool ok = true;
    int error_step = 0;

    for (; t <= S.n_remove; ++t) {
        // -------------------------------------------------------------- snapshots after t removals
        for (int q = 0; ((snap_bits[t >> 5] >> (t & 31)) & 1u) && q < S.n_snap; ++q) {
            if (S.snap_steps[q] != t) continue;      // uniform
            float *dst = S.W_snap + (size_t)q * m * d;
            for (int jl = wave; jl < nown; jl += NW) {
                const bool a = alive_own[jl] != 0;
                for (int i = lane; i < m; i += 64) dst[(size_t)i * d + j0 + jl] = a ? wt[(size_t)jl * m + i] : 0.f;
            }
        }
        if (t == S.n_remove) break;

        const unsigned tag = (unsigned)(t + 1);
        const int par = t & 1;

        // ---------------------------------------------------------- 1. local candidate + publish
        if (wave == 0) {
            double bs = 0.0;
            int bi = IDX_NONE;
            bool bad = false;
            for (int jl = lane; jl < nown; jl += 64) {
                if (!alive_own[jl]) continue;
                if (!(diag[jl] > 0.0)) { bad = true; continue; }
                if (better(score[jl], j0 + jl, bs, bi)) { bs = score[jl]; bi = j0 + jl; }
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                const double so = __shfl_xor(bs, o);
                const int io = __shfl_xor(bi, o);
                if (better(so, io, bs, bi)) { bs = so; bi = io; }
            }
            bad = __any(bad);
            if (lane == 0) {
                if (bad) bi = IDX_ERROR;
                misc[3] = bi;
                unsigned long long *slot = S.slots + ((size_t)par * nb + b) * SLOT_WORDS;
                ll_store(slot + 0, dhi(bs), tag);
                ll_store(slot + 1, dlo(bs), tag);
                ll_store(slot + 2, (unsigned)bi, tag);
            }
        }
        __syncthreads();
        {
            const int cand = misc[3];
            if (cand >= 0 && cand != IDX_ERROR) {
                const int cl = cand - j0;
                unsigned long long *pw = S.pay + ((size_t)par * nb + b) * S.pay_words;
                for (int i = tid; i < m; i += LT) ll_store(pw + i, __float_as_uint(wt[(size_t)cl * m + i]), tag);
                if (tid < k) {
                    const double u = uloc[tid * cpb + cl];
                    ll_store(pw + m + 2 * tid, dhi(u), tag);
                    ll_store(pw + m + 2 * tid + 1, dlo(u), tag);
                }
                if (tid == BMAX) {
                    const double dv = diag[cl];
                    ll_store(pw + m + 2 * BMAX, dhi(dv), tag);
                    ll_store(pw + m + 2 * BMAX + 1, dlo(dv), tag);
                }
            }
        }

        // ---------------------------------------------------------- 2. all candidates -> argmin
        {
            double s = 0.0;
            int idx = IDX_NONE;
            bool fail = false, err = false;
            for (int sb = tid; sb < nb; sb += LT) {
                const unsigned long long *slot = S.slots + ((size_t)par * nb + sb) * SLOT_WORDS;
                unsigned hi, lo, ix;
                if (!ll_wait(slot + 0, tag, hi, S.status) || !ll_wait(slot + 1, tag, lo, S.status) ||
                    !ll_wait(slot + 2, tag, ix, S.status)) { fail = true; break; }
                if ((int)ix == IDX_ERROR) { err = true; continue; }
                const double sv = dmake(hi, lo);
                if (better(sv, (int)ix, s, idx)) { s = sv; idx = (int)ix; }
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                const double so = __shfl_xor(s, o);
                const int io = __shfl_xor(idx, o);
                if (better(so, io, s, idx)) { s = so; idx = io; }
            }
            if (lane == 0) { red_s[wave] = s; red_i[wave] = idx; }
            if (fail) misc[0] = 1;
            if (err) misc[2] = 1;
            __syncthreads();
            if (tid == 0) {
                double bs = red_s[0];
                int bi = red_i[0];
                for (int w = 1; w < NW; ++w)
                    if (better(red_s[w], red_i[w], bs, bi)) { bs = red_s[w]; bi = red_i[w]; }
                misc[1] = bi;
                misc_d[0] = bs;
            }
            __syncthreads();
        }
        if (misc[0]) { ok = false; break; }
        const int p = misc[1];
        if (misc[2] || p < 0) { error_step = 1 + t; break; }   // same inputs in every workgroup: uniform
        const double best = misc_d[0];
        const int owner = p / cpb;

        // ---------------------------------------------------------- 3. winner's payload + stale column p
        {
            const unsigned long long *pw = S.pay + ((size_t)par * nb + owner) * S.pay_words;
            bool fail = false;
            // own rows, column p of the stored matrix (symmetric: equals row p, columns owned here)
            if (tid < nown && alive_own[tid]) hstale[tid] = S.Hd[(size_t)(j0 + tid) * d + p];
            for (int i = tid; i < m; i += LT) {
                unsigned v;
                if (!ll_wait(pw + i, tag, v, S.status)) { fail = true; break; }
                wcol[i] = __uint_as_float(v);
            }
            if (tid < k) {
                unsigned hi, lo;
                if (!ll_wait(pw + m + 2 * tid, tag, hi, S.status) || !ll_wait(pw + m + 2 * tid + 1, tag, lo, S.status)) fail = true;
                else hist[tid] = dmake(hi, lo);
            }
            if (tid == BMAX) {
                unsigned hi, lo;
                if (!ll_wait(pw + m + 2 * BMAX, tag, hi, S.status) || !ll_wait(pw + m + 2 * BMAX + 1, tag, lo, S.status)) fail = true;
                else { misc_d[1] = dmake(hi, lo); pivs[k] = dmake(hi, lo); }
            }
            if (fail) misc[0] = 1;
            __syncthreads();
        }
        if (misc[0]) { ok = false; break; }
        const double piv = misc_d[1];
        if (b == 0 && tid == 0) { S.order[t] = p; S.err[t] = best; }
        if (tid == 0) alive_bits[p >> 5] &= ~(1u << (p & 31));

        // ---------------------------------------------------------- 4. own slice of the pivot row, Eq. 3
        for (int jl = wave; jl < nown; jl += NW) {
            if (!alive_own[jl]) continue;                       // wave-uniform
            const int j = j0 + jl;
            if (j == p) {
                if (lane == 0) alive_own[jl] = 0;
                continue;
            }
            double term = 0.0;
            if (lane < k) term = (hist[lane] / pivs[lane]) * uloc[lane * cpb + jl];
            const double u = hstale[jl] - wave_sum(term);
            const double f = u / piv;
            double s = 0.0;
            for (int i = lane; i < m; i += 64) {
                float *w = wt + (size_t)jl * m + i;
                const float v = (float)((double)(*w) - (double)wcol[i] * f);
                *w = v;
                s += (double)v * (double)v;
            }
            s = wave_sum(s);
            if (lane == 0) {
                uloc[k * cpb + jl] = u;
                __hip_atomic_store(S.U + ((size_t)ublk * BMAX + k) * d + j, u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const double dj = diag[jl] - u * f;
                diag[jl] = dj;
                norm[jl] = s;
                score[jl] = s / dj;
            }
        }
        ++k;
        __syncthreads();

        // ---------------------------------------------------------- 5. flush the pending downdates
        if (k == BMAX || t + 1 == S.n_remove) {
            // all slices of the pending rows must be in memory before anyone reads them
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            ++bar_epoch;
            if (tid == 0) __hip_atomic_store(S.bar + b, bar_epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            {
                bool fail = false;
                for (int sb = tid; sb < nb; sb += LT) {
                    unsigned spins = 0;
                    unsigned long long t0 = 0;
                    while (__hip_atomic_load(S.bar + sb, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < bar_epoch) {
                        if ((++spins & 255u) == 0u) {
                            if (t0 == 0) t0 = wall_clock64();
                            if (__hip_atomic_load(S.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == -1 ||
                                wall_clock64() - t0 > kTimeoutTicks) {
                                __hip_atomic_store(S.status, -1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                                fail = true;
                                break;
                            }
                        }
                    }
                    if (fail) break;
                }
                if (fail) misc[0] = 1;
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            __syncthreads();
            if (misc[0]) { ok = false; break; }

            const double *Ub = S.U + (size_t)ublk * BMAX * d;
            for (int g0 = 0; g0 < nown; g0 += ROWS_PER_PASS) {
                const int nrow = min(ROWS_PER_PASS, nown - g0);
                for (int e = tid; e < BMAX * ROWS_PER_PASS; e += LT) {
                    const int kk = e / ROWS_PER_PASS, r = e % ROWS_PER_PASS;
                    double c = 0.0;
                    if (kk < k && r < nrow && alive_own[g0 + r]) c = uloc[kk * cpb + g0 + r] / pivs[kk];
                    coef[e] = c;
                }
                __syncthreads();
                for (int c = tid; c < d; c += LT) {
                    if (!((alive_bits[c >> 5] >> (c & 31)) & 1u)) continue;
                    double acc[ROWS_PER_PASS];
#pragma unroll
                    for (int r = 0; r < ROWS_PER_PASS; ++r) acc[r] = 0.0;
                    for (int kk = 0; kk < k; ++kk) {
                        const double u = Ub[(size_t)kk * d + c];
#pragma unroll
                        for (int r = 0; r < ROWS_PER_PASS; ++r) acc[r] += coef[kk * ROWS_PER_PASS + r] * u;
                    }
#pragma unroll
                    for (int r = 0; r < ROWS_PER_PASS; ++r)
                        if (r < nrow && alive_own[g0 + r]) S.Hd[(size_t)(j0 + g0 + r) * d + c] -= acc[r];
                }
                __syncthreads();
            }
            k = 0;
            ublk ^= 1;
        }
    }

    // ------------------------------------------------------------------ final masking + write-back
    __syncthreads();
    if (b == 0 && tid == 0 && error_step != 0)
        atomicCAS(S.status, 0, error_step);
    if (ok && error_step == 0) {
        for (int jl = 0; jl < nown; ++jl) {
            const size_t row = (size_t)(j0 + jl) * d;
            const bool a = alive_own[jl] != 0;
            for (int c = tid; c < d; c += LT) {
                const bool live = a && ((alive_bits[c >> 5] >> (c & 31)) & 1u);
                S.Hinv[row + c] = live ? (float)S.Hd[row + c] : 0.f;
            }
        }
        for (int jl = wave; jl < nown; jl += NW) {
            const bool a = alive_own[jl] != 0;
            for (int i = lane; i < m; i += 64) S.W[(size_t)i * d + j0 + jl] = a ? wt[(size_t)jl * m + i] : 0.f;
        }
    }
}

struct Plan {
    int nb, cpb, w_in_lds, pay_words;
    size_t lds_bytes;
    bool feasible;
};

static Plan make_plan(int d_row, int d_col) {
    Plan p = {};
    const int cus = device_cu_count();
    p.cpb = (d_col + cus - 1) / cus;
    p.nb = (d_col + p.cpb - 1) / p.cpb;
    p.pay_words = d_row + 2 * BMAX + 2;
    const size_t lds_cap = 150 * 1024;
    p.w_in_lds = lds_layout(d_row, d_col, p.cpb, true).total <= lds_cap ? 1 : 0;
    p.lds_bytes = lds_layout(d_row, d_col, p.cpb, p.w_in_lds != 0).total;
    p.feasible = p.lds_bytes <= lds_cap;
    return p;
}

struct Layout {
    State st;
    int *snap_steps;
    size_t bytes;
};

static Layout make_layout(int d_row, int d_col, int n_snap, const Plan &p, void *ws) {
    Layout l = {};
    State &s = l.st;
    Carver c(ws);
    s.Hd = c.take<double>((size_t)d_col * d_col);
    s.Wt = c.take<float>(p.w_in_lds ? 1 : (size_t)d_col * d_row);
    s.U = c.take<double>((size_t)2 * BMAX * d_col);
    // zero-initialised region: slots, payload, barrier epochs, status
    s.slots = c.take<unsigned long long>((size_t)2 * p.nb * SLOT_WORDS);
    s.pay = c.take<unsigned long long>((size_t)2 * p.nb * p.pay_words);
    s.bar = c.take<unsigned long long>((size_t)p.nb);
    s.status = c.take<int>(1);
    l.snap_steps = c.take<int>((size_t)(n_snap > 0 ? n_snap : 1));
    l.bytes = c.off;
    return l;
}

}  // namespace lazy

// Entry points used by prune.hip ------------------------------------------------------------------
bool lazy_columns_feasible(int d_row, int d_col) { return lazy::make_plan(d_row, d_col).feasible; }

size_t lazy_columns_workspace_bytes(int d_row, int d_col, int n_snap) {
    const lazy::Plan p = lazy::make_plan(d_row, d_col);
    return lazy::make_layout(d_row, d_col, n_snap, p, nullptr).bytes;
}

// Enqueues the whole loop.  *status_dev_out receives the device address of the status word.
int lazy_columns_launch(float *W, float *Hinv, int d_row, int d_col, int n_remove, int32_t *order_out,
                        double *err_out, const uint8_t *alive_in, int n_snap, const int32_t *snap_steps_host,
                        float *W_snap, void *workspace, hipStream_t st, int **status_dev_out) {
    using namespace lazy;
    const Plan p = make_plan(d_row, d_col);
    Layout l = make_layout(d_row, d_col, n_snap, p, workspace);
    State &S = l.st;
    S.W = W; S.Hinv = Hinv; S.m = d_row; S.d = d_col; S.n_remove = n_remove;
    S.order = order_out; S.err = err_out; S.alive_in = alive_in;
    S.n_snap = n_snap; S.snap_steps = l.snap_steps; S.W_snap = W_snap;
    S.cpb = p.cpb; S.w_in_lds = p.w_in_lds; S.pay_words = p.pay_words;
    if (n_snap > 0) {
        // pageable source: staged before the call returns
        ZIPLM_HIP_TRY(hipMemcpyAsync(l.snap_steps, snap_steps_host, sizeof(int) * (size_t)n_snap, hipMemcpyHostToDevice, st));
        ZIPLM_HIP_TRY(hipStreamSynchronize(st));
    }
    const size_t zero_bytes = reinterpret_cast<char *>(l.snap_steps) - reinterpret_cast<char *>(S.slots);
    ZIPLM_HIP_TRY(hipMemsetAsync(S.slots, 0, zero_bytes, st));
    static bool attr_set = false;
    if (!attr_set) {
        ZIPLM_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(prune_lazy_kernel),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        attr_set = true;
    }
    int per_cu = 0;
    ZIPLM_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, prune_lazy_kernel, LT, p.lds_bytes));
    if (per_cu < 1 || p.nb > per_cu * device_cu_count()) return ZIPLM_ERR_DEVICE;
    void *args[] = {&S};
    ZIPLM_HIP_TRY(hipLaunchCooperativeKernel(reinterpret_cast<void *>(prune_lazy_kernel), dim3(p.nb), dim3(LT), args,
                                             (unsigned)p.lds_bytes, st));
    *status_dev_out = S.status;
    return ZIPLM_OK;
}

}  // namespace ziplm
