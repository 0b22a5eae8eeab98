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
//     downdates not yet applied.  So the downdates of a block of consecutive steps (64, or 256 for wide layers) are kept as a list
//     of pivot rows and applied to the stored matrix in one pass ("flush"), a 16 x 64 x d
//     contraction per workgroup on the fp64 matrix cores.  The stored fp64 matrix is then read and
//     written once per block instead of once per step.
//   * W is compensated at every step (Eq. 3 needs no deferral: the scores need the current W).
//
// Work is divided by columns: workgroup b owns `cpb` consecutive columns j, i.e. column j of W (kept
// transposed as a row of `wt`, in LDS when it fits), row j of the fp64 inverse Hessian, its diagonal
// entry, squared norm and score.  The owned rows of the inverse Hessian are stored as a panel
// P[c][r] (column index outer, owned row inner, padded to 16 rows), so that "column p of my rows"
// -- by symmetry my slice of row p -- is one contiguous 128-byte read.  One wavefront works on one
// owned column at a time.  Per step:
//
//   1. every workgroup publishes its best owned column (score, index) and, speculatively, what the
//      others would need if it wins: that column of W, the entries u_k[p] of the pending pivot rows
//      and the current diagonal entry.  All of it is written as 64-bit words that carry their step
//      tag next to the data, so readers can tell a fresh word from an old one without any ordering
//      between stores ("flag in data"); buffers alternate with the step parity.
//   2. every workgroup reads all candidates, takes the argmin (lowest index on ties), reads the
//      winner's payload, forms its slice of the current pivot row, updates its diagonal entries,
//      compensates its columns of W and refreshes their norms and scores.  The wavefront that reports the
//      last of these scores publishes the workgroup's candidate for the next step at once: the barrier that
//      ends the step also waits for the step's global stores to be acknowledged, and a candidate held back
//      until then would reach the other workgroups most of a microsecond later.
//
// One exchange per step is the only device-wide synchronisation; at the end of a block one barrier makes the
// finished block of pending rows visible, and every workgroup applies the block to its panel at once, over
// the list of columns that are still alive (a removed column is never read again).  Spreading that work
// over the following steps' waits, an earlier form, lost to the plain one once the flush followed the
// live columns.  All waits are bounded: on a time-out the waiter raises status = -1 and leaves; the others
// then time out or see the flag, and the grid drains.
#include "common.h"
#include "lazy_timing.h"

namespace ziplm {

int device_cu_count();

namespace lazy {

typedef double doublex4 __attribute__((ext_vector_type(4)));
constexpr unsigned long long KEY_EMPTY_ = ~0ull;

constexpr int LT = 1024;                 // threads per workgroup (16 wavefronts)
constexpr int NW = LT / 64;
// Pending pivot rows between two flushes.  Every flush reads and writes the whole panel, so a longer block means a
// smaller share of that per step (0.52 -> 0.35 us at 3072 columns for 64 -> 256 rows) and a longer history that every
// step's payload carries and every pivot-row slice is corrected with (+0.3 us per step for the same change: slower at
// 3072 columns, 2.3% faster at 4096, where the panel is 1.8 times the size).  Wide layers whose workgroups own a single
// row group (they have the LDS for it) take the long block.
constexpr int BMAX_WIDE = 256, BMAX_NARROW = 64, WIDE_FROM_D = 4096;
static_assert(BMAX_WIDE % 64 == 0 && BMAX_WIDE >= 64 && BMAX_WIDE <= 256, "one to four pending rows per lane");
constexpr int RG = 16;                   // owned rows per matrix-core pass (panel rows are padded to this)
constexpr int LIST_MAX_D = 4096;         // layers up to this many columns keep a list of their live columns in LDS
constexpr unsigned long long kTimeoutTicks = 400000000ull;   // 4 s of the 100 MHz wall clock
constexpr int IDX_NONE = -1;             // workgroup has no live column
constexpr int IDX_ERROR = -2;            // workgroup met a non-positive diagonal entry
constexpr int MAX_CPB = 250;             // the local column index travels in 8 bits
constexpr int MAX_D = 65535;             // the global column index travels in 16 bits of the comparison key
// 64-bit words between the candidate slots of two workgroups: every slot has a 32-byte sector of its own, four slots
// share a 128-byte line.  Every workgroup polls every slot, and the polls load the fabric: with a line per slot a
// wavefront's poll is 64 line requests, with four slots per line 16; closer than a sector the writers of neighbouring
// slots and the readers polling them delay one another.  Loop at 768 x 3072 by words per slot: 16 -> 12.69 ms,
// 8 -> 12.55, 4 -> 12.34, 2 -> 12.45, 1 -> 13.15.
#ifndef ZIPLM_SLOT_STRIDE
#define ZIPLM_SLOT_STRIDE 4
#endif
constexpr int SLOT_STRIDE = ZIPLM_SLOT_STRIDE;

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
    double *P;                    // [nb][d][cp]  panels of the stored (stale between flushes) inverse Hessian
    float *Wt;                    // [d][m]       transposed W when it does not fit LDS, else unused
    double *U;                    // [2][block_rows][d] pending pivot rows of the current / previous block of steps
    unsigned long long *slots;    // [2][nb][SLOT_STRIDE], word 0 of each
    unsigned long long *pay;      // [2][nb][pay_words]
    unsigned long long *bar;      // [nb] flush-barrier epochs
    int *status;
    int cpb;                      // columns per workgroup
    int cp;                       // cpb rounded up to a multiple of RG
    int pay_words;                // m + 2 * block_rows + 2
    int stall_wg;                 // -1; the self-test of the bounded waits names a workgroup that never takes part
    ZIPLM_LAZY_TIMING_FIELD
};

// One launch runs the loops of up to MAX_PACK layers of one shape side by side, each on its own nb workgroups
// (Section 3.2: layers are independent).  A loop is bound by the hand-off between its workgroups, not by
// arithmetic or bandwidth, so several loops on a share of the compute units each finish sooner than one after
// another on all of them.  Workgroup x works on layer x / nb; the layers share nothing.
constexpr int MAX_PACK = 4;
struct StatePack {
    State s[MAX_PACK];
    int nb;                       // workgroups per layer
};

// ------------------------------------------------------------------------------------------------
// tagged words
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void ll_store(unsigned long long *p, unsigned data, unsigned tag) {
    __hip_atomic_store(p, ((unsigned long long)data << 32) | tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

struct Waiter {
    unsigned spins = 0;
    unsigned long long t0 = 0;
    // call after an unsuccessful poll; returns false when the wait must be abandoned
    __device__ __forceinline__ bool again(int *status) {
        if ((++spins & 255u) == 0u) {
            if (t0 == 0) t0 = wall_clock64();
            if (__hip_atomic_load(status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == -1) return false;
            if (wall_clock64() - t0 > kTimeoutTicks) {
                __hip_atomic_store(status, -1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                return false;
            }
        }
        return true;
    }
};

// One word: 32 bits of data, 32-bit tag.
__device__ __forceinline__ bool ll_wait(const unsigned long long *p, unsigned tag, unsigned &data, int *status) {
    Waiter w;
    for (;;) {
        const unsigned long long v = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((unsigned)(v & 0xffffffffu) == tag) { data = (unsigned)(v >> 32); return true; }
        if (!w.again(status)) return false;
    }
}
// Two adjacent words, each 32 bits of data and a 32-bit tag: both loads are issued before either is tested.
__device__ __forceinline__ bool ll_wait2(const unsigned long long *p, unsigned tag, unsigned &d0, unsigned &d1, int *status) {
    Waiter w;
    for (;;) {
        const unsigned long long v0 = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long v1 = __hip_atomic_load(p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((unsigned)(v0 & 0xffffffffu) == tag && (unsigned)(v1 & 0xffffffffu) == tag) {
            d0 = (unsigned)(v0 >> 32);
            d1 = (unsigned)(v1 >> 32);
            return true;
        }
        if (!w.again(status)) return false;
    }
}
// Candidate slot, one 64-bit word: [score bits 63..12 | local column index : 8 | tag : 4].
// Scores are positive doubles, whose order is the order of their bit patterns; dropping the 12 lowest
// mantissa bits keeps that order and merges only scores closer than 2^-40 relative, which then go to the
// lower column index like any tie.  The exact score of the winner is reported by its owner.
constexpr unsigned ENC_NONE = 0xFFu, ENC_ERROR = 0xFEu;
__device__ __forceinline__ void slot_store(unsigned long long *p, double score, unsigned enc_idx, unsigned tag4) {
    const unsigned long long b = (unsigned long long)__double_as_longlong(score);
    __hip_atomic_store(p, (b & ~0xfffull) | ((unsigned long long)enc_idx << 4) | tag4, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
// The same word without the tag, as kept in LDS for the workgroup's own columns: the smallest key is the
// best candidate (lower local index on equal truncated scores).
__device__ __forceinline__ unsigned long long cand_key_of(double score, unsigned enc_idx) {
    return ((unsigned long long)__double_as_longlong(score) & ~0xfffull) | ((unsigned long long)enc_idx << 4);
}
constexpr unsigned long long KEY_NONE = ~0ull & ~0xfull;     // index field reads ENC_NONE

// Waits for slot `sb` and turns it into a comparison key [score bits 63..16 | global column : 16]: the
// smallest key over all slots is the step's pivot (scores closer than 2^-36 relative count as tied and go
// to the lower column).  KEY_EMPTY for a workgroup without live columns; *err is set if it reported a
// non-positive diagonal entry.
constexpr unsigned long long KEY_EMPTY = ~0ull;
__device__ __forceinline__ bool slot_wait(const unsigned long long *p, unsigned tag4, int sb, int cpb,
                                          unsigned long long &key, bool &err, int *status) {
    Waiter w;
    for (;;) {
        const unsigned long long v = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((unsigned)(v & 0xfu) == tag4) {
            const unsigned e = (unsigned)((v >> 4) & 0xffu);
            if (e == ENC_ERROR) err = true;
            key = (e >= ENC_ERROR) ? KEY_EMPTY : ((v & ~0xffffull) | (unsigned long long)(sb * cpb + (int)e));
            return true;
        }
        if (!w.again(status)) return false;
    }
}

// A value that is the same in every lane, moved to scalar registers (frees two vector registers).
__device__ __forceinline__ unsigned long long uniform_u64(unsigned long long v) {
    return ((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)(v >> 32)) << 32) |
           (unsigned)__builtin_amdgcn_readfirstlane((int)(v & 0xffffffffu));
}

__device__ __forceinline__ unsigned dhi(double x) { return (unsigned)((unsigned long long)__double_as_longlong(x) >> 32); }
__device__ __forceinline__ unsigned dlo(double x) { return (unsigned)((unsigned long long)__double_as_longlong(x) & 0xffffffffu); }
__device__ __forceinline__ double dmake(unsigned hi, unsigned lo) {
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

// ------------------------------------------------------------------------------------------------
// wavefront reductions on the data-parallel-primitive lane permutes (no LDS traffic)
// ------------------------------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true); }
template <int CTRL>
__device__ __forceinline__ double dpp_d(double v) { return dmake((unsigned)dpp_i<CTRL>((int)dhi(v)), (unsigned)dpp_i<CTRL>((int)dlo(v))); }
__device__ __forceinline__ double readlane_d(double v, int lane) {
    return dmake((unsigned)__builtin_amdgcn_readlane((int)dhi(v), lane), (unsigned)__builtin_amdgcn_readlane((int)dlo(v), lane));
}
constexpr int DPP_XOR1 = 0xB1, DPP_XOR2 = 0x4E, DPP_HALF_MIRROR = 0x141, DPP_MIRROR = 0x140;

// Sum over the 64 lanes, returned in every lane.  Four butterfly steps inside the 16-lane rows, then
// the row totals are chained with the row-broadcast permutes (lane 15 of rows 0 and 2 into rows 1 and
// 3, lane 31 into rows 2 and 3), which leaves the grand total in lane 63.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_rows_d(double v) {
    return dmake((unsigned)__builtin_amdgcn_update_dpp(0, (int)dhi(v), CTRL, ROW_MASK, 0xf, false),
                 (unsigned)__builtin_amdgcn_update_dpp(0, (int)dlo(v), CTRL, ROW_MASK, 0xf, false));
}
__device__ __forceinline__ double wave_sum(double v) {
    v += dpp_d<DPP_XOR1>(v);
    v += dpp_d<DPP_XOR2>(v);
    v += dpp_d<DPP_HALF_MIRROR>(v);
    v += dpp_d<DPP_MIRROR>(v);          // every lane of a 16-lane row holds the row's sum
    v += dpp_rows_d<0x142, 0xa>(v);     // row_bcast:15 into rows 1 and 3 (other rows add 0)
    v += dpp_rows_d<0x143, 0xc>(v);     // row_bcast:31 into rows 2 and 3
    return readlane_d(v, 63);
}

template <int CTRL>
__device__ __forceinline__ unsigned long long dpp_u64(unsigned long long v) {
    return ((unsigned long long)(unsigned)dpp_i<CTRL>((int)(v >> 32)) << 32) | (unsigned)dpp_i<CTRL>((int)(v & 0xffffffffu));
}
__device__ __forceinline__ unsigned long long umin64(unsigned long long a, unsigned long long b) { return a < b ? a : b; }
// Minimum of a 64-bit key over the 64 lanes, returned in every lane.
__device__ __forceinline__ unsigned long long wave_min_u64(unsigned long long v) {
    v = umin64(v, dpp_u64<DPP_XOR1>(v));
    v = umin64(v, dpp_u64<DPP_XOR2>(v));
    v = umin64(v, dpp_u64<DPP_HALF_MIRROR>(v));
    v = umin64(v, dpp_u64<DPP_MIRROR>(v));
    unsigned long long r = KEY_EMPTY_;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const unsigned long long x = ((unsigned long long)(unsigned)__builtin_amdgcn_readlane((int)(v >> 32), 16 * q) << 32) |
                                     (unsigned)__builtin_amdgcn_readlane((int)(v & 0xffffffffu), 16 * q);
        r = umin64(r, x);
    }
    return r;
}

// ------------------------------------------------------------------------------------------------
// LDS carve-up (byte offsets), identical on host and device
// ------------------------------------------------------------------------------------------------
struct Lds {
    size_t uloc, coefa, cvec, pivs, rpivs, wcol, norm, diag, score, hstale, alive_own, alive_bits, snap_bits, live_list, word_prefix, misc, wt, total;
};
__host__ __device__ inline int padded_rows(int m) { return (m + 255) / 256 * 256; }   // Eq. 3 runs unguarded
// block length of a layer: the long one only where W stays in LDS and the launch holds one layer (one more kernel
// instantiation, the block length being a compile-time constant of each)
inline int block_rows(int cp, int d, bool w_in_lds, int pack) {
    return (cp == RG && d >= WIDE_FROM_D && w_in_lds && pack == 1) ? BMAX_WIDE : BMAX_NARROW;
}
__host__ __device__ inline Lds lds_layout(int m, int d, int cp, bool w_in_lds, int cpb, int bmax) {
    Lds l;
    const int mp = padded_rows(m);
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t r = o; o += (bytes + 15) / 16 * 16; return r; };
    l.uloc = take(sizeof(double) * bmax * cp);           // pending pivot rows, owned slice: [row][k]
    // matrix-core A fragments of the flush: one set per row group of a pass (up to three, see flush_panel)
    l.coefa = take(sizeof(double) * (bmax / 4 * 64) * (cp > RG ? 3 : 1));     // [row group][k-group][lane]
    l.cvec = take(sizeof(double) * bmax);                // u_k[p] / piv_k for the current pivot
    l.rpivs = take(sizeof(double) * bmax);               // reciprocals of the pivots of the pending rows
    l.pivs = take(sizeof(double) * bmax);                // pivots of the pending rows
    l.wcol = take(mp * sizeof(float));                   // column p of W, zero beyond row m
    l.norm = take(sizeof(double) * cp);
    l.diag = take(sizeof(double) * cp);
    l.score = take(sizeof(double) * cp);
    l.hstale = take(sizeof(double) * cp);
    l.alive_own = take(sizeof(int) * cp);
    l.alive_bits = take(sizeof(unsigned) * ((d + 31) / 32));
    l.snap_bits = take(sizeof(unsigned) * ((d + 32) / 32 + 1));
    // Columns alive at the end of the last block of steps, in ascending order: the deferred eliminations run over the
    // list, not over all columns (up to LIST_MAX_D columns: 8 KB; wider layers need the space for their pending rows)
    const bool listed = d <= LIST_MAX_D;
    l.live_list = take(listed ? sizeof(unsigned short) * d : 0);
    l.word_prefix = take(listed ? sizeof(int) * ((d + 31) / 32 + 1) : 0);
    l.misc = take(96);
    l.wt = take(w_in_lds ? sizeof(float) * (size_t)cpb * mp : 0);
    l.total = o;
    return l;
}


// Applies the k pending downdates to one workgroup's panel:
//   P[c][g0 + r] -= sum_kk (uloc[kk][g0 + r] / piv_kk) * U[kk][c]   on v_mfma_f64_16x16x4_f64.
// Lane l supplies A[row l%16][k l/16] and B[k l/16][col l%16]; its accumulator v holds
// D[row 4v + l/16][col l%16].  Matrix row i = 4v + q is mapped to owned row g0 + 4q + v, so a lane ends
// up with four consecutive rows of one column: 32 contiguous bytes of the panel.
// A panel wider than one row group (several layers share the launch, or d_col above 4096) is taken
// FLUSH_RGC row groups at a time, so that a tile of pending rows is fetched once for all of them (coefa holds one set
// of A fragments per row group of the pass).  Two or three is what the register budget of those instantiations
// allows; the one that the single-layer loop of a 768 x 3072 or 1024 x 4096 layer runs (W in LDS, one row group)
// keeps one.
constexpr int FLUSH_KB = 8;              // k-groups whose pending-row entries are requested together
template <int FLUSH_RGC, int BROWS>
__device__ __forceinline__ void flush_panel(double *__restrict__ P, const double *__restrict__ Ub,
                                                      const double *uloc, const double *pivs, double *coefa,
                                                      const int *alive_own, const unsigned *alive_bits,
                                                      const unsigned short *live_list, int nlist,
                                                      int k, int d, int cp) {
    // This runs once per block of steps.  The thread index is made opaque here so that the address arithmetic
    // below is redone on entry instead of being hoisted out of the step loop, where it would hold vector
    // registers through every step.
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, wave = tid >> 6;
    const int q4 = lane >> 4, cl16 = lane & 15;
    const int nks = (k + 3) / 4;
    constexpr int bmax = BROWS, afrag = BROWS / 4 * 64;
    // with a list of the live columns a tile is sixteen consecutive entries of the list (a column's rows of the panel
    // are one 128-byte line wherever the column lies), otherwise sixteen consecutive columns
    const int ntiles = ((live_list ? nlist : d) + 15) / 16;
    for (int g0 = 0; g0 < cp; g0 += RG * FLUSH_RGC) {
        const int nrgc = min(FLUSH_RGC, (cp - g0) / RG);
        // A fragment entry: row group e / afrag, k-group (e / 64) % (bmax / 4), lane e % 64; zeros for row groups past the panel
        for (int e = tid; e < (cp > RG ? FLUSH_RGC : 1) * afrag; e += LT) {
            const int rgc = e / afrag, l = e & 63, kk = 4 * ((e >> 6) % (bmax / 4)) + (l >> 4);
            const int arow = g0 + rgc * RG + 4 * (l & 3) + ((l & 15) >> 2);
            coefa[e] = (rgc < nrgc && kk < k && alive_own[arow]) ? -(uloc[arow * bmax + kk] / pivs[kk]) : 0.0;
        }
        __syncthreads();
        // bit x: one of this lane's four rows in row group x of the pass is alive (the three-row-group form, which the
        // launches of several layers use, has no register left for the test and keeps touching every row)
        unsigned rows_live = FLUSH_RGC < 3 ? 0u : ~0u;
#pragma unroll
        for (int x = 0; x < FLUSH_RGC; ++x) {
            if (FLUSH_RGC < 3 && x < nrgc) {
                const int r0 = g0 + x * RG + 4 * q4;
                if (alive_own[r0] | alive_own[r0 + 1] | alive_own[r0 + 2] | alive_own[r0 + 3]) rows_live |= 1u << x;
            }
        }
        if (FLUSH_RGC == 1 && live_list && k == bmax) {
            // The common case (a full block, one row group, a list of live columns) as straight-line code: nothing
            // about a request depends on the lane any more -- a lane past the end of the list asks for the list's
            // last column and keeps the result to itself, a lane whose four rows are dead asks anyway -- so the
            // requests of a tile go out back to back, the A fragments are read from LDS in batches ahead of the
            // matrix instructions that use them, and those follow one another with five requests in flight ahead of
            // them.  (The general form below compiles to a test around every request and a full wait in front of every
            // matrix instruction.)
            const bool rows_ok = (rows_live & 1u) != 0;
            // the panel entries of the next tile are asked for before this tile's pending rows: two tiles of the panel
            // in flight per wavefront (the flush is bound by the panel's read-modify-write)
            int ct = wave, c_next = 0;
            bool ok_next = false;
            doublex4 acc_next = {0.0, 0.0, 0.0, 0.0};
            if (ct < ntiles) {
                const int li = ct * 16 + cl16;
                ok_next = li < nlist;
                c_next = (int)live_list[ok_next ? li : nlist - 1];
                acc_next = *reinterpret_cast<const doublex4 *>(P + (size_t)c_next * cp + g0 + 4 * q4);
            }
            while (ct < ntiles) {
                const int c = c_next;
                const bool col_ok = ok_next;
                doublex4 acc = acc_next;
                double *pc = P + (size_t)c * cp + g0 + 4 * q4;
                const int ctn = ct + NW;
                if (ctn < ntiles) {
                    const int li = ctn * 16 + cl16;
                    ok_next = li < nlist;
                    c_next = (int)live_list[ok_next ? li : nlist - 1];
                    acc_next = *reinterpret_cast<const doublex4 *>(P + (size_t)c_next * cp + g0 + 4 * q4);
                }
                const unsigned voff = ((unsigned)q4 * (unsigned)d + (unsigned)c) * (unsigned)sizeof(double);
                // the A fragments are read again for every tile (an opaque lane index keeps them from being held in
                // thirty-two registers across the whole loop, which the second tile in flight needs)
                int alane = lane;
                asm volatile("" : "+v"(alane));
#pragma unroll
                for (int h = 0; h < BROWS / 4; h += FLUSH_KB) {
                    double bv[FLUSH_KB], av[FLUSH_KB];
#pragma unroll
                    for (int e = 0; e < FLUSH_KB; ++e) {
                        const char *base = reinterpret_cast<const char *>(Ub + (size_t)(h + e) * 4 * d);
                        bv[e] = __hip_atomic_load(reinterpret_cast<const double *>(base + voff), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
#pragma unroll
                    for (int e = 0; e < FLUSH_KB; ++e) av[e] = coefa[(h + e) * 64 + alane];
#pragma unroll
                    for (int e = 0; e < FLUSH_KB; ++e) acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av[e], bv[e], acc, 0, 0, 0);
                }
                if (col_ok && rows_ok) *reinterpret_cast<doublex4 *>(pc) = acc;
                ct = ctn;
            }
        } else
        for (int ct = wave; ct < ntiles; ct += NW) {
            int c = ct * 16 + cl16;
            bool col_ok;
            if (live_list) {
                col_ok = c < nlist;
                c = col_ok ? (int)live_list[c] : 0;
            } else {
                col_ok = (c < d) && ((alive_bits[c >> 5] >> (c & 31)) & 1u);
            }
            if (!__any(col_ok)) continue;
            // The accumulators start as the panel's entries and the A fragments are negated: the tile's entries are
            // asked for together with the first pending rows and leave with a plain store, instead of a dependent
            // read-modify-write behind the products.  A lane's four rows: nothing to read or write when none of them is
            // alive (the padding rows of the panel never are, and owned columns die as the run goes on).
            doublex4 acc[FLUSH_RGC];
#pragma unroll
            for (int x = 0; x < FLUSH_RGC; ++x) {
                acc[x] = doublex4{0.0, 0.0, 0.0, 0.0};
                if (col_ok && x < nrgc && ((rows_live >> x) & 1u))
                    acc[x] = *reinterpret_cast<const doublex4 *>(P + (size_t)c * cp + g0 + x * RG + 4 * q4);
            }
            // a uniform base per k-group plus one 32-bit lane offset: one address register for all the requests
            const unsigned voff = ((unsigned)q4 * (unsigned)d + (unsigned)c) * (unsigned)sizeof(double);
            for (int h = 0; h < nks; h += FLUSH_KB) {
                double bv[FLUSH_KB];
#pragma unroll
                for (int e = 0; e < FLUSH_KB; ++e) {
                    const int kk = 4 * (h + e) + q4;
                    const char *base = reinterpret_cast<const char *>(Ub + (size_t)(h + e) * 4 * d);
                    bv[e] = (kk < k && col_ok) ? __hip_atomic_load(reinterpret_cast<const double *>(base + voff), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.0;
                }
#pragma unroll
                for (int e = 0; e < FLUSH_KB; ++e) {
                    if (h + e < nks) {
#pragma unroll
                        for (int x = 0; x < FLUSH_RGC; ++x)
                            if (x == 0 || cp > RG) acc[x] = __builtin_amdgcn_mfma_f64_16x16x4f64(coefa[x * afrag + (h + e) * 64 + lane], bv[e], acc[x], 0, 0, 0);
                    }
                }
            }
            if (col_ok) {
#pragma unroll
                for (int x = 0; x < FLUSH_RGC; ++x)
                    if (x < nrgc && ((rows_live >> x) & 1u))
                        *reinterpret_cast<doublex4 *>(P + (size_t)c * cp + g0 + x * RG + 4 * q4) = acc[x];
            }
        }
        __syncthreads();
    }
}

// PACKED: several layers share the launch.  The single-layer instantiations address the one State through
// constant offsets of the kernel argument; with the layer chosen at run time the compiler re-reads fields
// inside the loop, which costs the single-layer loop 2.5%.
template <bool W_IN_LDS, bool PACKED, int BROWS>
__global__ __launch_bounds__(LT) void prune_lazy_kernel(const StatePack pack) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    ZIPLM_LAZY_TIMING_LOCALS
    const int nb = PACKED ? pack.nb : (int)gridDim.x;
    const int layer = PACKED ? blockIdx.x / nb : 0, b = blockIdx.x - layer * nb;
    const State &S = pack.s[layer];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (!PACKED && S.stall_wg == b) {
        // Self-test of the bounded waits (single-layer launches only): this workgroup withholds its candidates, the
        // others wait for them, give up at the limit and raise the status word, which this workgroup polls (bounded
        // as well) before it leaves.
        if (tid == 0) { Waiter w; while (w.again(S.status)) {} }
        return;
    }
    const int m = S.m, d = S.d, cpb = S.cpb, cp = S.cp;
    constexpr int bmax = BROWS;               // steps per block of deferred eliminations
    const Lds L = lds_layout(m, d, cp, W_IN_LDS, cpb, bmax);
    double *uloc = reinterpret_cast<double *>(smem + L.uloc);
    double *cvec = reinterpret_cast<double *>(smem + L.cvec);
    double *rpivs = reinterpret_cast<double *>(smem + L.rpivs);
    double *pivs = reinterpret_cast<double *>(smem + L.pivs);
    float *wcol = reinterpret_cast<float *>(smem + L.wcol);
    double *coefa = reinterpret_cast<double *>(smem + L.coefa);
    double *norm = reinterpret_cast<double *>(smem + L.norm);
    double *diag = reinterpret_cast<double *>(smem + L.diag);
    double *score = reinterpret_cast<double *>(smem + L.score);
    double *hstale = reinterpret_cast<double *>(smem + L.hstale);
    int *alive_own = reinterpret_cast<int *>(smem + L.alive_own);
    unsigned *alive_bits = reinterpret_cast<unsigned *>(smem + L.alive_bits);
    unsigned *snap_bits = reinterpret_cast<unsigned *>(smem + L.snap_bits);
    unsigned short *live_list = reinterpret_cast<unsigned short *>(smem + L.live_list);
    int *word_prefix = reinterpret_cast<int *>(smem + L.word_prefix);
    int *misc = reinterpret_cast<int *>(smem + L.misc);   // [0] fail flag, [2] error seen, [7] length of live_list
    unsigned long long *cand_key = reinterpret_cast<unsigned long long *>(smem + L.misc + 64);   // best owned column
    unsigned long long *gkey_min = reinterpret_cast<unsigned long long *>(smem + L.misc + 80);   // arg-min of the exchange; the pair
    unsigned long long *gkey_max = reinterpret_cast<unsigned long long *>(smem + L.misc + 88);   // is 16-byte aligned: one read
    double *misc_d = reinterpret_cast<double *>(smem + L.misc + 32);  // [1] pivot, [2] 1 / pivot

    const int j0 = b * cpb;
    const int nown = max(0, min(cpb, d - j0));
    double *P = S.P + (size_t)b * d * cp;       // this workgroup's panel: P[c * cp + r] = Hinv[j0 + r][c]
    float *wt_lds = reinterpret_cast<float *>(smem + L.wt);
    const int mp = padded_rows(m);               // row pitch of wt and length of wcol: padding holds zeros
    float *wt_glb = S.Wt + (size_t)j0 * mp;
#define WT(jl, i) (*(W_IN_LDS ? &wt_lds[(size_t)(jl) * mp + (i)] : &wt_glb[(size_t)(jl) * mp + (i)]))

    // ------------------------------------------------------------------ set-up (own data only)
    for (int w = tid; w < (d + 31) / 32; w += LT) {
        unsigned bits = 0;
        for (int e = 0; e < 32; ++e) {
            const int c = w * 32 + e;
            if (c < d && (S.alive_in ? S.alive_in[c] != 0 : true)) bits |= 1u << e;
        }
        alive_bits[w] = bits;
    }
    if (tid == 0) { misc[0] = 0; misc[2] = 0; *cand_key = KEY_NONE; *gkey_min = KEY_EMPTY; *gkey_max = 0; }
    for (int w = tid; w < (d + 32) / 32 + 1; w += LT) snap_bits[w] = 0;
    for (int r = tid; r < cp; r += LT) { alive_own[r] = 0; norm[r] = 0.0; diag[r] = 1.0; score[r] = 0.0; hstale[r] = 0.0; }
    for (int e = tid; e < bmax * cp; e += LT) uloc[e] = 0.0;
    for (int i = tid; i < mp; i += LT) wcol[i] = 0.f;
    __syncthreads();
    for (int q = tid; q < S.n_snap; q += LT) {
        const int sstep = S.snap_steps[q];
        atomicOr(&snap_bits[sstep >> 5], 1u << (sstep & 31));
    }
    for (int c = tid; c < d; c += LT)
        for (int r = 0; r < cp; ++r) P[(size_t)c * cp + r] = (r < nown) ? (double)S.Hinv[(size_t)(j0 + r) * d + c] : 0.0;
    for (int jl = wave; jl < nown; jl += NW) {
        const int j = j0 + jl;
        double s = 0.0;
        for (int i = lane; i < mp; i += 64) {
            const float w = (i < m) ? S.W[(size_t)i * d + j] : 0.f;
            WT(jl, i) = w;
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
            if (alive) atomicMin(cand_key, (dj > 0.0) ? cand_key_of(s / dj, (unsigned)jl) : cand_key_of(0.0, ENC_ERROR));
        }
    }
    __syncthreads();

    if (tid == 0) {
        int n = 0;
        for (int jl = 0; jl < nown; ++jl) n += alive_own[jl] ? 1 : 0;
        misc[5] = n;
    }
    __syncthreads();
    int nlive = misc[5];        // live owned columns (uniform)
    // bit r: owned column wave + NW * r is alive -- what alive_own says, without a dependent LDS read at the head
    // of step 4 (every such read on the path from the exchange to the next slot costs a fifth of a microsecond)
    unsigned my_live = 0;
    for (int jl = wave, r = 0; jl < nown; jl += NW, ++r) my_live |= (alive_own[jl] ? 1u : 0u) << r;
    bool slot_early = false;    // the slot of the coming step was already published at the end of the last one

    unsigned long long bar_epoch = 0;
    int k = 0;          // pending pivot rows
    int ublk = 0;       // which half of U the current block of steps writes
    int t = 0;
    bool ok = true;
    int error_step = 0;
    unsigned tag4 = 0;
    double tau = 1.0e300;   // publish the payload ahead of the exchange only if my best score is <= tau
    const unsigned long long cpb_magic = (0x100000000ull + (unsigned)cpb - 1) / (unsigned)cpb;

    for (; t <= S.n_remove; ++t) {
        // -------------------------------------------------------------- snapshots after t removals
        for (int q = 0; S.n_snap > 0 && ((snap_bits[t >> 5] >> (t & 31)) & 1u) && q < S.n_snap; ++q) {
            if (S.snap_steps[q] != t) continue;      // uniform
            float *dst = S.W_snap + (size_t)q * m * d;
            for (int jl = wave; jl < nown; jl += NW) {
                const bool a = alive_own[jl] != 0;
                for (int i = lane; i < m; i += 64) dst[(size_t)i * d + j0 + jl] = a ? WT(jl, i) : 0.f;
            }
        }
        if (t == S.n_remove) break;

        const unsigned tag = (unsigned)(t + 1);
        tag4 = (tag4 == 15u) ? 1u : tag4 + 1u;              // 1..15: never 0 (the initial fill), differs from step t - 2
        const int par = t & 1;
        TICK(0);

        // ---------------------------------------------------------- 1. local candidate + publish
        // the owned columns' wavefronts have reduced their (score, index) keys into one LDS word
        const unsigned long long key = *cand_key;
        const unsigned key_idx = (unsigned)((key >> 4) & 0xffu);
        const int cand = (key_idx == ENC_NONE) ? IDX_NONE : (key_idx == ENC_ERROR) ? IDX_ERROR : j0 + (int)key_idx;
        const double cand_score_trunc = __longlong_as_double((long long)(key & ~0xfffull));
        if (tid == 0) {
            if (!slot_early)
                __hip_atomic_store(S.slots + ((size_t)par * nb + b) * SLOT_STRIDE, key | tag4, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ZIPLM_LAZY_TIMING_LOCAL_DONE;
        }
        // The payload travels ahead of the exchange only from workgroups that are likely to win (score
        // within the range of the previous step's leaders); any other winner publishes after the
        // exchange.  Readers wait on the tags either way, so this is a matter of traffic, not of
        // correctness.
        const bool published = (cand >= 0) && (cand_score_trunc <= tau);
        auto publish_payload = [&](int col) {
            const int cl = col - j0;
            unsigned long long *pw = S.pay + ((size_t)par * nb + b) * S.pay_words;
            for (int i = tid; i < m; i += LT) ll_store(pw + i, __float_as_uint(WT(cl, i)), tag);
            if (tid >= LT - bmax && tid - (LT - bmax) < k) {     // the last wavefronts: rarely busy in step 4
                const int kk = tid - (LT - bmax);
                const double u = uloc[cl * bmax + kk];
                ll_store(pw + m + 2 * kk, dhi(u), tag);
                ll_store(pw + m + 2 * kk + 1, dlo(u), tag);
            }
            if (tid == LT - bmax - 1) {
                const double dv = diag[cl];
                ll_store(pw + m + 2 * bmax, dhi(dv), tag);
                ll_store(pw + m + 2 * bmax + 1, dlo(dv), tag);
            }
        };
        if (published) publish_payload(cand);
        TICK(1);

        // ---------------------------------------------------------- 2. all candidates -> argmin
        int p;
        {
            unsigned long long mykey = KEY_EMPTY;
            bool fail = false, err = false;
            for (int sb = tid; sb < nb; sb += LT) {
                unsigned long long kv;
                if (!slot_wait(S.slots + ((size_t)par * nb + sb) * SLOT_STRIDE, tag4, sb, cpb, kv, err, S.status)) { fail = true; break; }
                ZIPLM_LAZY_TIMING_OWN_SLOT;
                mykey = umin64(mykey, kv);
            }
            const int nwaves_used = min(NW, (nb + 63) / 64);
            if (wave < nwaves_used) {
                mykey = wave_min_u64(mykey);
                // the smallest key of all slots, and the largest of the per-wavefront minima (next threshold)
                if (lane == 0) {
                    atomicMin(gkey_min, mykey);
                    if (mykey != KEY_EMPTY) atomicMax(gkey_max, mykey);
                }
            }
            if (fail) misc[0] = 1;
            if (err) misc[2] = 1;
            __syncthreads();
            typedef unsigned long long ullx2 __attribute__((ext_vector_type(2)));
            const ullx2 kmm = *reinterpret_cast<const ullx2 *>(gkey_min);
            const unsigned long long kmin = kmm[0], kmax = kmm[1];
            p = (kmin == KEY_EMPTY) ? IDX_NONE : (int)(kmin & 0xffffu);
            // next step's publication threshold: the largest of the per-wavefront minima (each over 64
            // workgroups); with a single wavefront of candidates everybody keeps publishing
            tau = (nwaves_used >= 2) ? __longlong_as_double((long long)(kmax | 0xffffull)) : 1.0e300;
        }
        TICK(2);
        ZIPLM_LAZY_TIMING_EXCHANGE_DONE;
        // A dependent LDS read costs a fifth of a microsecond on this path: the time-out and error flags of the
        // exchange are looked at after step 3 (p is a valid column or "none" whatever they say).
        // same inputs in every workgroup: uniform.  No candidate at all: nothing is left alive (the caller asked for
        // more removals than live columns), unless a workgroup reported a non-positive diagonal entry -- told apart
        // after the loop
        if (p < 0) { error_step = -(2 + t); break; }
        const int owner = (int)(((unsigned long long)(unsigned)p * cpb_magic) >> 32);      // p / cpb
        // The thread index is made opaque for this stretch: predicates on it are then recomputed (one compare) where
        // they are used instead of being kept across the whole step loop in scalar register pairs, of which the
        // kernel has none to spare -- they were spilled to vector lanes and read back two lanes per predicate.
        int tid3 = tid;
        asm volatile("" : "+v"(tid3));
        if (tid3 == 0) { *cand_key = KEY_NONE; misc[6] = 0; }   // every thread read the key before the barrier of the exchange
        if (owner == b && !published) publish_payload(p);

        // ---------------------------------------------------------- 3. winner's payload + stale column p
        {
            const unsigned long long *pw = S.pay + ((size_t)par * nb + owner) * S.pay_words;
            bool fail = false;
            // The first N3 wavefronts do all of this step.  After the barrier of the exchange the sixteen wavefronts
            // share four instruction issuers: the last ones reach this point a quarter of a microsecond after the
            // first, so whatever the step waits for is given to those that arrive first, and every thread asks for
            // everything it needs (up to three words of the W column, one pair of words of the pending rows or the
            // diagonal, its entry of the stale column) before it waits for any of it.
            constexpr int N3 = 6, T3 = 64 * N3, WQ = 3;
            if (tid3 < T3) {
                // the first wavefront fetches the stale column, the next ones the history (one pending row per thread)
                // and the diagonal entry behind it
                static_assert(64 + BROWS < T3, "history and diagonal fit the wavefronts of this step");
                const int kk_hist = tid3 - 64;
                const bool r_hist = kk_hist >= 0 && kk_hist < k;
                const bool r_diag = tid3 == 64 + bmax;
                const unsigned long long *pa = r_hist ? pw + m + 2 * kk_hist : r_diag ? pw + m + 2 * bmax : nullptr;
                double hv = 0.0;
                // column p of the stored matrix restricted to my rows (= my slice of row p, by symmetry)
                if (tid3 < cp) hv = P[(size_t)p * cp + tid3];
                unsigned long long a0 = 0, a1 = 0, w0[WQ];
                if (pa) {
                    a0 = __hip_atomic_load(pa, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    a1 = __hip_atomic_load(pa + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
#pragma unroll
                for (int q = 0; q < WQ; ++q) {
                    const int i = tid3 + q * T3;
                    w0[q] = (i < m) ? __hip_atomic_load(pw + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0ull;
                }
                double rp = 0.0;                  // reciprocal pivot of my pending row: asked for ahead of the waits
                if (r_hist) rp = rpivs[kk_hist];
                ZIPLM_LAZY_TIMING_PAYLOAD_SEEN(w0[0]);
                if (tid3 < cp) hstale[tid3] = hv;
                if (pa) {
                    unsigned hi = (unsigned)(a0 >> 32), lo = (unsigned)(a1 >> 32);
                    const bool there = (unsigned)(a0 & 0xffffffffu) == tag && (unsigned)(a1 & 0xffffffffu) == tag;
                    if (!there && !ll_wait2(pa, tag, hi, lo, S.status)) fail = true;
                    const double val = dmake(hi, lo);
                    if (r_hist) cvec[kk_hist] = val * rp;
                    else {
                        // reciprocal by two Newton steps from the hardware estimate: short enough not to hold up the barrier
                        double r = __builtin_amdgcn_rcp(val);
                        r = __builtin_fma(__builtin_fma(-val, r, 1.0), r, r);
                        r = __builtin_fma(__builtin_fma(-val, r, 1.0), r, r);
                        misc_d[1] = val;
                        misc_d[2] = r;
                    }
                }
#pragma unroll
                for (int q = 0; q < WQ; ++q) {
                    const int i = tid3 + q * T3;
                    if (i < m) {
                        unsigned v = (unsigned)(w0[q] >> 32);
                        if ((unsigned)(w0[q] & 0xffffffffu) != tag && !ll_wait(pw + i, tag, v, S.status)) fail = true;
                        wcol[i] = __uint_as_float(v);
                    }
                }
                for (int i = tid3 + WQ * T3; i < m && !fail; i += T3) {        // layers with more than 1152 rows
                    unsigned v;
                    if (!ll_wait(pw + i, tag, v, S.status)) { fail = true; break; }
                    wcol[i] = __uint_as_float(v);
                }
            }
            if (fail) misc[0] = 1;
            __syncthreads();
        }
        TICK(3);
        // One LDS round trip for all four; the two failure flags are acted on after step 4 (a branch here would
        // keep the column wavefronts from issuing their loads; nothing of a failed run is written back).
        const int flag_fail = misc[0], flag_err = misc[2];
        const double piv = misc_d[1], rpiv = misc_d[2];
        // columns that will report a new score in step 4; the last one to do so publishes the workgroup's
        // slot of the next step at once, without waiting for the barrier and the loop head
        const int participants = nlive - (owner == b ? 1 : 0);
        const bool more_steps = t + 1 < S.n_remove;

        // ---------------------------------------------------------- 4. own slice of the pivot row, Eq. 3
        for (int jl = wave, r = 0; jl < nown; jl += NW, ++r) {
            // wave-uniform; with W in the workspace the kernel has no register to spare for what the early
            // answer lets the compiler hoist, and asks LDS instead
            if (W_IN_LDS ? !((my_live >> r) & 1u) : !alive_own[jl]) continue;
            const int j = j0 + jl;
            if (j == p) {
                if (lane == 0) alive_own[jl] = 0;
                my_live &= ~(1u << r);
                continue;
            }
            typedef float floatx4 __attribute__((ext_vector_type(4)));
            // W in the workspace: the column's first 1024 rows are requested before anything else of the column, so
            // that one round trip to the L2 covers them all and overlaps the reduction of the pivot-row entry
            // (one request at a time made this phase the longest of the step when several layers share the launch)
            constexpr int WPRE = 4;
            floatx4 wpre[WPRE];
            if (!W_IN_LDS) {
#pragma unroll
                for (int q = 0; q < WPRE; ++q)      // no branches between the requests: blocks beyond mp re-read the last one
                    wpre[q] = *reinterpret_cast<const floatx4 *>(&WT(jl, min(256 * q, mp - 256) + 4 * lane));
            }
            const double diag_old = diag[jl];        // asked for here, needed after the column's pass
            double term = (lane < k) ? cvec[lane] * uloc[jl * bmax + lane] : 0.0;
#pragma unroll
            for (int q = 1; q < BROWS / 64; ++q)
                if (lane + 64 * q < k) term += cvec[lane + 64 * q] * uloc[jl * bmax + lane + 64 * q];
            const double u = hstale[jl] - wave_sum(term);
            const double f = u * rpiv;
            const float nf = -(float)f;
            double s = 0.0;
            if (!W_IN_LDS) {
                for (int i0 = 0; i0 < mp; i0 += 256 * WPRE) {
                    if (i0 > 0) {
#pragma unroll
                        for (int q = 0; q < WPRE; ++q)
                            wpre[q] = *reinterpret_cast<const floatx4 *>(&WT(jl, min(i0 + 256 * q, mp - 256) + 4 * lane));
                    }
#pragma unroll
                    for (int q = 0; q < WPRE; ++q) {
                        if (i0 + 256 * q < mp) {
                            const floatx4 c = *reinterpret_cast<const floatx4 *>(&wcol[i0 + 256 * q + 4 * lane]);
                            floatx4 w = wpre[q];
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                w[e] = __builtin_fmaf(c[e], nf, w[e]);
                                s += (double)w[e] * (double)w[e];
                            }
                            *reinterpret_cast<floatx4 *>(&WT(jl, i0 + 256 * q + 4 * lane)) = w;
                        }
                    }
                }
            } else
            for (int i0 = 0; i0 < mp; i0 += 256) {         // rows beyond m hold zeros and stay zero
                // four consecutive rows per lane: one 128-bit LDS access per operand
                floatx4 *wp = reinterpret_cast<floatx4 *>(&WT(jl, i0 + 4 * lane));
                floatx4 w = *wp;
                const floatx4 c = *reinterpret_cast<const floatx4 *>(&wcol[i0 + 4 * lane]);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    w[e] = __builtin_fmaf(c[e], nf, w[e]);               // Eq. 3 on the fp32 state, one rounding
                    s += (double)w[e] * (double)w[e];
                }
                *wp = w;
            }
            s = wave_sum(s);
            if (lane == 0) {
                const double dj = diag_old - u * f;
                // s / dj by Newton steps from the hardware reciprocal estimate plus one correction of the quotient: a
                // third of the instructions of a full division, on the path that decides when the next slot goes out
                double rd = __builtin_amdgcn_rcp(dj);
                rd = __builtin_fma(__builtin_fma(-dj, rd, 1.0), rd, rd);
                rd = __builtin_fma(__builtin_fma(-dj, rd, 1.0), rd, rd);
                double sc = s * rd;
                sc = __builtin_fma(__builtin_fma(-dj, sc, s), rd, sc);
                // INVARIANT (the only place where the kernel relies on the order in which one wavefront's LDS operations
                // are issued): merge the key, count, read the minimum back -- in this order, back to back, one round
                // trip.  LDS executes a wavefront's operations in issue order, and the atomics of different wavefronts
                // one at a time; so the wavefront whose count comes out last reads a minimum that holds every other
                // column's key, each of which was issued ahead of its own count.  The three are relaxed atomics on two
                // addresses: nothing in the language stops a compiler from swapping the merge and the count, which
                // would let the last counter publish a minimum that misses a key.  This compiler keeps atomics in
                // program order, and tests/test_kernel_resources.py checks the generated code for exactly this
                // sequence.  (A fence between them would make the order a language-level fact at the price of a second
                // LDS round trip on the chain that decides when the next slot goes out.)
                atomicMin(cand_key, (dj > 0.0) ? cand_key_of(sc, (unsigned)jl) : cand_key_of(0.0, ENC_ERROR));
                const int reported = atomicAdd(&misc[6], 1);
                // (an atomic load, not a volatile one: the latter is compiled to a flat load with system scope, which
                // also waits for the stores to global memory still in flight)
                const unsigned long long knext = __hip_atomic_load(cand_key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                // bookkeeping nobody waits for
                uloc[jl * bmax + k] = u;
                diag[jl] = dj;
                norm[jl] = s;
                score[jl] = sc;
                if (reported == participants - 1 && more_steps) {
                    const unsigned tag4_next = (tag4 == 15u) ? 1u : tag4 + 1u;
                    __hip_atomic_store(S.slots + ((size_t)((t + 1) & 1) * nb + b) * SLOT_STRIDE, knext | tag4_next, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                }
                __hip_atomic_store(S.U + ((size_t)ublk * bmax + k) * d + j, u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        // bookkeeping that nobody needs before the next step, after the columns (thread 0 belongs to a column wavefront)
        if (owner == b && tid == 0) { S.order[t] = p; S.err[t] = score[p - j0]; }   // exact score, not the truncated one
        if (tid == 0) { alive_bits[p >> 5] &= ~(1u << (p & 31)); pivs[k] = piv; rpivs[k] = rpiv; *gkey_min = KEY_EMPTY; *gkey_max = 0; }
        if (flag_fail) { ok = false; break; }
        if (flag_err) { error_step = 1 + t; break; }
        slot_early = participants > 0 && more_steps;
        if (owner == b) --nlive;
        ++k;
        __syncthreads();
        TICK(4);

        // ---------------------------------------------------------- 5. flush the pending downdates
        if (k == bmax || t + 1 == S.n_remove) {
            // all slices of the pending rows must be in memory before anyone reads them
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            ++bar_epoch;
            if (tid == 0) __hip_atomic_store(S.bar + b, bar_epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            {
                bool fail = false;
                for (int sb = tid; sb < nb; sb += LT) {
                    Waiter w;
                    while (__hip_atomic_load(S.bar + sb, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < bar_epoch)
                        if (!w.again(S.status)) { fail = true; break; }
                    if (fail) break;
                }
                if (fail) misc[0] = 1;
            }
            // No acquire fence: the pending rows are the only data of other workgroups read after this barrier,
            // and they are read with device-scope loads (an invalidation of the L2 here costs a third of a
            // microsecond per step, mostly in refetching this workgroup's own panel).
            __syncthreads();
            TICK(5);
            if (misc[0]) { ok = false; break; }

            // The columns alive now, listed: what the flush of this block has to touch.
            const bool listed = d <= LIST_MAX_D;
            if (listed) {
                const int nwords = (d + 31) / 32;
                if (wave == 0) {
                    int carry = 0;
                    for (int w0 = 0; w0 < nwords; w0 += 64) {
                        const int w = w0 + lane;
                        const int cnt = (w < nwords) ? __popc(alive_bits[w]) : 0;
                        int incl = cnt;
#pragma unroll
                        for (int o = 1; o < 64; o <<= 1) {
                            const int v = __shfl_up(incl, o);
                            if (lane >= o) incl += v;
                        }
                        if (w < nwords) word_prefix[w] = carry + incl - cnt;
                        carry += __shfl(incl, 63);
                    }
                    if (lane == 0) misc[7] = carry;
                }
                __syncthreads();
                for (int c = tid; c < d; c += LT) {
                    const unsigned bits = alive_bits[c >> 5];
                    if ((bits >> (c & 31)) & 1u) {
                        const int at = word_prefix[c >> 5] + __popc(bits & ((1u << (c & 31)) - 1u));
                        live_list[at] = (unsigned short)c;
                    }
                }
                __syncthreads();
            }

            flush_panel<PACKED ? 3 : (W_IN_LDS ? 1 : 2), BROWS>(P, S.U + (size_t)ublk * bmax * d, uloc, pivs, coefa, alive_own, alive_bits,
                                                         listed ? live_list : nullptr, misc[7], k, d, cp);
            k = 0;
            ublk ^= 1;
            TICK(6);
        }
    }

    // ------------------------------------------------------------------ final masking + write-back
    __syncthreads();
    ZIPLM_LAZY_TIMING_WRITE_BACK;
    // status: 1 + step for a non-positive diagonal entry, -(2 + step) when nothing was left to remove
    if (error_step < -1 && misc[2]) error_step = -error_step - 1;
    if (b == 0 && tid == 0 && error_step != 0) atomicCAS(S.status, 0, error_step);
    if (ok && error_step == 0) {
        for (int c = tid; c < d; c += LT) {
            const bool col_live = (alive_bits[c >> 5] >> (c & 31)) & 1u;
            for (int r = 0; r < nown; ++r)
                S.Hinv[(size_t)(j0 + r) * d + c] = (col_live && alive_own[r]) ? (float)P[(size_t)c * cp + r] : 0.f;
        }
        for (int jl = wave; jl < nown; jl += NW) {
            const bool a = alive_own[jl] != 0;
            for (int i = lane; i < m; i += 64) S.W[(size_t)i * d + j0 + jl] = a ? WT(jl, i) : 0.f;
        }
    }
#undef WT
}

struct Plan {
    int nb, cpb, cp, w_in_lds, pay_words, brows;
    size_t lds_bytes;
    bool feasible;
};

// pack: layers that share the launch; each gets an equal share of the compute units
static Plan make_plan(int d_row, int d_col, int pack = 1) {
    Plan p = {};
    const int cus = max(1, device_cu_count() / pack);
    p.cpb = (d_col + cus - 1) / cus;
    p.cp = (p.cpb + RG - 1) / RG * RG;
    p.nb = (d_col + p.cpb - 1) / p.cpb;
    const size_t lds_cap = 158 * 1024;
    // W in LDS if it fits beside the long block where that applies, else beside the short one, else in the workspace
    p.brows = block_rows(p.cp, d_col, true, pack);
    p.w_in_lds = lds_layout(d_row, d_col, p.cp, true, p.cpb, p.brows).total <= lds_cap ? 1 : 0;
    if (!p.w_in_lds && p.brows != BMAX_NARROW) {
        p.brows = BMAX_NARROW;
        p.w_in_lds = lds_layout(d_row, d_col, p.cp, true, p.cpb, p.brows).total <= lds_cap ? 1 : 0;
    }
    p.lds_bytes = lds_layout(d_row, d_col, p.cp, p.w_in_lds != 0, p.cpb, p.brows).total;
    p.pay_words = d_row + 2 * p.brows + 2;
    p.feasible = p.lds_bytes <= lds_cap && p.cpb <= MAX_CPB && d_col <= MAX_D;
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
    s.P = c.take<double>((size_t)p.nb * d_col * p.cp);
    s.Wt = c.take<float>(p.w_in_lds ? 1 : (size_t)d_col * padded_rows(d_row));
    s.U = c.take<double>((size_t)2 * p.brows * d_col);
    // zero-initialised region: slots, payload, barrier epochs, status
    s.slots = c.take<unsigned long long>((size_t)2 * p.nb * SLOT_STRIDE);
    s.pay = c.take<unsigned long long>((size_t)2 * p.nb * p.pay_words);
    s.bar = c.take<unsigned long long>((size_t)p.nb);
    s.status = c.take<int>(1);
    l.snap_steps = c.take<int>((size_t)(n_snap > 0 ? n_snap : 1));
    ZIPLM_LAZY_TIMING_TAKE(s, c);
    l.bytes = c.off;
    return l;
}

// ------------------------------------------------------------------------------------------------
// Exchange area: the candidate slots and the winner's payload, the two things other workgroups wait for, of one
// layer.  They live in the caller's workspace unless the caller passes a separate area (uncached device memory
// makes a store visible to the other XCDs' loads sooner than the write path of the L2: 3% of the loop).
// ------------------------------------------------------------------------------------------------
static size_t exchange_bytes_needed(const Plan &p) {
    return align_up(sizeof(unsigned long long) * (size_t)2 * p.nb * SLOT_STRIDE) + align_up(sizeof(unsigned long long) * (size_t)2 * p.nb * p.pay_words);
}

}  // namespace lazy

// Entry points used by prune.hip ------------------------------------------------------------------
bool lazy_columns_feasible(int d_row, int d_col) { return lazy::make_plan(d_row, d_col).feasible; }

size_t lazy_columns_workspace_bytes(int d_row, int d_col, int n_snap) {
    const lazy::Plan p = lazy::make_plan(d_row, d_col);
    return lazy::make_layout(d_row, d_col, n_snap, p, nullptr).bytes;
}

// Layers of one shape that one launch takes side by side when n_layers are waiting: as many as the kernel's
// argument holds, fewer while a layer's share of the compute units cannot hold its state.
int lazy_columns_pack(int n_layers, int d_row, int d_col) {
    int pack = n_layers < lazy::MAX_PACK ? n_layers : lazy::MAX_PACK;
    while (pack > 1 && !lazy::make_plan(d_row, d_col, pack).feasible) --pack;
    return pack < 1 ? 1 : pack;
}

// workspace of one launch of `pack` layers
size_t lazy_columns_pack_workspace_bytes(int pack, int d_row, int d_col, int n_snap) {
    const lazy::Plan p = lazy::make_plan(d_row, d_col, pack);
    return (size_t)pack * lazy::make_layout(d_row, d_col, n_snap, p, nullptr).bytes;
}

// bytes of a separate exchange area for one launch of `pack` layers
size_t lazy_columns_pack_exchange_bytes(int pack, int d_row, int d_col) {
    const lazy::Plan p = lazy::make_plan(d_row, d_col, pack);
    return p.feasible ? (size_t)pack * lazy::exchange_bytes_needed(p) : 0;
}

// Enqueues the whole loop of `pack` layers (layer l: W + l * stride_w, Hinv + l * stride_hinv, order_out and
// err_out + l * n_remove, W_snap + l * n_snap * d_row * d_col).  status_dev_out[l] receives the device address
// of layer l's status word.  alive_in applies to a single layer only.  exchange: nullptr (the slots and payloads
// then live in the workspace) or an area of at least lazy_columns_pack_exchange_bytes bytes.  stall_wg: -1, or the
// workgroup (of layer 0) that the self-test of the bounded waits keeps out of the loop.
int lazy_columns_launch(float *W, float *Hinv, int pack, int64_t stride_w, int64_t stride_hinv, int d_row, int d_col,
                        int n_remove, int32_t *order_out, double *err_out, const uint8_t *alive_in, int n_snap,
                        const int32_t *snap_steps_host, float *W_snap, void *workspace, void *exchange,
                        hipStream_t st, int **status_dev_out, int stall_wg) {
    using namespace lazy;
    if (pack < 1 || pack > MAX_PACK || (pack > 1 && alive_in)) return ZIPLM_ERR_INVALID_ARG;
    const Plan p = make_plan(d_row, d_col, pack);
    if (!p.feasible) return ZIPLM_ERR_UNSUPPORTED;
    const size_t layer_bytes = make_layout(d_row, d_col, n_snap, p, nullptr).bytes;
    StatePack pk = {};
    pk.nb = p.nb;
    Layout lay[MAX_PACK];
    for (int q = 0; q < pack; ++q) {
        lay[q] = make_layout(d_row, d_col, n_snap, p, static_cast<char *>(workspace) + (size_t)q * layer_bytes);
        State &S = lay[q].st;
        S.W = W + (size_t)q * stride_w; S.Hinv = Hinv + (size_t)q * stride_hinv;
        S.m = d_row; S.d = d_col; S.n_remove = n_remove;
        S.order = order_out ? order_out + (size_t)q * n_remove : nullptr;
        S.err = err_out ? err_out + (size_t)q * n_remove : nullptr;
        S.alive_in = alive_in;
        S.n_snap = n_snap; S.snap_steps = lay[0].snap_steps;
        S.W_snap = W_snap ? W_snap + (size_t)q * n_snap * d_row * d_col : nullptr;
        S.cpb = p.cpb; S.cp = p.cp; S.pay_words = p.pay_words;
        S.stall_wg = (q == 0) ? stall_wg : -1;
    }
    if (n_snap > 0) {
        // pageable source: staged before the call returns
        ZIPLM_HIP_TRY(hipMemcpyAsync(lay[0].snap_steps, snap_steps_host, sizeof(int) * (size_t)n_snap, hipMemcpyHostToDevice, st));
        ZIPLM_HIP_TRY(hipStreamSynchronize(st));
    }
    const bool xa = exchange != nullptr;
    if (xa) {
        Carver cx(exchange);
        for (int q = 0; q < pack; ++q) {
            lay[q].st.slots = cx.take<unsigned long long>((size_t)2 * p.nb * SLOT_STRIDE);
            lay[q].st.pay = cx.take<unsigned long long>((size_t)2 * p.nb * p.pay_words);
        }
        if (zero_fill(exchange, cx.off, st) != ZIPLM_OK) return ZIPLM_ERR_DEVICE;
    }
    for (int q = 0; q < pack; ++q) {
        // zero-initialised: slots, payload, barrier epochs, status (contiguous in the workspace, in this order)
        Layout ws_lay = make_layout(d_row, d_col, n_snap, p, static_cast<char *>(workspace) + (size_t)q * layer_bytes);
        char *zero_from = reinterpret_cast<char *>(xa ? (void *)ws_lay.st.bar : (void *)ws_lay.st.slots);
        if (zero_fill(zero_from, reinterpret_cast<char *>(ws_lay.snap_steps) - zero_from, st) != ZIPLM_OK) return ZIPLM_ERR_DEVICE;
        pk.s[q] = lay[q].st;
        status_dev_out[q] = lay[q].st.status;
    }
    const int variant = (p.brows == BMAX_WIDE) ? 4 : (p.w_in_lds ? 1 : 0) + (pack > 1 ? 2 : 0);
    void (*const kernels[5])(const StatePack) = {prune_lazy_kernel<false, false, BMAX_NARROW>, prune_lazy_kernel<true, false, BMAX_NARROW>,
                                                 prune_lazy_kernel<false, true, BMAX_NARROW>, prune_lazy_kernel<true, true, BMAX_NARROW>,
                                                 prune_lazy_kernel<true, false, BMAX_WIDE>};
    const void *fn = reinterpret_cast<const void *>(kernels[variant]);
    // every time: the attribute belongs to the current device's copy of the kernel, and the call costs microseconds
    ZIPLM_HIP_TRY(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    int per_cu = 0;
    ZIPLM_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernels[variant], LT, p.lds_bytes));
    if (per_cu < 1 || pack * p.nb > per_cu * device_cu_count()) return ZIPLM_ERR_DEVICE;
    void *args[] = {&pk};
    ZIPLM_HIP_TRY(hipLaunchCooperativeKernel(const_cast<void *>(fn), dim3(pack * p.nb), dim3(LT), args, (unsigned)p.lds_bytes, st));
    ZIPLM_LAZY_TIMING_REPORT(lay[0].st, p.nb, n_remove, st);
    return ZIPLM_OK;
}

}  // namespace ziplm
