/*
 * ziplm_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain, slow, double-precision CPU statement of the layer-wise structured
 * Optimal-Brain-Surgeon pruner of ZipLM (Section 3.1, Eq. 1-4, Algorithm 1).
 * It exists so that the GPU library can be checked against something that can
 * be read against the paper by eye.  It shares no code with the GPU library,
 * uses no BLAS/LAPACK, and does no blocking or fusion: every function below is
 * the formula it cites written out as loops.  OpenMP "parallel for" over
 * independent rows is the only concession to run time.
 *
 * Only tests, the smoke check and the CPU-baseline leg of the benchmark may
 * load this file's shared object.
 *
 * Conventions (Section 3.1, "Problem formulation"):
 *   W  : d_row x d_col, row-major; a structure is a set of COLUMNS of W.
 *   X  : d_col x n_tok, row-major (one row per input feature).
 *   H  : d_col x d_col, row-major, symmetric positive definite.
 *   group s (0-based) = columns [s*g, (s+1)*g)   ("Pruned structures": d_head
 *   consecutive columns of the attention out-matrix, single columns of FC2).
 *
 * Readings of points the paper leaves open are listed next to the code that
 * takes them.
 *
 * Pins: every exported function is checked in tests/test_oracle_pins.py against
 * brute-force least squares, fresh inverses of the surviving sub-Hessian,
 * closed forms and special cases; none is "parity unpinned".
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#include <stdint.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_INVALID_ARG (-1)
#define ORACLE_ERR_NOT_PD (-2)

/* Number of threads the OpenMP loops below will use (for reporting timings). */
int ziplm_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------ */
/* H <- H + scale * X X^T                                                    */
/* Section 3.1 "Saliency scores and weight update" defines H = X X^T; the    */
/* caption of Algorithm 1 uses 2 X X^T.  `scale` carries that factor.        */
/* H_ij = scale * sum_k X_ik X_jk is symmetric in (i,j), so the lower        */
/* triangle is summed and copied to the upper one.                           */
/* ------------------------------------------------------------------------ */
int ziplm_oracle_hessian(double *H, const double *X, int d_col, int64_t n_tok,
                         double scale)
{
    if (!H || !X || d_col <= 0 || n_tok < 0) return ORACLE_ERR_INVALID_ARG;
    #pragma omp parallel for schedule(dynamic, 4)
    for (int i = 0; i < d_col; ++i) {
        const double *xi = X + (size_t)i * n_tok;
        for (int j = 0; j <= i; ++j) {
            const double *xj = X + (size_t)j * n_tok;
            double s = 0.0;
            for (int64_t k = 0; k < n_tok; ++k) s += xi[k] * xj[k];
            H[(size_t)i * d_col + j] += scale * s;
        }
    }
    for (int i = 0; i < d_col; ++i)
        for (int j = 0; j < i; ++j)
            H[(size_t)j * d_col + i] = H[(size_t)i * d_col + j];
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------ */
/* Cholesky A = L L^T of an n x n matrix with leading dimension lda, lower   */
/* triangle of A read, L written to the lower triangle of L (ld = ldl).      */
/* Returns 0, or 1+j if pivot j is not positive.  Plain column-by-column     */
/* (Cholesky-Banachiewicz) recurrences.                                      */
/* ------------------------------------------------------------------------ */
static int cholesky_lower(const double *A, int lda, double *L, int ldl, int n,
                          int parallel)
{
    for (int j = 0; j < n; ++j) {
        double s = A[(size_t)j * lda + j];
        for (int k = 0; k < j; ++k) s -= L[(size_t)j * ldl + k] * L[(size_t)j * ldl + k];
        if (!(s > 0.0)) return 1 + j;
        const double ljj = sqrt(s);
        L[(size_t)j * ldl + j] = ljj;
        #pragma omp parallel for schedule(static) if (parallel && n - j > 256)
        for (int i = j + 1; i < n; ++i) {
            double t = A[(size_t)i * lda + j];
            for (int k = 0; k < j; ++k) t -= L[(size_t)i * ldl + k] * L[(size_t)j * ldl + k];
            L[(size_t)i * ldl + j] = t / ljj;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Hinv = (H + lambda I)^-1 with lambda = damp_rel * mean(diag H).           */
/* Algorithm 1's caption gives H^-1 = (2XX^T + lambda I)^-1 without a value  */
/* for lambda or a method; reading: lambda relative to the mean diagonal,    */
/* inverse through the Cholesky factor: H+lambda I = L L^T, T = L^-1,        */
/* Hinv = T^T T.  T is held transposed (Tt[c][k] = T[k][c]) so that the dot  */
/* products run over contiguous memory.                                      */
/* *info = 0, or the 0-based index of the first non-positive pivot.          */
/* ------------------------------------------------------------------------ */
int ziplm_oracle_hinv(const double *H, double *Hinv, int d_col, double damp_rel,
                      double *lambda_out, int *info)
{
    if (!H || !Hinv || d_col <= 0) return ORACLE_ERR_INVALID_ARG;
    const int d = d_col;
    double tr = 0.0;
    for (int i = 0; i < d; ++i) tr += H[(size_t)i * d + i];
    const double lambda = damp_rel * (tr / d);
    if (lambda_out) *lambda_out = lambda;
    if (info) *info = 0;

    double *A = (double *)malloc(sizeof(double) * (size_t)d * d);
    double *L = (double *)calloc((size_t)d * d, sizeof(double));
    double *Tt = (double *)calloc((size_t)d * d, sizeof(double));
    if (!A || !L || !Tt) { free(A); free(L); free(Tt); return ORACLE_ERR_INVALID_ARG; }
    memcpy(A, H, sizeof(double) * (size_t)d * d);
    for (int i = 0; i < d; ++i) A[(size_t)i * d + i] += lambda;

    int bad = cholesky_lower(A, d, L, d, d, 1);
    if (bad) {
        if (info) *info = bad - 1;
        free(A); free(L); free(Tt);
        return ORACLE_ERR_NOT_PD;
    }
    /* forward substitution L T = I, one column c of T at a time */
    #pragma omp parallel for schedule(dynamic, 8)
    for (int c = 0; c < d; ++c) {
        double *t = Tt + (size_t)c * d;            /* t[k] = T[k][c], zero for k < c */
        for (int i = c; i < d; ++i) {
            double s = (i == c) ? 1.0 : 0.0;
            for (int k = c; k < i; ++k) s -= L[(size_t)i * d + k] * t[k];
            t[i] = s / L[(size_t)i * d + i];
        }
    }
    /* Hinv_ab = sum_k T_ka T_kb, k >= max(a,b) */
    #pragma omp parallel for schedule(dynamic, 8)
    for (int a = 0; a < d; ++a) {
        for (int b = 0; b <= a; ++b) {
            double s = 0.0;
            for (int k = a; k < d; ++k) s += Tt[(size_t)a * d + k] * Tt[(size_t)b * d + k];
            Hinv[(size_t)a * d + b] = s;
        }
    }
    for (int a = 0; a < d; ++a)
        for (int b = 0; b < a; ++b) Hinv[(size_t)b * d + a] = Hinv[(size_t)a * d + b];
    free(A); free(L); free(Tt);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------ */
/* Score of one structure, Eq. 2:                                            */
/*   sum_i W_{i,S} ((Hinv)_{S,S})^-1 W_{i,S}^T                               */
/* with (Hinv)_{S,S} = Ls Ls^T factored once per structure and reused for    */
/* every row (last paragraph before "Pruned structures"): for each row,      */
/* y = Ls^-1 w^T by forward substitution and the row's term is y.y.          */
/* The printed upper bound d_row of the sum is read as "all d_row rows".     */
/* Returns 0, or nonzero if the block is not positive definite.              */
/* ------------------------------------------------------------------------ */
static int structure_score(const double *W, const double *Hinv, int d_row, int d_col,
                           int g, int s, double *Ls, double *y, double *score)
{
    const int c0 = s * g;
    if (cholesky_lower(Hinv + (size_t)c0 * d_col + c0, d_col, Ls, g, g, 0)) return 1;
    double total = 0.0;
    for (int i = 0; i < d_row; ++i) {
        const double *w = W + (size_t)i * d_col + c0;
        for (int a = 0; a < g; ++a) {
            double t = w[a];
            for (int b = 0; b < a; ++b) t -= Ls[(size_t)a * g + b] * y[b];
            y[a] = t / Ls[(size_t)a * g + a];
            total += y[a] * y[a];
        }
    }
    *score = total;
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Algorithm 1.                                                              */
/*                                                                           */
/* W (d_row x d_col) and Hinv (d_col x d_col) are updated in place.          */
/* alive_in   : optional uint8[G], G = d_col/g; groups with 0 are treated as */
/*              already removed (their W columns / Hinv rows+columns must    */
/*              already be consistent, i.e. zero).                           */
/* forced     : optional int[n_remove]; when given, step t removes           */
/*              forced[t] instead of the argmin (used to follow another      */
/*              implementation through a near-tie).                          */
/* order_out  : int[n_remove]   removed group per step.                      */
/* err_out    : double[n_remove] Eq. 2 score of the removed group.           */
/* best_out   : optional double[n_remove] smallest score among live groups   */
/*              at that step (== err_out when not forced).                   */
/* gap_out    : optional double[n_remove] (second smallest - smallest) /     */
/*              smallest at that step; +inf when one group is left.          */
/* snapshots  : after snap_steps[i] removals W is copied to                  */
/*              W_snap + i*d_row*d_col (the per-layer database of Section    */
/*              3.2 comes out of one run this way).                          */
/*                                                                           */
/* Readings:                                                                 */
/*  - ties in the argmin go to the lowest group index (strict < scan).       */
/*  - Eq. 3 and Eq. 4 of one step both use the rows Hinv_{S,:} as they were  */
/*    BEFORE that step's updates; they are copied out first.                 */
/*  - after the updates the removed columns of W and the removed rows and    */
/*    columns of Hinv are zero in exact arithmetic; they are set to exactly  */
/*    zero here at once, which is the algorithm's final masking line applied */
/*    early, and removed groups take no further part in the argmin.          */
/* ------------------------------------------------------------------------ */
int ziplm_oracle_prune(double *W, double *Hinv, int d_row, int d_col, int g,
                       int n_remove, const uint8_t *alive_in, const int32_t *forced,
                       int32_t *order_out, double *err_out, double *best_out,
                       double *gap_out, int n_snap, const int32_t *snap_steps,
                       double *W_snap)
{
    if (!W || !Hinv || d_row <= 0 || d_col <= 0 || g <= 0 || d_col % g) return ORACLE_ERR_INVALID_ARG;
    const int G = d_col / g;
    if (n_remove < 0 || n_remove > G || !order_out || !err_out) return ORACLE_ERR_INVALID_ARG;
    if (n_snap < 0 || (n_snap > 0 && (!snap_steps || !W_snap))) return ORACLE_ERR_INVALID_ARG;
    const size_t d = (size_t)d_col;
    int rc = ORACLE_OK;

    uint8_t *alive = (uint8_t *)malloc((size_t)G);
    double *score = (double *)malloc(sizeof(double) * (size_t)G);
    int *bad = (int *)calloc((size_t)G, sizeof(int));
    double *Lp = (double *)malloc(sizeof(double) * (size_t)g * g);   /* factor of Hinv_PP   */
    double *B = (double *)malloc(sizeof(double) * (size_t)g * g);    /* (Hinv_PP)^-1        */
    double *R = (double *)malloc(sizeof(double) * (size_t)g * d);    /* Hinv_{P,:} pre-step */
    double *CW = (double *)malloc(sizeof(double) * (size_t)d_row * g);
    double *CH = (double *)malloc(sizeof(double) * d * (size_t)g);
    int n_alive = 0;
    for (int s = 0; s < G; ++s) { alive[s] = alive_in ? (alive_in[s] != 0) : 1; n_alive += alive[s]; }
    if (n_remove > n_alive) rc = ORACLE_ERR_INVALID_ARG;

    /* snapshots requested "after 0 removals" */
    for (int q = 0; rc == ORACLE_OK && q < n_snap; ++q)
        if (snap_steps[q] == 0) memcpy(W_snap + (size_t)q * d_row * d, W, sizeof(double) * d_row * d);

    for (int t = 0; rc == ORACLE_OK && t < n_remove; ++t) {
        /* --- Eq. 2 for every remaining structure ------------------------ */
        #pragma omp parallel
        {
            double *Ls = (double *)malloc(sizeof(double) * (size_t)g * g);
            double *y = (double *)malloc(sizeof(double) * (size_t)g);
            #pragma omp for schedule(static)
            for (int s = 0; s < G; ++s) {
                if (!alive[s]) continue;
                bad[s] = structure_score(W, Hinv, d_row, d_col, g, s, Ls, y, &score[s]);
            }
            free(Ls); free(y);
        }
        /* --- argmin over the remaining structures ----------------------- */
        int p = -1, failed = 0;
        double best = INFINITY, second = INFINITY;
        for (int s = 0; s < G; ++s) {
            if (!alive[s]) continue;
            if (bad[s]) { failed = 1; break; }
            if (score[s] < best) { second = best; best = score[s]; p = s; }
            else if (score[s] < second) second = score[s];
        }
        if (failed || p < 0) { rc = ORACLE_ERR_NOT_PD; break; }
        if (forced) {
            p = forced[t];
            if (p < 0 || p >= G || !alive[p]) { rc = ORACLE_ERR_INVALID_ARG; break; }
        }
        order_out[t] = p;
        err_out[t] = score[p];
        if (best_out) best_out[t] = best;
        if (gap_out) gap_out[t] = (second - best) / best;

        /* --- B = (Hinv_PP)^-1 via its Cholesky factor -------------------- */
        const size_t c0 = (size_t)p * g;
        if (cholesky_lower(Hinv + c0 * d + c0, d_col, Lp, g, g, 0)) { rc = ORACLE_ERR_NOT_PD; break; }
        for (int c = 0; c < g; ++c) {
            /* column c of B: solve Lp z = e_c, then Lp^T b = z */
            double *b = CH;                 /* borrow g doubles of scratch */
            for (int a = 0; a < g; ++a) {
                double s = (a == c) ? 1.0 : 0.0;
                for (int k = 0; k < a; ++k) s -= Lp[(size_t)a * g + k] * b[k];
                b[a] = s / Lp[(size_t)a * g + a];
            }
            for (int a = g - 1; a >= 0; --a) {
                double s = b[a];
                for (int k = a + 1; k < g; ++k) s -= Lp[(size_t)k * g + a] * b[k];
                b[a] = s / Lp[(size_t)a * g + a];
            }
            for (int a = 0; a < g; ++a) B[(size_t)a * g + c] = b[a];
        }
        /* --- pre-step copies: R = Hinv_{P,:} ; CW = W_{:,P} B ; CH = Hinv_{:,P} B */
        for (int a = 0; a < g; ++a) memcpy(R + (size_t)a * d, Hinv + (c0 + a) * d, sizeof(double) * d);
        for (int i = 0; i < d_row; ++i)
            for (int c = 0; c < g; ++c) {
                double s = 0.0;
                for (int a = 0; a < g; ++a) s += W[(size_t)i * d + c0 + a] * B[(size_t)a * g + c];
                CW[(size_t)i * g + c] = s;
            }
        for (size_t i = 0; i < d; ++i)
            for (int c = 0; c < g; ++c) {
                double s = 0.0;
                for (int a = 0; a < g; ++a) s += Hinv[i * d + c0 + a] * B[(size_t)a * g + c];
                CH[i * g + c] = s;
            }
        /* --- Eq. 3: W <- W - W_{:,P} B Hinv_{P,:} ------------------------- */
        #pragma omp parallel for schedule(static)
        for (int i = 0; i < d_row; ++i)
            for (int c = 0; c < g; ++c) {
                const double f = CW[(size_t)i * g + c];
                const double *r = R + (size_t)c * d;
                double *w = W + (size_t)i * d;
                for (size_t j = 0; j < d; ++j) w[j] -= f * r[j];
            }
        /* --- Eq. 4: Hinv <- Hinv - Hinv_{:,P} B Hinv_{P,:} ---------------- */
        /* rows of removed groups are identically zero and stay zero: skip   */
        #pragma omp parallel for schedule(static)
        for (int i = 0; i < d_col; ++i) {
            if (!alive[i / g]) continue;
            for (int c = 0; c < g; ++c) {
                const double f = CH[(size_t)i * g + c];
                const double *r = R + (size_t)c * d;
                double *h = Hinv + (size_t)i * d;
                for (size_t j = 0; j < d; ++j) h[j] -= f * r[j];
            }
        }
        /* --- R <- R - {S}; masking line of Algorithm 1 applied now -------- */
        alive[p] = 0;
        for (int i = 0; i < d_row; ++i)
            for (int a = 0; a < g; ++a) W[(size_t)i * d + c0 + a] = 0.0;
        for (int a = 0; a < g; ++a)
            for (size_t j = 0; j < d; ++j) { Hinv[(c0 + a) * d + j] = 0.0; Hinv[j * d + c0 + a] = 0.0; }

        for (int q = 0; q < n_snap; ++q)
            if (snap_steps[q] == t + 1) memcpy(W_snap + (size_t)q * d_row * d, W, sizeof(double) * d_row * d);
    }
    free(alive); free(score); free(bad); free(Lp); free(B); free(R); free(CW); free(CH);
    return rc;
}

/* ------------------------------------------------------------------------ */
/* Layer-wise error of dropping a whole module ("Pruned structures": a      */
/* whole attention or feed-forward module may be removed): every column is  */
/* pruned and nothing is left to compensate, so the error of Eq. 1, in the   */
/* quadratic form the pruner uses, is                                       */
/*   sum_i W_i (H + lambda I) W_i^T  =  tr(W (H + lambda I) W^T).            */
/* With H = scale * X X^T and lambda = 0 this is scale * ||W X||_F^2, the    */
/* squared denominator of the prior p_s (Section 3.2).                       */
/* Written as the double sum it is; rows are independent.                    */
/* ------------------------------------------------------------------------ */
int ziplm_oracle_module_error(const double *W, const double *H, int d_row, int d_col,
                              double lambda, double *err_out)
{
    if (!W || !H || !err_out || d_row <= 0 || d_col <= 0) return ORACLE_ERR_INVALID_ARG;
    const size_t d = (size_t)d_col;
    double total = 0.0;
    #pragma omp parallel for schedule(static) reduction(+ : total)
    for (int i = 0; i < d_row; ++i) {
        const double *w = W + (size_t)i * d;
        double row = 0.0;
        for (size_t j = 0; j < d; ++j) {
            double hw = lambda * w[j];                    /* ((H + lambda I) w^T)_j */
            for (size_t k = 0; k < d; ++k) hw += H[j * d + k] * w[k];
            row += w[j] * hw;
        }
        total += row;
    }
    *err_out = total;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------ */
/* Prior of Section 3.2 ("Structured SPDY search"):                          */
/*   p_s = ||W_s X - W X|| / ||W X||                                        */
/* for the layer after its first t+1 removals.  The squared numerator is the */
/* layer-wise error of the pruned layer, which is the running sum of the     */
/* per-step errors of Algorithm 1 (the cross terms vanish because each       */
/* intermediate W is the least-squares optimum on its support); the squared  */
/* denominator is the whole-module error above.  The text calls p_s a        */
/* "squared error" but prints a ratio of norms; reading: the printed ratio,  */
/* i.e. the square root of the ratio of the quadratic forms, measured with   */
/* the same (dampened) H the pruner works with.  A fully dropped layer gives */
/* 1, as the text says.                                                      */
/* ------------------------------------------------------------------------ */
int ziplm_oracle_prior(const double *err, int n, double total, double *prior_out)
{
    if (n < 0 || (n > 0 && (!err || !prior_out)) || !(total > 0.0)) return ORACLE_ERR_INVALID_ARG;
    double run = 0.0;
    for (int t = 0; t < n; ++t) {
        run += err[t];
        prior_out[t] = sqrt(run / total);
    }
    return ORACLE_OK;
}
