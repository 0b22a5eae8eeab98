// Host-side search for a per-layer sparsity configuration under a runtime budget (Section 3.2, "Finding the optimal
// sparsity configuration" and "Structured SPDY search").  Plain C++, no device work: the greedy loop has produced, for
// every layer, a database of pruned versions (levels) with their priors p_s; a latency table gives every level's
// runtime.  A configuration picks one level per layer.
//
//   ziplm_search_select   exact minimiser of  sum_l cost[l][s_l]  subject to  sum_l time[l][s_l] <= budget,
//                         by dynamic programming over the layers on a time axis of `buckets` equal steps; every
//                         level's time is rounded UP to whole steps, so whatever is returned meets the budget
//                         in the unrounded times as well (the section's "any candidate ... actually achieves the
//                         target speedup").
//   ziplm_search_mutate   the outer loop: cost[l][s] = c_l * p[l][s] with one sensitivity coefficient c_l per layer;
//                         for a fixed number of steps (the paper: 1000) every coefficient is redrawn with probability
//                         `mutate_prob` (the paper: 10% in expectation), the dynamic programme picks the configuration,
//                         the caller's callback scores it (lower is better, e.g. the calibration loss of the stitched
//                         model), and the mutation is kept if the score did not get worse.
//
// The paper refers to the SPDY method for everything it does not restate; this file takes these readings, all of them
// arguments or documented here: the coefficients start at 1 and a mutated coefficient is a fresh uniform number in (0, 1];
// ties in the dynamic programme go to the lower level index (less pruning first: levels are ordered by sparsity);
// a step whose candidate does not fit the budget at all cannot occur (level 0 of every layer must fit, else an error).
// Random numbers are the caller's: two uniforms in [0, 1) per step and layer, so that results can be reproduced.
#include <stdint.h>

#include <limits>
#include <vector>

#include "ziplm.h"

namespace {

struct Levels {
    int n_layers;
    const int32_t *n_levels;
    std::vector<int64_t> offset;     // first level of layer l in the flat arrays
    int64_t total;
};

bool make_levels(int n_layers, const int32_t *n_levels, Levels &L) {
    if (n_layers <= 0 || !n_levels) return false;
    L.n_layers = n_layers;
    L.n_levels = n_levels;
    L.offset.assign((size_t)n_layers + 1, 0);
    for (int l = 0; l < n_layers; ++l) {
        if (n_levels[l] <= 0) return false;
        L.offset[l + 1] = L.offset[l] + n_levels[l];
    }
    L.total = L.offset[n_layers];
    return true;
}

// steps[i] = time of flat level i in whole steps of budget / buckets, rounded up; -1 if it exceeds the budget alone
void time_steps(const Levels &L, const double *time, double budget, int buckets, std::vector<int> &steps) {
    const double step = budget / buckets;
    steps.resize((size_t)L.total);
    for (int64_t i = 0; i < L.total; ++i) {
        const double t = time[i];
        if (!(t >= 0.0) || t > budget) { steps[i] = -1; continue; }
        int s = (int)(t / step);
        while ((double)s * step < t) ++s;            // ceil, robust against the division's rounding
        steps[i] = s > buckets ? -1 : s;
    }
}

// The dynamic programme.  best[l][b] = least cost of layers 0..l-1 using at most b steps.  Returns false if nothing fits.
bool select(const Levels &L, const std::vector<int> &steps, const double *cost, int buckets, int32_t *choice,
            double *cost_out) {
    const double inf = std::numeric_limits<double>::infinity();
    const int nl = L.n_layers, nb = buckets + 1;
    std::vector<double> best((size_t)(nl + 1) * nb, inf);
    std::vector<int32_t> arg((size_t)nl * nb, -1);
    for (int b = 0; b < nb; ++b) best[b] = 0.0;
    for (int l = 0; l < nl; ++l) {
        const double *prev = &best[(size_t)l * nb];
        double *cur = &best[(size_t)(l + 1) * nb];
        for (int s = 0; s < L.n_levels[l]; ++s) {
            const int64_t i = L.offset[l] + s;
            const int st = steps[i];
            if (st < 0) continue;
            const double c = cost[i];
            for (int b = st; b < nb; ++b) {
                const double v = prev[b - st] + c;
                if (v < cur[b]) { cur[b] = v; arg[(size_t)l * nb + b] = s; }     // strict: the lower level keeps a tie
            }
        }
    }
    if (!(best[(size_t)nl * nb + buckets] < inf)) return false;
    int b = buckets;
    for (int l = nl - 1; l >= 0; --l) {
        const int s = arg[(size_t)l * nb + b];
        choice[l] = s;
        b -= steps[L.offset[l] + s];
    }
    if (cost_out) *cost_out = best[(size_t)nl * nb + buckets];
    return true;
}

}  // namespace

extern "C" int ziplm_search_select(int n_layers, const int32_t *n_levels_host, const double *time_host,
                                   const double *cost_host, double budget, int buckets, int32_t *choice_out_host,
                                   double *cost_out_host, double *time_out_host) {
    Levels L;
    if (!make_levels(n_layers, n_levels_host, L) || !time_host || !cost_host || !choice_out_host) return ZIPLM_ERR_INVALID_ARG;
    if (!(budget > 0.0) || buckets < 1 || buckets > (1 << 24)) return ZIPLM_ERR_INVALID_ARG;
    for (int64_t i = 0; i < L.total; ++i)
        if (!(cost_host[i] >= 0.0) || !(time_host[i] >= 0.0)) return ZIPLM_ERR_INVALID_ARG;
    std::vector<int> steps;
    time_steps(L, time_host, budget, buckets, steps);
    if (!select(L, steps, cost_host, buckets, choice_out_host, cost_out_host)) return ZIPLM_ERR_UNSUPPORTED;   // nothing fits
    if (time_out_host) {
        double t = 0.0;
        for (int l = 0; l < n_layers; ++l) t += time_host[L.offset[l] + choice_out_host[l]];
        *time_out_host = t;
    }
    return ZIPLM_OK;
}

extern "C" int ziplm_search_mutate(int n_layers, const int32_t *n_levels_host, const double *time_host,
                                   const double *prior_host, double budget, int buckets, int n_steps,
                                   double mutate_prob, const double *uniform_host,
                                   ziplm_score_fn score, void *user,
                                   int32_t *choice_out_host, double *coef_out_host, double *score_out_host) {
    Levels L;
    if (!make_levels(n_layers, n_levels_host, L) || !time_host || !prior_host || !choice_out_host || !score) return ZIPLM_ERR_INVALID_ARG;
    if (!(budget > 0.0) || buckets < 1 || buckets > (1 << 24) || n_steps < 0 || !(mutate_prob >= 0.0 && mutate_prob <= 1.0))
        return ZIPLM_ERR_INVALID_ARG;
    if (n_steps > 0 && !uniform_host) return ZIPLM_ERR_INVALID_ARG;
    for (int64_t i = 0; i < L.total; ++i)
        if (!(prior_host[i] >= 0.0) || !(time_host[i] >= 0.0)) return ZIPLM_ERR_INVALID_ARG;
    std::vector<int> steps;
    time_steps(L, time_host, budget, buckets, steps);
    std::vector<double> coef((size_t)n_layers, 1.0), trial((size_t)n_layers), cost((size_t)L.total);
    std::vector<int32_t> cand((size_t)n_layers);
    auto configure = [&](const std::vector<double> &c, int32_t *out) {
        for (int l = 0; l < n_layers; ++l)
            for (int s = 0; s < n_levels_host[l]; ++s) cost[L.offset[l] + s] = c[l] * prior_host[L.offset[l] + s];
        return select(L, steps, cost.data(), buckets, out, nullptr);
    };
    if (!configure(coef, choice_out_host)) return ZIPLM_ERR_UNSUPPORTED;
    double best = score(choice_out_host, user);
    for (int t = 0; t < n_steps; ++t) {
        const double *u = uniform_host + (size_t)t * n_layers * 2;
        trial = coef;
        for (int l = 0; l < n_layers; ++l)
            if (u[2 * l] < mutate_prob) trial[l] = 1.0 - u[2 * l + 1];            // uniform in (0, 1]
        if (!configure(trial, cand.data())) return ZIPLM_ERR_UNSUPPORTED;
        const double sc = score(cand.data(), user);
        if (sc <= best) {
            best = sc;
            coef = trial;
            for (int l = 0; l < n_layers; ++l) choice_out_host[l] = cand[l];
        }
    }
    if (coef_out_host) for (int l = 0; l < n_layers; ++l) coef_out_host[l] = coef[l];
    if (score_out_host) *score_out_host = best;
    return ZIPLM_OK;
}
