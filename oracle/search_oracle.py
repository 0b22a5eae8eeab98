"""Oracle of the host-side configuration search (Section 3.2): exhaustive, slow, obviously correct.

TEST INFRASTRUCTURE: only tests may import this module.

  select(levels_time, levels_cost, budget, buckets)
      every combination of one level per layer is enumerated; a combination is admissible when the sum of its
      times, each rounded UP to a whole step of budget / buckets, is at most `buckets` steps; among the admissible
      ones the least total cost wins.  Returns (choice, cost, time) or None.
  mutate(levels_time, levels_prior, budget, buckets, uniforms, mutate_prob, score)
      the outer loop exactly as the section describes it: coefficients c_l (all 1 at the start), per step every
      coefficient is redrawn with probability mutate_prob, the configuration of least sum c_l * p[l][s] is selected,
      scored, and kept if not worse.  The random numbers come in as `uniforms[step][layer] = (decision, value)`.

The readings this oracle shares with the library (the paper defers to the SPDY method for them): start at 1, a redrawn
coefficient is 1 - value (uniform in (0, 1]), a trial with an equal score replaces the incumbent.
"""
import itertools
import math


def _steps(t, budget, buckets):
    step = budget / buckets
    s = int(t / step)
    while s * step < t:
        s += 1
    return s


def select(levels_time, levels_cost, budget, buckets):
    best = None
    for choice in itertools.product(*[range(len(t)) for t in levels_time]):
        used = sum(_steps(levels_time[l][s], budget, buckets) for l, s in enumerate(choice))
        if used > buckets:
            continue
        cost = math.fsum(levels_cost[l][s] for l, s in enumerate(choice))
        if best is None or cost < best[1]:
            best = (choice, cost)
    if best is None:
        return None
    choice, cost = best
    return list(choice), cost, math.fsum(levels_time[l][s] for l, s in enumerate(choice))


def mutate(levels_time, levels_prior, budget, buckets, uniforms, mutate_prob, score):
    n = len(levels_time)
    coef = [1.0] * n

    def configure(c):
        r = select(levels_time, [[c[l] * p for p in levels_prior[l]] for l in range(n)], budget, buckets)
        return None if r is None else r[0]

    choice = configure(coef)
    if choice is None:
        return None
    best = score(choice)
    for u in uniforms:
        trial = [(1.0 - u[l][1]) if u[l][0] < mutate_prob else coef[l] for l in range(n)]
        cand = configure(trial)
        sc = score(cand)
        if sc <= best:
            best, coef, choice = sc, trial, cand
    return choice, coef, best
