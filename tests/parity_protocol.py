"""GPU-vs-oracle comparison protocol for the greedy loop (helper, not a test module).

Algorithm 1 is a greedy heuristic, so the removal order has to be reproduced step by step; given
the removed set, W, Hinv and the cumulative error are unique.  Two exact-arithmetic ties (or
scores closer than fp32 inputs can resolve) may legitimately be taken in either order, hence:

  1. walk the steps; where the orders differ the oracle's relative score gap at that step must
     be <= ORDER_GAP (1e-6), otherwise fail;
  2. after an accepted difference the oracle is re-run in forced-order mode on the GPU's order,
     so later steps are compared on the same trajectory, and the forced choice must be within
     (1 + ORDER_GAP) of the oracle's own best score at every step;
  3. per-step errors agree to REL_TOL (1e-4) relative;
  4. matrices (W, its snapshots, the surviving inverse Hessian) are compared COLUMN BY COLUMN
     (assert_columns_close): every live column within REL_TOL of the oracle's in relative
     Euclidean norm, every removed column exactly zero.  One norm over the whole matrix would let
     a single wrong column among thousands pass.
"""
import numpy as np

ORDER_GAP = 1e-6
REL_TOL = 1e-4


def compare_run(oracle, W32, Hinv32, group_size, n_remove, order_gpu, err_gpu, alive=None, snap_steps=None):
    """Returns the oracle result (forced onto the GPU's order if that was needed and allowed).
    Raises AssertionError with a description on any violation."""
    order_gpu = np.asarray(order_gpu)
    err_gpu = np.asarray(err_gpu, dtype=np.float64)
    free = oracle.prune(W32, Hinv32, group_size, n_remove, alive=alive, snap_steps=snap_steps)
    ref = free
    diff = np.nonzero(free["order"] != order_gpu)[0]
    forced = False
    first_diff = None
    if len(diff):
        t = int(diff[0])
        first_diff = (t, float(free["gap"][t]))
        assert free["gap"][t] <= ORDER_GAP, (
            "removal order differs at step %d (gpu %d, oracle %d) where the oracle's gap is %.3e > %.0e"
            % (t, order_gpu[t], free["order"][t], free["gap"][t], ORDER_GAP))
        assert sorted(order_gpu.tolist()) == sorted(set(order_gpu.tolist())), "gpu order repeats a structure"
        ref = oracle.prune(W32, Hinv32, group_size, n_remove, alive=alive, forced=order_gpu.astype(np.int32),
                           snap_steps=snap_steps)
        forced = True
        worst = (ref["err"] / ref["best"]).max()
        assert worst <= 1.0 + ORDER_GAP, "forced gpu choice is %.3e above the oracle's best score" % (worst - 1.0)
    rel = np.abs(err_gpu - ref["err"]) / np.abs(ref["err"])
    assert rel.max() <= REL_TOL, "err differs: max rel %.3e at step %d" % (rel.max(), int(rel.argmax()))
    ref["forced"] = forced
    ref["first_diff"] = first_diff          # (step, oracle's gap there) of the first accepted difference, or None
    ref["min_gap"] = float(free["gap"][:max(n_remove - 1, 0)].min()) if n_remove > 1 else float("inf")
    ref["err_rel_max"] = float(rel.max())
    return ref


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    nb = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / nb) if nb > 0 else float(np.linalg.norm(a))


def column_errors(got, want):
    """Per column j: ||got[:, j] - want[:, j]|| / ||want[:, j]|| for the columns the oracle keeps
    (non-zero in `want`); returns (rel array over live columns, live mask)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, "shape %s vs %s" % (got.shape, want.shape)
    nw = np.linalg.norm(want, axis=0)
    live = nw > 0.0
    rel = np.linalg.norm(got[:, live] - want[:, live], axis=0) / nw[live]
    return rel, live


def assert_columns_close(got, want, what, tol=REL_TOL):
    """Eq. 3 / Eq. 4 parity: every column the oracle keeps agrees to `tol` in relative Euclidean norm,
    every column the oracle has zeroed is exactly zero.  Returns the worst relative column error."""
    rel, live = column_errors(got, want)
    got = np.asarray(got)
    assert np.all(got[:, ~live] == 0.0), "%s: a removed column is not exactly zero" % what
    if rel.size == 0:
        return 0.0
    j = int(np.argmax(rel))
    assert rel[j] <= tol, "%s: live column #%d (of %d) off by %.3e relative (bar %.0e)" % (
        what, j, rel.size, rel[j], tol)
    return float(rel[j])
