"""Writes tests/golden/oracle_small_cases.json from the CPU oracle alone.

Run from the repository root:  python tests/golden/make_golden.py
The stored values are the oracle's removal order, per-step errors (Eq. 2) and damping for a
few small seeded layers; they serve as a regression guard for the oracle itself.  The paper
prints no worked numbers for Algorithm 1, so there is nothing of the paper's to store here.
"""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import ziplm_oracle as oracle                      # noqa: E402
from paper_2302_04089_amd import workloads                      # noqa: E402

SPECS = [  # d_row, d_col, group, n_tok, x_kind, seed
    (6, 24, 1, 96, "gelu", 0),
    (5, 32, 4, 128, "scaled_normal", 1),
    (3, 16, 16, 64, "normal", 2),
]


def main():
    out = []
    for s in SPECS:
        spec = workloads.small(*s[:4], x_kind=s[4], seed=s[5])
        X = workloads.make_X(spec)
        W = workloads.make_W(spec)
        H = oracle.hessian(X, 2.0)
        Hi, lam = oracle.hinv(H, spec.damp_rel)
        r = oracle.prune(W, Hi, spec.group_size, spec.n_groups)
        out.append({"spec": list(s), "lambda": lam, "order": r["order"].tolist(),
                    "err": [float(e) for e in r["err"]]})
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_small_cases.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    main()
