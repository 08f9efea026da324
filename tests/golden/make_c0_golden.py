"""Writes tests/golden/c0_golden.json: tokens, accept lengths and iteration
count of the oracle on workload C0 (the tiny toy problem).  Calls only the CPU
oracle and the seeded input generator; run from the repository root:

    python tests/golden/make_c0_golden.py

The stored values are a regression fixture for the oracle itself (the paper
prints no worked example); they were frozen after the closed-form and
statistical pins in tests/test_oracle_*.py passed.
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import scd                                   # noqa: E402
from paper_2510_24211_amd import workload as wl          # noqa: E402


def run():
    w = wl.WORKLOADS["C0"]
    toy = wl.ToyLogits(w)
    cfg = scd.ScdConfig(B=w.B, L=w.L, N=w.N, V=w.V, seed=w.seed)

    def model(b, i, Lw, toks, t, age):
        return np.stack([toy.table[b, i + s, min(int(age[s]), w.age_cap)] for s in range(Lw)])
    o = scd.decode(cfg, model)
    return dict(workload="C0", tokens=[int(x) for x in o.out[0]],
                accept_len=[int(a) for a in o.accept_hist[0]], nfe=int(o.t[0]))


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c0_golden.json")
    with open(path, "w") as f:
        json.dump(run(), f, indent=1)
    print("wrote", path)
