"""Writes tests/golden/cfg1_oracle.json: the states and residual history of the smallest benchmark workload
(dense q=8, N=16, m=4, two levels, F-relaxation, 4 cycles, seed 0) as the CPU oracle computes them, plus the
adjoint solve and parameter gradient about those states.  Calls only the input generator and oracle/;
run from the repository root:  python tests/golden/make_cfg1_oracle.py"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import mgrit_inputs as I                      # noqa: E402
from oracle import mgrit_oracle as O          # noqa: E402


def compute():
    wl = I.cfg1()
    d = I.generate(wl)
    U, hist, it = O.fas_forward(d["W"], d["b"], d["u0"], wl.h, wl.m, wl.max_levels, wl.min_coarse, wl.relax,
                                wl.max_iter, wl.layer, wl.act)
    lamN = np.random.default_rng(1).standard_normal(wl.state_shape).astype(np.float32)
    Lam, dW, db, hist_a, _ = O.fas_adjoint(d["W"], d["b"], U.astype(np.float32), lamN, wl.h, wl.m, wl.max_levels,
                                           wl.min_coarse, wl.relax, wl.max_iter, wl.layer, wl.act)
    return {"workload": wl.name, "cycles": it, "residual_history": hist, "U": U.tolist(),
            "adjoint_residual_history": hist_a, "Lam": Lam.tolist(), "dW": dW.tolist(), "db": db.tolist()}


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cfg1_oracle.json")
    with open(out, "w") as f:
        json.dump(compute(), f)
    print("wrote", out)
