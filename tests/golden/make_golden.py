"""Writes tests/golden/cfg1_oracle.json: the tridiagonal, the ten largest Ritz
values and a checksum of one update step for the smallest workload, computed
by the CPU oracle alone (run from the repository root:
`python tests/golden/make_golden.py`).  The paper prints no worked numeric
example, so these are oracle-written regression values, not paper values."""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402
import workloads as wl  # noqa: E402


def main():
    w = wl.planted_workload(1)
    op = lambda v: oracle.hvp_planted(w.U, w.lam, float(w.shift), v)
    res = oracle.lanczos(op, w.v1, w.m)
    rz = oracle.ritz(res.Q, res.alpha, res.beta, res.m_eff, w.k, w.l)
    p = w.params
    w1, b1 = oracle.fosi_step(w.w0, w.grad(0), rz.V, rz.evals, np.zeros(w.n),
                              float(p.alpha), float(p.lr), float(p.momentum))
    out = {
        "workload": "planted spectrum, n=4096, r=32, m=40, k=10, l=0",
        "m_eff": int(res.m_eff),
        "alpha": [float(x) for x in res.alpha[: res.m_eff]],
        "beta": [float(x) for x in res.beta[: res.m_eff]],
        "ritz_top10": [float(x) for x in rz.evals],
        "step_update_norm": float(np.linalg.norm(w1 - w.w0)),
        "step_update_first4": [float(x) for x in (w1 - w.w0)[:4]],
        "momentum_norm": float(np.linalg.norm(b1)),
    }
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "cfg1_oracle.json"), "w") as f:
        json.dump(out, f, indent=1)


if __name__ == "__main__":
    main()
