"""Writes tests/golden/tiny_oracle.json: float64 oracle values on the tiny workload (seed 0).

The paper prints no worked numerical example, so there is no value of the paper's to store; these values come
from the CPU oracle only (never from the GPU path) and serve as a regression guard for the oracle and the
workload generator, and as a fixed target for the GPU parity test of the tiny configuration.
Run from the repository root:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import nadmm_oracle as orc  # noqa: E402
from paper_1807_07132_amd import workloads  # noqa: E402


def main():
    w = workloads.tiny(0)
    prob = orc.Problem(w.A, w.b, w.C, s=w.s, lam=w.lam, rho=w.rho, z=w.z, y=w.y)
    f0, g0 = orc.loss_grad(prob, w.X0)
    hv = orc.hessvec(prob, w.X0, w.V)
    X1, st = orc.local_newton(prob, w.X0, 1, 10, 0.0, 0.0, w.beta, w.gamma, w.max_ls)
    out = {
        "source": "oracle/nadmm_oracle.py on workloads.tiny(seed=0); Sections 2.1-2.6, Algorithms 2 and 3",
        "loss_at_X0": f0,
        "grad_at_X0": g0.tolist(),
        "hessvec_at_X0": hv.tolist(),
        "newton_1step_10cg_X": X1.tolist(),
        "newton_alpha": st["iters"][0]["alpha"],
        "newton_loss_final": st["loss_final"],
    }
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_oracle.json"), "w") as f:
        json.dump(out, f, indent=1)


if __name__ == "__main__":
    main()
