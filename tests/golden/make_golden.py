"""Writes tests/golden/fd_tiny.json: a frozen worked example of the whole path (Algorithm 1, Phase I and II; Method,
FD paragraph and "Agreement Scoring and Selection") on a tiny seeded input, computed by the CPU oracle alone.

The paper prints no numerical worked example, so this fixture is not the paper's: it freezes what the oracle, pinned
in tests/test_oracle_pins.py against LAPACK, closed forms and the FD invariants, returns on one small case. A change
of the oracle's arithmetic shows up as a mismatch here (tests/test_golden.py) and must be justified from the paper.

Run from the repository root:  python tests/golden/make_golden.py
Calls only oracle/ and the seeded input generator; never the HIP library.
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import Oracle  # noqa: E402
from paper_2510_02470_amd import inputs  # noqa: E402

RECIPE = dict(N=96, D=24, ell=4, k=2, batch=20, keep=0.125, r=3, s_scale=4.0, s_power=1.0, tau=0.02, sigma_norm=0.3,
              flip_prob=0.1, flip="neg", u_orth=True, w_orth=True, seed=7)


def workload():
    return inputs.WORKLOADS[1].scaled(name="golden_tiny", dtype="f32", eta=0.0, **RECIPE)


def run():
    w = workload()
    G = inputs.generate_numpy(w)
    o = Oracle(w.ell, w.D, 0)
    for lo in range(0, w.N, w.batch):
        o.update(G[lo:lo + w.batch])
    o.basis(w.k)
    for lo in range(0, w.N, w.batch):
        o.score(G[lo:lo + w.batch])
    idx = o.select(w.keep)
    B = o.B
    return w, G, o, idx, B.T @ B


def main():
    w, G, o, idx, cov = run()
    out = {
        "citation": "Algorithm 1 (Phase I: streaming FD sketch with delta = sigma_ell^2 and S <- Sigma' V^T; Phase II: "
                    "z = V_k^T g, zhat, consensus u, alpha = <zhat, u>, top keep*N); values by oracle/ (fp64)",
        "recipe": RECIPE,
        "input_checksum": float(np.abs(G.astype(np.float64)).sum()),
        "n_shrinks": o.n_shrinks, "fill": o.fill,
        "sum_delta": o.sum_delta, "frob2": o.frob2,
        "sketch_covariance": [[float(x) for x in row] for row in cov],
        "projector": [[float(x) for x in row] for row in (o.V.T @ o.V)],
        "alpha": [float(a) for a in o.alpha],
        "selected": [int(i) for i in idx],
    }
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "fd_tiny.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    main()
