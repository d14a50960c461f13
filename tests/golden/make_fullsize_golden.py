"""Writes the full-size fixtures tests/golden/{cfg2_full,cfg3_full,ell256_cycles}.npz: what the CPU oracle returns
for the whole path (Algorithm 1, Phase I and II; Method, FD paragraph and "Agreement Scoring and Selection") on seeded
synthetic streams that are too long to run through the oracle inside a test:

  cfg2_full      the second workload of the task at its full size (N = 50,000 rows, D = 5,130, ell = 64, k = 32,
                 batches of 1,024, keep rate 5%): 780 shrink cycles
  cfg3_full      the third workload at its full size (N = 50,000, D = 51,300, ell = 128, k = 64, batches of 2,048,
                 keep rate 10%): 390 shrink cycles. Its sketch rows (26 MB) are not stored: counters, squared singular
                 values, consensus direction, scores and selection are
  ell256_cycles  a bf16 stream of the fifth workload's recipe at D = 4,096 with ell = 256, k = 128, batches of 1,024,
                 22 shrink cycles: the sketch size at which every dense kernel of the GPU cycle has its own code

The paper prints no numerical worked example, so these are not the paper's values: they freeze what the oracle (pinned
in tests/test_oracle_pins.py against LAPACK, closed forms and the FD invariants) returns. Each file holds the rows of
the oracle's sketch that are in use (stored as float32: a relative change of 6e-8, against a parity bar of 1e-4 on the
covariance), its counters, the squared singular values of the frozen buffer, the consensus direction, every score and
the selection.

Run from the repository root:   python tests/golden/make_fullsize_golden.py [names ...] [--mode 0|1]
mode 1 (fp64 Gram + two-sided Jacobi) or mode 0 (one-sided Jacobi on the rows: the definition, several times slower).
Without --mode every stream takes the route its committed fixture was written with: cfg2_full mode 0 (eight minutes on
eight cores; tests/test_golden.py holds the Gram route to it), the other two mode 1.
Calls only oracle/ and the seeded input generator; never the HIP library.
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import Oracle  # noqa: E402
from paper_2510_02470_amd import inputs  # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))
ROWS_NOT_STORED = ("cfg3_full",)


def workloads():
    W = inputs.WORKLOADS
    return {
        "cfg2_full": W[2],
        "cfg3_full": W[3],
        "ell256_cycles": W[5].scaled(name="ell256_cycles", N=256 * 23 + 31, D=4096, r=300, batch=1024, keep=0.05),
    }


def run(name, mode):
    w = workloads()[name]
    G = inputs.generate_numpy(w)
    o = Oracle(w.ell, w.D, mode)
    t0 = time.time()
    for lo in range(0, w.N, w.batch):
        o.update(G[lo:lo + w.batch])
        print("  %s: update %d / %d  (%.0f s)" % (name, min(w.N, lo + w.batch), w.N, time.time() - t0), flush=True)
    o.basis(w.k)
    sig2 = o.sig2
    for lo in range(0, w.N, w.batch):
        o.score(G[lo:lo + w.batch])
    idx = o.select(w.keep)
    print("  %s: scored and selected (%.0f s)" % (name, time.time() - t0), flush=True)
    B = o.B
    used = o.fill
    A = inputs.bf16_bits_to_f32(G) if G.dtype == np.uint16 else G
    out = dict(
        citation=np.array("Algorithm 1 (Phase I: FD sketch, delta = sigma_ell^2, S <- Sigma' V^T; Phase II: z = V_k^T g, "
                          "zhat, consensus u, alpha = <zhat, u>, top keep*N); values by oracle/ (fp64), mode %d" % mode),
        input_checksum=np.float64(np.abs(A.astype(np.float64)).sum()),
        mode=np.int64(mode), n_shrinks=np.int64(o.n_shrinks), fill=np.int64(used), rows_seen=np.int64(o.rows_seen),
        sum_delta=np.float64(o.sum_delta), frob2=np.float64(o.frob2),
        sig2=sig2, u=o.u, alpha=o.alpha, selected=idx.astype(np.int64),
    )
    if name not in ROWS_NOT_STORED:
        out["sketch_rows"] = B[:used].astype(np.float32)
    path = os.path.join(HERE, name + ".npz")
    np.savez_compressed(path, **out)
    print("wrote %s (%d bytes)" % (path, os.path.getsize(path)), flush=True)


DEFAULT_MODE = {"cfg2_full": 0, "cfg3_full": 1, "ell256_cycles": 1}


def main(argv):
    mode = None
    names = []
    it = iter(argv)
    for a in it:
        if a == "--mode":
            mode = int(next(it))
        else:
            names.append(a)
    for name in names or list(workloads()):
        run(name, DEFAULT_MODE[name] if mode is None else mode)


if __name__ == "__main__":
    main(sys.argv[1:])
