#!/usr/bin/env python3
"""Throughput of the SAGE hot path on one MI355X.

Workload: the largest single-GPU configuration of BASELINE.json at the metric's ell = 256 (config 5, "large-head
stress": D = 2,049,000 bf16 rows, fp32 sketch and accumulation, ell = 256, k = 128, batches of 1024 rows;
--workload 4 gives the fp32 D = 1,048,576 configuration). Rows are synthetic, generated on the device before the
timed region.

A step = one batch through the whole path: sage_fd_update(batch) in pass 1 and sage_score(batch) in pass 2.
The timed region runs pass 1 over the K batches, forms the basis once (sage_fd_basis), runs pass 2 over the same
K batches and selects once (sage_select), exactly as the two-pass method does; the once-per-pass work is thus
amortised over only K batches, which is pessimistic against a full-length stream.

Prints ONE JSON line (see the fields at the bottom).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_F32 = 157.3e12   # flop/s, dense fp32 matrix cores, MI355X
PEAK_HBM = 8.0e12          # B/s


def cpu_baseline(w, seconds_hint=20.0):
    """The CPU oracle, as it stands, on a bounded sample of the same recipe (narrower rows), timed here."""
    import numpy as np

    import oracle
    from paper_2510_02470_amd import inputs

    Ds = 32768
    ws = w.scaled(N=768 + 256, D=Ds, r=min(w.r, 256))
    G = inputs.generate_numpy(ws)
    o = oracle.Oracle(ws.ell, Ds, 1)
    t0 = time.perf_counter()
    o.update(G[:768])            # two shrink cycles at ell = 256
    t_up = time.perf_counter() - t0
    t0 = time.perf_counter()
    o.basis(ws.k)
    t_basis = time.perf_counter() - t0
    t0 = time.perf_counter()
    o.score(G[768:])
    o.select(ws.keep)
    t_sc = time.perf_counter() - t0
    # per-row cost of update and scoring is linear in D: scale the sampled rates to the full width
    scale = Ds / float(w.D)
    upd = 768.0 / t_up * scale
    sc = 256.0 / t_sc * scale
    both = 1.0 / (1.0 / upd + 1.0 / sc)
    return {
        "value": both, "unit": "rows/s", "cores": oracle.oracle_threads(), "kind": "oracle",
        "update_rows_per_s": upd, "score_rows_per_s": sc,
        "sample": "oracle (fp64, Gram route, OpenMP) on the same recipe at D=%d: 768 update rows (2 shrink cycles, "
                  "%.1f s), basis (%.1f s), 256 scored rows (%.1f s); rates scaled by %d/%d since the cost per row "
                  "is linear in D" % (Ds, t_up, t_basis, t_sc, Ds, w.D),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", type=int, default=5, choices=[3, 4, 5])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2510_02470_amd import inputs
    from paper_2510_02470_amd.binding import Sage

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    w = inputs.WORKLOADS[args.workload]
    K, W = args.steps, max(1, args.warmup)
    esz = 2 if w.dtype == "bf16" else 4

    ds = inputs.DeviceStream(w, w_dtype=torch.bfloat16)
    # W warm-up batches, K timed batches, K fresh batches for the per-kernel timing pass
    batches = [ds.batch(b) for b in range(W + 2 * K)]
    torch.cuda.synchronize()

    s = Sage(w.ell, w.D, dtype=w.dtype, max_rows=(W + 2 * K) * w.batch)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]

    # ---- warm-up: W batches through both passes (fills the buffer, first-use allocations, code load)
    for b in range(W):
        s.fd_update(batches[b])
    s.fd_basis(w.k)
    for b in range(W):
        s.score(batches[b])
    s.select(w.keep)
    torch.cuda.synchronize()

    # ---- timed: exactly K steps
    t_wall0 = time.perf_counter()
    ev[0].record()
    for b in range(W, W + K):
        s.fd_update(batches[b])
    ev[1].record()
    s.fd_basis(w.k)
    for b in range(W, W + K):
        s.score(batches[b])
    ev[2].record()
    idx = s.select(w.keep)
    ev[3].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_wall0
    ms_update = ev[0].elapsed_time(ev[1])
    ms_score = ev[1].elapsed_time(ev[2])
    ms_select = ev[2].elapsed_time(ev[3])
    total_ms = ev[0].elapsed_time(ev[3])
    rows = K * w.batch
    value = rows / (total_ms * 1e-3)
    upd_rows_s = rows / (ms_update * 1e-3)
    sc_rows_s = rows / ((ms_score + ms_select) * 1e-3)
    st = s.stats()

    # ---- per-kernel durations with HIP events on the library's stream (separate pass, same work)
    kern = {}
    roof = None
    if not args.no_kernel_timing:
        s.profile_enable(True)
        s.profile_read()
        for b in range(W + K, W + 2 * K):
            s.fd_update(batches[b])
        s.fd_basis(w.k)
        for b in range(W + K, W + 2 * K):
            s.score(batches[b])
        s.select(w.keep)
        pr = s.profile_read()
        s.profile_enable(False)
        n = 2 * w.ell
        algo = {
            # algorithmic flops / bytes per launch
            "gram": ("mfma", float(n) * (n + 1) * w.D),                       # lower triangle of B B^T
            "rebuild": ("mfma", 2.0 * w.ell * n * w.D),                       # M B (basis launches are smaller)
            "project": ("hbm", w.batch * (esz * w.D + 4.0 * w.k) + 4.0 * w.k * w.D),
            "insert": ("hbm", (esz + 4.0) * w.ell * w.D),
        }
        for name, (ms, cnt) in pr.items():
            if not cnt:
                continue
            e = {"avg_ms": ms / cnt, "launches": cnt, "total_ms": ms}
            if name in algo:
                bound, work = algo[name]
                rate = work / (ms / cnt * 1e-3)
                e["bound"] = bound
                e["achieved"] = rate / 1e12 if bound == "mfma" else rate / 1e9
                e["unit"] = "TFLOP/s" if bound == "mfma" else "GB/s"
                e["frac"] = rate / (PEAK_MFMA_F32 if bound == "mfma" else PEAK_HBM)
            kern[name] = e
        g = kern.get("gram")
        if g:
            roof = {"kernel": "gram_kernel<8> (C = B B^T, lower triangle, fp32 MFMA)", "bound": "mfma",
                    "achieved": g["achieved"], "peak": PEAK_MFMA_F32 / 1e12, "unit": "TFLOP/s", "frac": g["frac"],
                    "traffic": None, "avg_launch_ms": g["avg_ms"], "launches": g["launches"],
                    "algorithmic_flop_per_launch": float(n) * (n + 1) * w.D}

    out = {
        "metric": "gradient rows/sec ingested (FD update + scoring) at ell=256; % MFMA / HBM peak",
        "value": value, "unit": "rows/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": total_ms / K, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "N_timed": rows, "D": w.D, "ell": w.ell, "k": w.k, "batch": w.batch,
                   "row_dtype": w.dtype, "keep": w.keep},
        "update_rows_per_s": upd_rows_s,
        "update_frac_mfma_peak": upd_rows_s * 8.0 * w.ell * w.D / PEAK_MFMA_F32,
        "score_rows_per_s": sc_rows_s,
        "score_GBps": sc_rows_s * (esz * w.D + 4.0 * w.k * w.D / w.batch + 4.0 * w.k) / 1e9,
        "score_frac_hbm_peak": sc_rows_s * (esz * w.D + 4.0 * w.k * w.D / w.batch + 4.0 * w.k) / PEAK_HBM,
        "score_frac_mfma_peak": sc_rows_s * 2.0 * w.k * w.D / PEAK_MFMA_F32,
        "ms": {"update": ms_update, "basis_plus_score": ms_score, "select": ms_select, "wall": wall * 1e3},
        "selected": int(idx.numel()), "jacobi_sweeps_last": st.last_sweeps, "n_shrinks": int(st.n_shrinks),
        "roofline": roof, "kernels": kern,
    }
    del batches
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
