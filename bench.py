#!/usr/bin/env python3
"""Throughput of the SAGE hot path on one MI355X.

Workload: the largest single-GPU configuration of BASELINE.json at the metric's ell = 256 (config 5, "large-head
stress": D = 2,049,000 bf16 rows, fp32 sketch and accumulation, ell = 256, k = 128, batches of 1024 rows;
--workload 4 gives the fp32 D = 1,048,576 configuration). Rows are synthetic, generated on the device before the
timed region.

A step = one batch through the whole path: sage_fd_update(batch) in pass 1 and sage_score(batch) in pass 2.
The timed region runs pass 1 over the K batches, forms the basis once (sage_fd_basis), runs pass 2 over the same
K batches and selects once (sage_select), exactly as the two-pass method does; `value` counts all of it, so the
once-per-pass work (basis, selection) is amortised over only K batches, which is pessimistic against a full-length
stream. The update and the scoring calls are also reported on their own.

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
PEAK_MFMA_BF16 = 2.5e15    # flop/s, dense bf16 matrix cores
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
    ap.add_argument("--steps", type=int, default=16)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", type=int, default=5, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB copy kernel (untimed): the known traffic that rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE readings are scaled by")
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
    if (W + K) * w.batch > w.N:          # small workloads: no more steps than the stream has batches
        K = max(1, w.N // w.batch - W)
    esz = 2 if w.dtype == "bf16" else 4
    ell, n, D, k = w.ell, 2 * w.ell, w.D, w.k

    if args.copy_probe:
        from paper_2510_02470_amd.binding import copy_probe
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        copy_probe(dst, src)
        torch.cuda.synchronize()
        del src, dst

    ds = inputs.DeviceStream(w, w_dtype=torch.bfloat16)
    batches = [ds.batch(b) for b in range(W + K)]  # resident in HBM before anything is timed
    torch.cuda.synchronize()

    def note(msg):   # progress on stderr (stdout carries the one JSON line)
        print("bench: " + msg, file=sys.stderr, flush=True)

    note("inputs resident")

    # class labels for the class-balanced variant (CB-SAGE): the workload's class count where it is a last-layer shape
    n_classes = {2: 10, 3: 100, 5: 1000}.get(args.workload, 10)
    gl = torch.Generator(device="cuda")
    gl.manual_seed(99)
    labels = [torch.randint(0, n_classes, (b.shape[0],), generator=gl, device="cuda", dtype=torch.int32) for b in batches]

    def run_pass(s, timed):
        """W warm-up steps then K steps of the whole path; returns the event times of the K steps (ms)."""
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(7)]
        for b in range(W):
            s.fd_update(batches[b])
        s.fd_basis(k)
        for b in range(W):
            s.score(batches[b])
        s.select(w.keep)
        torch.cuda.synchronize()
        note("warm-up done")
        t0 = time.perf_counter()
        ev[0].record()
        for b in range(W, W + K):
            s.fd_update(batches[b])
        ev[1].record()
        s.fd_basis(k)
        ev[2].record()
        for b in range(W, W + K):
            s.score_labeled(batches[b], labels[b])      # sage_score plus a 4-byte label per row
        ev[3].record()
        idx = s.select(w.keep)
        ev[4].record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        ev[5].record()
        idx_cb = s.select_cb(w.keep, n_classes)         # the class-balanced selection of the same pass (not in `value`)
        ev[6].record()
        torch.cuda.synchronize()
        note("timed steps done")
        ms = [ev[i].elapsed_time(ev[i + 1]) for i in range(4)] + [ev[5].elapsed_time(ev[6])]
        return ms, wall, (idx, idx_cb)

    # ---- timed: exactly K steps (the events are recorded on the stream the library launches on)
    s = Sage(ell, D, dtype=w.dtype, max_rows=(W + K) * w.batch)
    (ms_update, ms_basis, ms_score, ms_select, ms_select_cb), wall, (idx, idx_cb) = run_pass(s, True)
    total_ms = ms_update + ms_basis + ms_score + ms_select
    rows = K * w.batch
    value = rows / (total_ms * 1e-3)
    upd_rows_s = rows / (ms_update * 1e-3)
    sc_rows_s = rows / (ms_score * 1e-3)          # the scoring calls alone (steady state of a long stream)
    sc_all_rows_s = rows / ((ms_basis + ms_score + ms_select) * 1e-3)
    st = s.stats()
    s.close()
    del s

    # ---- per-kernel durations with HIP events on the library's stream: the same work again on a fresh context
    # (every launch bracketed by events, which serialises the side stream's work into the context stream)
    kern = {}
    roof = None
    tile_flop = 2.0 * 64 * 64 * D                       # one 64x64 Gram tile over D columns
    gram_tiles = (n // 64) * (n // 64 + 1) // 2 - (ell // 64) * (ell // 64 + 1) // 2   # top x top block is known
    # The library's default arithmetic for the shrink's products (SAGE_MM_SPLIT): fp32 values as three bf16 parts, six
    # bf16 matrix-core products per fp32 product, where a kernel exists (rebuild: padded ell 128 or 256; the steady-state
    # Gram blocks: padded ell 256). Those kernels are priced in executed bf16 flops against the bf16 peak.
    LP = 32
    while LP < ell:
        LP *= 2
    split_rebuild, split_gram = LP in (128, 256), LP == 256
    algo = {
        # work per launch: (bound, executed flops or algorithmic bytes, peak)
        "gram": ("mfma", gram_tiles * tile_flop * (6.0 if split_gram else 1.0),   # per cycle; split over its launches below
                 PEAK_MFMA_BF16 if split_gram else PEAK_MFMA_F32),
        "rebuild": ("mfma", 2.0 * ell * n * D * (6.0 if split_rebuild else 1.0),
                    PEAK_MFMA_BF16 if split_rebuild else PEAK_MFMA_F32),
        "project": ("hbm", w.batch * (esz * D + 4.0 * k) + 4.0 * k * D, PEAK_HBM),
        "insert": ("hbm", (esz + 4.0) * ell * D, PEAK_HBM),
    }
    if not args.no_kernel_timing:
        s = Sage(ell, D, dtype=w.dtype, max_rows=(W + K) * w.batch)
        for b in range(W):
            s.fd_update(batches[b])
        s.profile_enable(True)
        s.profile_read()
        for b in range(W, W + K):
            s.fd_update(batches[b])
        pr_upd = s.profile_read()
        s.fd_basis(k)
        s.profile_read()            # the basis launches (a smaller rebuild, one more Gram) are not the steady state
        for b in range(W, W + K):
            s.score(batches[b])
        s.select(w.keep)
        pr = s.profile_read()
        pr.update({kk: vv for kk, vv in pr_upd.items() if vv[1]})
        s.profile_enable(False)
        s.close()
        del s
        note("per-kernel pass done")
        traffic = {}
        tpath = os.path.join(ROOT, "profiles", "hbm_traffic_cfg%d.json" % args.workload)
        if os.path.exists(tpath):
            with open(tpath) as f:
                traffic = json.load(f)     # bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
        for name, (ms, cnt) in pr.items():
            if not cnt:
                continue
            e = {"avg_ms": ms / cnt, "launches": cnt, "total_ms": ms}
            if name in algo:
                bound, work, peak = algo[name]
                if name == "gram":   # two launches per cycle (new x new block, new x top block): rate over both
                    work = work * pr["rebuild"][1] / cnt
                rate = work / (ms / cnt * 1e-3)
                e["bound"] = bound
                e["achieved"] = rate / 1e12 if bound == "mfma" else rate / 1e9
                e["unit"] = "TFLOP/s" if bound == "mfma" else "GB/s"
                e["frac"] = rate / peak
                e["peak"] = peak / (1e12 if bound == "mfma" else 1e9)
            if name in traffic:
                e["traffic"] = traffic[name]
            kern[name] = e
        g = kern.get("rebuild")
        if g:
            roof = {"kernel": ("rebuild_split_kernel (B[0:ell] <- diag(w) Y^T B; bf16 MFMA on three-way split fp32 values, "
                               "6 bf16 products per fp32 product; the longest kernel of a cycle)") if split_rebuild else
                              "rebuild_kernel (B[0:ell] <- diag(w) Y^T B, fp32 MFMA; the longest kernel of a cycle)",
                    "bound": "mfma", "achieved": g["achieved"], "peak": g["peak"], "unit": "TFLOP/s",
                    "frac": g["frac"], "traffic": g.get("traffic"), "avg_launch_ms": g["avg_ms"],
                    "launches": g["launches"],
                    "algorithmic_flop_per_launch": 2.0 * ell * n * D * (6.0 if split_rebuild else 1.0),
                    "fp32_equivalent_TFLOPs": 2.0 * ell * n * D / (g["avg_ms"] * 1e-3) / 1e12}

    score_bytes_row = esz * D + 4.0 * k * D / w.batch + 4.0 * k
    exec_flop_row = (gram_tiles * tile_flop + 2.0 * ell * n * D) / ell      # what the update executes per row
    out = {
        "metric": "gradient rows/sec ingested (FD update + scoring) at ell=256; % MFMA / HBM peak",
        "value": value, "unit": "rows/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": total_ms / K, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "N_timed": rows, "D": D, "ell": ell, "k": k, "batch": w.batch,
                   "row_dtype": w.dtype, "keep": w.keep},
        "update_rows_per_s": upd_rows_s,
        "update_arithmetic": ("fp32 values as three bf16 parts, 6 bf16 MFMA products per fp32 product (fp32 accuracy)"
                              if split_rebuild else "fp32 MFMA"),
        # fp32-equivalent flops (Gram without the known block + rebuild) against the fp32 matrix-core peak; the
        # 8*ell*D convention counts the whole triangle
        "update_frac_mfma_peak": upd_rows_s * exec_flop_row / PEAK_MFMA_F32,
        "update_frac_mfma_peak_8ellD": upd_rows_s * 8.0 * ell * D / PEAK_MFMA_F32,
        "score_rows_per_s": sc_rows_s,
        "score_GBps": sc_rows_s * score_bytes_row / 1e9,
        "score_frac_hbm_peak": sc_rows_s * score_bytes_row / PEAK_HBM,
        "score_with_basis_and_select_rows_per_s": sc_all_rows_s,
        "ms": {"update": ms_update, "basis": ms_basis, "score": ms_score, "select": ms_select, "wall": wall * 1e3},
        "cb_sage": {"classes": n_classes, "select_cb_ms": ms_select_cb, "selected": int(idx_cb.numel()),
                    "note": "class-balanced selection of the same scored pass; not part of value"},
        "selected": int(idx.numel()), "jacobi_sweeps_last": st.last_sweeps, "n_shrinks": int(st.n_shrinks),
        "roofline": roof, "kernels": kern,
    }
    del batches
    # ---- the same path fed with the two factors of last-layer gradient rows instead of the rows (not part of value)
    shape = {2: (10, 512), 3: (100, 512), 5: (1000, 2048)}.get(args.workload)
    if shape is not None:
        Cn, dh = shape
        Ko = min(K, 8)
        df = inputs.DeviceFactors(Cn, dh, w.dtype, seed=w.seed)
        fac = [df.batch(b, w.batch) for b in range(1 + Ko)]
        s = Sage(ell, D, dtype=w.dtype, max_rows=(1 + Ko) * w.batch)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        s.fd_update_outer(fac[0][0], fac[0][1])
        s.fd_basis(k)
        s.score_outer(fac[0][0], fac[0][1])
        torch.cuda.synchronize()
        ev[0].record()
        for E, H, _ in fac[1:]:
            s.fd_update_outer(E, H)
        ev[1].record()
        sweeps_outer = s.stats().last_sweeps   # (waits for the update; the basis call below starts its own count)
        s.fd_basis(k)
        ev[2].record()
        for E, H, _ in fac[1:]:
            s.score_outer(E, H)
        ev[3].record()
        torch.cuda.synchronize()
        ro = Ko * w.batch
        out["outer_rows"] = {
            "classes": Cn, "features": dh, "rows_timed": ro,
            "update_rows_per_s": ro / (ev[0].elapsed_time(ev[1]) * 1e-3),
            "score_rows_per_s": ro / (ev[2].elapsed_time(ev[3]) * 1e-3),
            "jacobi_sweeps_last": sweeps_outer,   # these rows have another spectrum than the row-major stream's
            "note": "sage_fd_update_outer / sage_score_outer: rows given as logit error (x) [features; 1]; "
                    "the D-long rows are never stored",
        }
        s.close()
        del s, fac
        note("factored-row pass done")
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
