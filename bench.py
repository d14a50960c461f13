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

Beside the headline run the line carries: the same update with the shrink's products on the fp32 matrix cores
(`update_fp32_mfma`), short runs of the other four workloads (`workloads`), the factored-row entry points
(`outer_rows`), the class-balanced selection (`cb_sage`) and the CPU oracle timed on this host (`cpu_baseline`).

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


def note(msg):   # progress on stderr (stdout carries the one JSON line)
    print("bench: " + msg, file=sys.stderr, flush=True)


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(w):
    """The CPU oracle, as it stands, on a bounded sample of the same recipe, timed here.

    A shrink cycle of the oracle's Gram route is a Gram matrix and a rebuild whose cost is linear in D, and an n x n
    Jacobi eigensolve whose cost does not depend on D. The sample runs two cycles at a narrower D and one eigensolve of
    a Gram matrix of the same buffer on its own; only the D-linear share is scaled to the full width."""
    import numpy as np

    import oracle
    from paper_2510_02470_amd import inputs

    Ds = 32768
    ws = w.scaled(N=768 + 256, D=Ds, r=min(w.r, 256))
    G = inputs.generate_numpy(ws)
    A = (inputs.bf16_bits_to_f32(G) if G.dtype == np.uint16 else G)[:2 * ws.ell].astype(np.float64)
    t0 = time.perf_counter()
    oracle.sym_jacobi(A @ A.T)   # the D-independent step of one cycle (numpy forms the matrix outside the timed call)
    t_eig = time.perf_counter() - t0
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
    cycles = 2
    lin = max(t_up - cycles * t_eig, 0.0)                 # Gram + rebuild + insert of the two cycles at D = Ds
    t_up_full = lin * (w.D / float(Ds)) + cycles * t_eig    # ... at the full width
    upd = 768.0 / t_up_full
    sc = 256.0 / (t_sc * (w.D / float(Ds)))               # projection: linear in D
    both = 1.0 / (1.0 / upd + 1.0 / sc)
    return {
        "value": both, "unit": "rows/s", "cores": oracle.oracle_threads(), "kind": "oracle", "cpu_model": cpu_model(),
        "build": "gcc -O3 -fopenmp, no -march=native (the same library runs on whatever host the GPU box has), plain "
                 "loops, no BLAS",
        "update_rows_per_s": upd, "score_rows_per_s": sc,
        "seconds": {"update_2_cycles": t_up, "one_eigensolve_512": t_eig, "basis": t_basis, "score_256_rows": t_sc},
        "sample": "oracle (fp64, Gram route, OpenMP) on the same recipe at D=%d: 768 update rows = 2 shrink cycles "
                  "(%.1f s, of which 2 x %.1f s for the 512 x 512 Jacobi eigensolve, timed on its own), basis (%.1f s), "
                  "256 scored rows (%.1f s); the D-linear share (Gram, rebuild, projection) is scaled by %d/%d, the "
                  "eigensolve is not" % (Ds, t_up, t_eig, t_basis, t_sc, w.D, Ds),
    }


def padded(ell):
    LP = 32
    while LP < ell:
        LP *= 2
    return LP


def run_workload(torch, inputs, Sage, w, K, W, split=True, labels_classes=None, per_kernel=False, traffic=None):
    """W warm-up steps, then K timed steps of the whole path on workload w; optionally a second pass with every launch
    bracketed by HIP events (per-kernel durations). Returns a dict of rates and fractions."""
    if (W + K) * w.batch > w.N:          # small workloads: no more steps than the stream has batches
        K = max(1, w.N // w.batch - W)
    esz = 2 if w.dtype == "bf16" else 4
    ell, n, D, k = w.ell, 2 * w.ell, w.D, w.k
    ds = inputs.DeviceStream(w, w_dtype=torch.bfloat16)
    batches = [ds.batch(b) for b in range(W + K)]  # resident in HBM before anything is timed
    del ds
    torch.cuda.synchronize()
    note("%s: %d batches resident" % (w.name, W + K))
    labels = None
    if labels_classes:
        gl = torch.Generator(device="cuda")
        gl.manual_seed(99)
        labels = [torch.randint(0, labels_classes, (b.shape[0],), generator=gl, device="cuda", dtype=torch.int32)
                  for b in batches]

    # ---- timed: exactly K steps (the events are recorded on the stream the library launches on)
    s = Sage(ell, D, dtype=w.dtype, max_rows=(W + K) * w.batch)
    s.set_update_arithmetic(split)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(7)]
    for b in range(W):
        s.fd_update(batches[b])
    s.fd_basis(k)
    for b in range(W):
        s.score(batches[b])
    s.select(w.keep)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    for b in range(W, W + K):
        s.fd_update(batches[b])
    st = s.stats()      # runs a shrink that the last call left pending and waits: all K batches' work is in `update`
    ev[1].record()
    s.fd_basis(k)
    ev[2].record()
    for b in range(W, W + K):
        if labels:
            s.score_labeled(batches[b], labels[b])      # sage_score plus a 4-byte label per row
        else:
            s.score(batches[b])
    ev[3].record()
    idx = s.select(w.keep)
    ev[4].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    res = {}
    if labels:
        ev[5].record()
        idx_cb = s.select_cb(w.keep, labels_classes)    # the class-balanced selection of the same pass (not in `value`)
        ev[6].record()
        torch.cuda.synchronize()
        res["cb_sage"] = {"classes": labels_classes, "select_cb_ms": ev[5].elapsed_time(ev[6]),
                          "selected": int(idx_cb.numel()),
                          "note": "class-balanced selection of the same scored pass (budgets sum to `selected` of the "
                                  "plain selection); not part of value"}
    ms_update, ms_basis, ms_score, ms_select = [ev[i].elapsed_time(ev[i + 1]) for i in range(4)]
    total_ms = ms_update + ms_basis + ms_score + ms_select
    rows = K * w.batch
    upd_rows_s = rows / (ms_update * 1e-3)
    sc_rows_s = rows / (ms_score * 1e-3)          # the scoring calls alone (steady state of a long stream)
    score_bytes_row = esz * D + 4.0 * k * D / w.batch + 4.0 * k
    LP = padded(ell)
    split_rebuild, split_gram = split and LP in (128, 256), split and LP == 256
    # Rows of a bf16 stream have one bf16 part, not three: the split kernels issue 3 products (not 6) where a buffered
    # stream row is one factor and 1 where both are (the products left out are exact zeros).
    one_part = w.dtype == "bf16"
    rebuild_products = (6.0 + 3.0) / 2.0 if one_part else 6.0                  # top half 6, new half 3
    gram_products = (16 * 3.0 + 10 * 1.0) / 26.0 if one_part else 6.0          # 16 tiles new x top, 10 tiles new x new
    res.update({
        "K": K, "W": W, "rows": rows, "value": rows / (total_ms * 1e-3), "ms_per_step": total_ms / K,
        "update_rows_per_s": upd_rows_s,
        # the task's convention: 8 ell D flop per ingested row (lower-triangle Gram + rebuild), as a rate and against the
        # fp32 matrix-core peak the task names. With the split arithmetic the products run on the bf16 matrix cores, so
        # this is an fp32-equivalent rate, not a utilisation of the fp32 cores.
        "update_TFLOPs_8ellD": upd_rows_s * 8.0 * ell * D / 1e12,
        "update_8ellD_over_fp32_mfma_peak": upd_rows_s * 8.0 * ell * D / PEAK_MFMA_F32,
        "score_rows_per_s": sc_rows_s,
        "score_GBps": sc_rows_s * score_bytes_row / 1e9,
        "score_frac_hbm_peak": sc_rows_s * score_bytes_row / PEAK_HBM,
        "score_with_basis_and_select_rows_per_s": rows / ((ms_basis + ms_score + ms_select) * 1e-3),
        "ms": {"update": ms_update, "basis": ms_basis, "score": ms_score, "select": ms_select, "wall": wall * 1e3},
        "selected": int(idx.numel()), "jacobi_sweeps_last": st.last_sweeps, "n_shrinks": int(st.n_shrinks),
        "unconverged_solves": int(st.n_unconverged),
        "update_arithmetic": (("fp32 values as three bf16 parts, 6 bf16 MFMA products per fp32 product (fp32 accuracy)"
                               + ("; bf16 stream rows have one part: 3 products where one factor is such a row, 1 where "
                                  "both are (same bits)" if one_part else ""))
                              if split_rebuild else "fp32 MFMA"),
    })
    s.close()
    del s

    if per_kernel:
        # per-kernel durations with HIP events on the library's stream: the same work again on a fresh context (every
        # launch bracketed by events, which serialises the side stream's work into the context stream)
        tile_flop = 2.0 * 64 * 64 * D                       # one 64x64 Gram tile over D columns
        gram_tiles = (n // 64) * (n // 64 + 1) // 2 - (ell // 64) * (ell // 64 + 1) // 2   # top x top block is known
        rebuild_flop = 2.0 * ell * n * D                    # the method's work per launch: B[0:ell] <- M B
        mm_peak_g = PEAK_MFMA_BF16 if split_gram else PEAK_MFMA_F32
        mm_peak_r = PEAK_MFMA_BF16 if split_rebuild else PEAK_MFMA_F32
        algo = {   # (bound, algorithmic work per launch / cycle, peak of the unit that executes it, instructions' factor)
            "gram": ("mfma", gram_tiles * tile_flop, mm_peak_g, gram_products if split_gram else 1.0),
            "rebuild": ("mfma", rebuild_flop, mm_peak_r, rebuild_products if split_rebuild else 1.0),
            "project": ("hbm", w.batch * (esz * D + 4.0 * k) + 4.0 * k * D, PEAK_HBM, 1.0),
            "insert": ("hbm", (esz + 4.0) * ell * D, PEAK_HBM, 1.0),
        }
        s = Sage(ell, D, dtype=w.dtype, max_rows=(W + K) * w.batch)
        s.set_update_arithmetic(split)
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
        kern = {}
        for name, (ms, cnt) in pr.items():
            if not cnt:
                continue
            e = {"avg_ms": ms / cnt, "launches": cnt, "total_ms": ms}
            if name in algo:
                bound, work, peak, factor = algo[name]
                if name == "gram":   # two launches per cycle (new x new block, new x top block): rate over both
                    work = work * pr["rebuild"][1] / cnt
                rate = work / (ms / cnt * 1e-3)
                e["bound"] = bound
                e["achieved"] = rate / 1e12 if bound == "mfma" else rate / 1e9
                e["unit"] = "TFLOP/s" if bound == "mfma" else "GB/s"
                e["frac"] = rate / peak
                e["peak"] = peak / (1e12 if bound == "mfma" else 1e9)
                if bound == "mfma":
                    e["executed_frac"] = rate * factor / peak   # matrix-core instructions issued (emulating fp32: x6,
                    e["products_per_fp32_product"] = factor     # less where a factor has one bf16 part)
            if traffic and name in traffic:
                e["traffic"] = traffic[name]
            kern[name] = e
        res["kernels"] = kern
        g = kern.get("rebuild")
        if g:
            fp32_equiv = rebuild_flop / (g["avg_ms"] * 1e-3)
            res["roofline"] = {
                "kernel": ("rebuild_split_kernel (B[0:ell] <- diag(w) Y^T B on the bf16 matrix cores: fp32 values as three "
                           "bf16 parts, %.1f bf16 products per fp32 product; the longest single kernel of a cycle)"
                           % rebuild_products)
                if split_rebuild else "rebuild_kernel (B[0:ell] <- diag(w) Y^T B, fp32 MFMA; the longest single kernel of a cycle)",
                "bound": "mfma", "achieved": g["achieved"], "peak": g["peak"], "unit": "TFLOP/s",
                # the method's flops (2 ell n D per launch) over the peak of the unit that executes them
                "frac": g["frac"],
                "frac_of_bf16_peak": fp32_equiv / PEAK_MFMA_BF16 if split_rebuild else None,
                "executed_frac": g["executed_frac"],
                "fp32_equivalent_over_fp32_peak": fp32_equiv / PEAK_MFMA_F32,
                "traffic": g.get("traffic"), "avg_launch_ms": g["avg_ms"], "launches": g["launches"],
                "algorithmic_flop_per_launch": rebuild_flop,
                "executed_flop_per_launch": rebuild_flop * (rebuild_products if split_rebuild else 1.0),
            }
    del batches, labels
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=16)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", type=int, default=5, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the headline run (no fp32-MFMA update, other workloads, factored rows): for profiler runs")
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

    if args.copy_probe:
        from paper_2510_02470_amd.binding import copy_probe
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        copy_probe(dst, src)
        torch.cuda.synchronize()
        del src, dst

    traffic = {}
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_cfg%d.json" % args.workload)
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic = json.load(f)     # bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs

    # class labels for the class-balanced variant (CB-SAGE): the workload's class count where it is a last-layer shape
    n_classes = {2: 10, 3: 100, 5: 1000}.get(args.workload, 10)
    head = run_workload(torch, inputs, Sage, w, K, W, split=True, labels_classes=n_classes,
                        per_kernel=not args.no_kernel_timing, traffic=traffic)
    note("headline run done")
    K = head["K"]
    out = {
        "metric": "gradient rows/sec ingested (FD update + scoring) at ell=256; % MFMA / HBM peak",
        "value": head["value"], "unit": "rows/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "N_timed": head["rows"], "D": w.D, "ell": w.ell, "k": w.k, "batch": w.batch,
                   "row_dtype": w.dtype, "keep": w.keep},
    }
    for key in ("update_rows_per_s", "update_arithmetic", "update_TFLOPs_8ellD", "update_8ellD_over_fp32_mfma_peak",
                "score_rows_per_s", "score_GBps", "score_frac_hbm_peak", "score_with_basis_and_select_rows_per_s", "ms",
                "cb_sage", "selected", "jacobi_sweeps_last", "n_shrinks", "unconverged_solves"):
        out[key] = head.get(key)
    out["roofline"] = head.get("roofline")
    out["kernels"] = head.get("kernels", {})

    if not args.no_extras:
        # ---- the same update with the shrink's products on the fp32 matrix cores (sage_set_update_arithmetic)
        f32 = run_workload(torch, inputs, Sage, w, min(K, 8), W, split=False, per_kernel=not args.no_kernel_timing)
        rf = f32.get("roofline") or {}
        out["update_fp32_mfma"] = {
            "update_rows_per_s": f32["update_rows_per_s"], "steps": f32["K"],
            "update_TFLOPs_8ellD": f32["update_TFLOPs_8ellD"],
            "update_8ellD_over_fp32_mfma_peak": f32["update_8ellD_over_fp32_mfma_peak"],
            "rebuild_kernel": {kk: rf.get(kk) for kk in ("achieved", "peak", "unit", "frac", "avg_launch_ms", "launches")},
            "gram_kernels": {kk: (f32.get("kernels", {}).get("gram") or {}).get(kk)
                             for kk in ("achieved", "peak", "unit", "frac", "avg_ms", "launches")},
            "eigensolve_avg_ms": (f32.get("kernels", {}).get("eigensolve") or {}).get("avg_ms"),
            "note": "SAGE_MM_F32: Gram blocks and rebuild as v_mfma_f32_32x32x2_f32; frac = algorithmic flops over the "
                    "fp32 matrix-core peak",
        }
        note("fp32-MFMA update done")
        # ---- short runs of the other workloads (same code path; the small ones are bound by launch latency)
        wl = {}
        for i in (1, 2, 3, 4, 5):
            if i == args.workload:
                continue
            wi = inputs.WORKLOADS[i]
            r = run_workload(torch, inputs, Sage, wi, 8, 2, split=True)
            wl[wi.name] = {kk: r[kk] for kk in ("K", "rows", "value", "update_rows_per_s", "update_TFLOPs_8ellD",
                                                "update_8ellD_over_fp32_mfma_peak", "score_rows_per_s", "score_GBps",
                                                "score_frac_hbm_peak", "ms", "update_arithmetic")}
            wl[wi.name]["config"] = {"D": wi.D, "ell": wi.ell, "k": wi.k, "batch": wi.batch, "row_dtype": wi.dtype}
        out["workloads"] = wl
        note("other workloads done")
        # ---- the same path fed with the two factors of last-layer gradient rows instead of the rows (not part of value)
        shape = {2: (10, 512), 3: (100, 512), 5: (1000, 2048)}.get(args.workload)
        if shape is not None:
            Cn, dh = shape
            Ko = min(K, 8)
            ell, D, k = w.ell, w.D, w.k
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
            sweeps_outer = s.stats().last_sweeps   # (runs a pending shrink and waits: part of the update)
            ev[1].record()
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
    sys.stdout.flush()


if __name__ == "__main__":
    main()
