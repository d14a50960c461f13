"""GPU checks at the full row width of the two workloads at the metric's sketch size (config 5, the benchmark's headline:
D = 2,049,000 bf16 rows, ell = 256, k = 128, batches of 1024; config 4: D = 1,048,576 fp32 rows, batches of 512), in
the launch configuration bench.py times. The CPU oracle cannot run a whole pass at this width
in a test, so it is asked for what it can compute one by one: the projection of sampled rows, Gram entries of sampled
row pairs, and the consensus / cosine / selection steps on the k-column problem the GPU's projections define; the
rest are properties of the sketch that hold at any size (Method, FD paragraph; Algorithm 1).
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from oracle import Oracle  # noqa: E402
from paper_2510_02470_amd import inputs  # noqa: E402

pytestmark = pytest.mark.gpu


def _host_rows(Gd, rows):
    """Rows of a device batch on the host in the oracle's input form (float32, or uint16 bf16 bit patterns)."""
    sub = Gd[torch.as_tensor(rows, device=Gd.device)]
    if sub.dtype == torch.bfloat16:
        return sub.view(torch.int16).cpu().numpy().view(np.uint16)
    return sub.cpu().numpy()


def _oracle_consensus_scores(zhat, keep):
    """Consensus, cosine and selection by the oracle on stored normalised projections: they are rows of a k-column
    problem whose basis is the identity (normalising unit rows again changes them by rounding only)."""
    k = zhat.shape[1]
    o = Oracle(2, k, 1)
    o.set_basis(np.eye(k))
    o.score(np.ascontiguousarray(zhat, dtype=np.float32))
    idx = o.select(keep)
    return o.alpha, idx


@pytest.mark.parametrize("cfg", [5, 4])
def test_scoring_at_full_width_matches_the_oracle(cfg):
    """z = V^T g and zhat for sampled rows of two full-width batches against the oracle's projection of the same bytes
    on the same given basis (random rows: the arithmetic does not need it to be orthonormal); consensus, cosine and
    selection of all rows against the oracle run on the stored projections."""
    from paper_2510_02470_amd.binding import Sage

    w = inputs.WORKLOADS[cfg]
    ds = inputs.DeviceStream(w, w_dtype=torch.bfloat16)
    batches = [ds.batch(b) for b in range(2)]
    del ds
    g = torch.Generator(device="cuda")
    g.manual_seed(12345)
    V = torch.randn((w.k, w.D), generator=g, device="cuda", dtype=torch.float32) / np.sqrt(w.D)
    s = Sage(w.ell, w.D, dtype=w.dtype, max_rows=2 * w.batch)
    s.set_basis(V)
    for b in batches:
        s.score(b)
    idx = s.select(0.05).cpu().numpy()
    alpha = s.scores().cpu().numpy()
    zhat = s.zhat().cpu().numpy()
    N = 2 * w.batch
    # sampled rows through the oracle's own projection (first and last row of each launch tile included)
    rng = np.random.default_rng(11)
    sample = sorted(set(rng.choice(N, size=8, replace=False).tolist()) | {0, 511, 512 % N, w.batch - 1, w.batch, N - 1})
    o = Oracle(w.ell, w.D, 1)
    o.set_basis(V.cpu().numpy())
    for i in sample:
        o.score(_host_rows(batches[i // w.batch], [i % w.batch]))
    assert np.abs(zhat[sample] - o.zhat).max() <= 1e-5
    del o
    al, oidx = _oracle_consensus_scores(zhat, 0.05)
    assert np.abs(alpha - al).max() <= 1e-4
    m = int(np.floor(0.05 * N + 0.5))
    assert len(idx) == m and idx.tolist() == oracle.topm_f32(alpha, m).tolist()
    tau = float(np.min(al[oidx]))
    for i in set(idx.tolist()) ^ set(oidx.tolist()):
        assert abs(al[i] - tau) <= 1e-4


@pytest.mark.parametrize("cfg,n_batches,cycles", [(5, 3, 11), (4, 6, 11)])
def test_update_at_full_width_properties_and_sampled_gram(cfg, n_batches, cycles):
    """3 x 1024 (config 5) or 6 x 512 (config 4) rows, 11 shrink cycles, the side-stream path included, at full width: sampled Gram entries against
    the oracle's Gram entries (fp64 dot products, one by one) of the exported rows; after the stream the shrunk rows are orthogonal, row ell-1 on is zero,
    and the energy bookkeeping holds: frob2 = sum ||g||^2, ell * sum(delta) <= ||A||_F^2 - ||B||_F^2."""
    from paper_2510_02470_amd.binding import Sage

    w = inputs.WORKLOADS[cfg]
    ell = w.ell
    ds = inputs.DeviceStream(w, w_dtype=torch.bfloat16)
    s = Sage(ell, w.D, dtype=w.dtype)
    fro = 0.0
    for b in range(n_batches):
        G = ds.batch(b)
        fro += float((G.to(torch.float32).double() ** 2).sum())
        s.fd_update(G)
    # 100 more rows so that the buffer holds shrunk rows and raw rows
    G = ds.batch(n_batches, rows=100)
    fro += float((G.to(torch.float32).double() ** 2).sum())
    s.fd_update(G)
    del G
    st = s.stats()
    assert st.n_shrinks == cycles and st.fill == ell + 100 and st.rows_seen == n_batches * w.batch + 100
    assert abs(st.frob2 - fro) <= 1e-5 * fro
    assert 0.0 <= st.sum_delta <= fro / ell
    B = s.sketch()
    assert not bool(B[ell - 1:ell].any()) and not bool(B[ell + 100:].any())
    b2 = float((B.double() ** 2).sum())
    assert ell * st.sum_delta <= (fro - b2) + 1e-5 * fro
    # sampled Gram entries of the buffer (matrix cores, split over D) against fp64 dot products
    Cm, _, _ = s.probe_gram_eig(False)
    Cm = Cm.cpu().numpy()
    rng = np.random.default_rng(5)
    rows = sorted(set(rng.integers(0, ell + 100, size=10).tolist()) | {0, ell - 2, ell, ell + 99})
    Bs = B[rows].cpu().numpy().astype(np.float64)
    ref = np.array([[oracle.row_dot(a, b) for b in Bs] for a in Bs])
    got = Cm[np.ix_(rows, rows)]
    scale = np.sqrt(np.outer(np.diag(ref), np.diag(ref))).max()
    assert np.abs(got - ref).max() <= 2e-5 * scale  # fp32 accumulation of ~25,000 products per split
    # the same for the split-arithmetic kernels of the steady state (new x top and new x new blocks)
    Cs = s.probe_gram_split().cpu().numpy()
    rows_new = [r for r in rows if r >= ell]
    cols = sorted(set(rows) | {1, ell - 3})
    Bn = B[rows_new].cpu().numpy().astype(np.float64)
    Bc = B[cols].cpu().numpy().astype(np.float64)
    ref2 = np.array([[oracle.row_dot(a, b) for b in Bc] for a in Bn])
    got2 = Cs[np.ix_(rows_new, cols)]
    sc2 = np.sqrt(np.outer((Bn * Bn).sum(axis=1), (Bc * Bc).sum(axis=1))).max()
    assert np.abs(got2 - ref2).max() <= 2e-5 * sc2
    # the rows a shrink wrote are mutually orthogonal (relative to their norms)
    T = B[:ell - 1].double()
    Ct = (T @ T.T).cpu().numpy()
    off = np.abs(Ct - np.diag(np.diag(Ct)))
    assert off.max() <= 1e-5 * np.diag(Ct).max()


def test_factored_scoring_at_full_width():
    """sage_score_outer at the headline shape (1000 classes x 2048 features + 1000 biases = 2,049,000 columns, bf16,
    k = 128, 2 x 1024 rows): zhat of sampled rows against the oracle's projection of the rows it writes out from the
    factors, and all scores against the row-major entry point fed with the same rows written out on the device."""
    from paper_2510_02470_amd.binding import Sage

    w = inputs.WORKLOADS[5]
    Cn, dh = 1000, 2048
    assert Cn * (dh + 1) == w.D
    df = inputs.DeviceFactors(Cn, dh, "bf16", seed=3)
    fac = [df.batch(b, w.batch) for b in range(2)]
    g = torch.Generator(device="cuda")
    g.manual_seed(777)
    V = torch.randn((w.k, w.D), generator=g, device="cuda", dtype=torch.float32) / np.sqrt(w.D)
    s = Sage(w.ell, w.D, dtype=w.dtype, max_rows=2 * w.batch)
    s.set_basis(V)
    for E, H, _ in fac:
        s.score_outer(E, H)
    idx = s.select(0.05).cpu().numpy()
    alpha = s.scores().cpu().numpy()
    zhat = s.zhat().cpu().numpy()
    assert idx.tolist() == oracle.topm_f32(alpha, len(idx)).tolist()
    # sampled rows, written out by the oracle's definition of the rows and projected by the oracle
    rng = np.random.default_rng(8)
    sample = np.sort(rng.choice(2 * w.batch, size=12, replace=False))
    Eh = torch.cat([f[0] for f in fac]).view(torch.int16).cpu().numpy().view(np.uint16)
    Hh = torch.cat([f[1] for f in fac]).view(torch.int16).cpu().numpy().view(np.uint16)
    o = Oracle(w.ell, w.D, 1)
    o.set_basis(V.cpu().numpy())
    for lo in range(0, len(sample), 4):
        o.score(oracle.last_layer_rows(Eh[sample[lo:lo + 4]], Hh[sample[lo:lo + 4]]))
    assert np.abs(zhat[sample] - o.zhat).max() <= 1e-5
    del o
    # the row-major entry point on the same rows (written out on the device, rounded to bf16 like stored rows)
    s.set_basis(V)
    for E, H, _ in fac:
        G = torch.empty((w.batch, w.D), dtype=torch.bfloat16, device="cuda")
        for lo in range(0, w.batch, 128):
            e, h = E[lo:lo + 128].float(), H[lo:lo + 128].float()
            G[lo:lo + 128, :Cn * dh] = (e[:, :, None] * h[:, None, :]).reshape(e.shape[0], -1).to(torch.bfloat16)
            G[lo:lo + 128, Cn * dh:] = E[lo:lo + 128]
        s.score(G)
        del G
    s.select(0.05)
    assert np.abs(s.zhat().cpu().numpy() - zhat).max() <= 1e-5
    assert np.abs(s.scores().cpu().numpy() - alpha).max() <= 1e-4

@pytest.mark.parametrize("cfg", [4, 5])
def test_one_shrink_at_full_width_against_the_oracle(cfg):
    """The exact shapes of the two workloads at the metric's sketch size (config 4: D = 1,048,576 fp32 rows; config 5:
    D = 2,049,000 bf16 rows; ell = 256): the first 612 rows of the stream -- buffer fill, one shrink, 100 more rows --
    through the oracle's Gram route on the host (half a minute to a minute: a full-width shrink is 1 to 2e12 fp64 flop
    in plain loops) and through the GPU path in the launch configuration of the benchmark; sketch covariance to the
    1e-4 bar, sum(delta), counters."""
    from paper_2510_02470_amd.binding import Sage
    from helpers import cov_diff_spec_norm

    w = inputs.WORKLOADS[cfg]
    ds = inputs.DeviceStream(w, w_dtype=torch.bfloat16)
    parts = [ds.batch(0, rows=2 * w.ell), ds.batch(1, rows=100)]
    del ds
    s = Sage(w.ell, w.D, dtype=w.dtype)
    o = Oracle(w.ell, w.D, 1)
    fro = 0.0
    for G in parts:
        s.fd_update(G)
        Gh = _host_rows(G, list(range(G.shape[0])))
        fro += float((G.to(torch.float32).double() ** 2).sum())
        print("oracle: %d rows of width %d ..." % (Gh.shape[0], w.D), flush=True)
        o.update(Gh)
        del Gh
    del parts
    st = s.stats()
    assert st.n_shrinks == o.n_shrinks == 1 and st.fill == o.fill == w.ell + 100 and st.n_unconverged == 0
    # (frob2 is the sum of the Gram diagonal: dot products of D terms with fp32 accumulation inside a column range)
    assert abs(st.sum_delta - o.sum_delta) <= 1e-5 * fro and abs(st.frob2 - fro) <= 5e-5 * fro
    Bg = s.sketch().cpu().numpy()[:st.fill]
    err = cov_diff_spec_norm(Bg, o.B[:o.fill]) / fro
    print("one shrink at D = %d: covariance error %.3g" % (w.D, err), flush=True)
    assert err <= 1e-4, err
