"""GPU parity at the sizes the task names, and on the independent route of the oracle.

  * the second workload at its full size (50,000 x 5,130, ell = 64, 780 shrink cycles) and a 22-cycle bf16 stream at
    ell = 256 against fixtures the oracle wrote (tests/golden/make_fullsize_golden.py);
  * sketches at ell = 64 and ell = 128 against the oracle's one-sided Jacobi on the rows (mode 0), which shares neither
    the Gram matrix nor the two-sided rotations with the GPU path;
  * a stream whose spectrum changes abruptly between cycles (the eigensolve must still converge);
  * bit-equal results of two runs with the same cut of the stream at ell = 256, side stream active;
  * bit-equal results with and without the one-part shortcut the split kernels take for rows of a bf16 stream.

Bars as in tests/test_gpu_parity.py.
"""
import os

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from helpers import check_basis_and_scores, cov_diff_spec_norm, run_gpu, run_oracle, to_dev  # noqa: E402
import oracle  # noqa: E402
from oracle import Oracle  # noqa: E402
from paper_2510_02470_amd import inputs  # noqa: E402

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
COV_TOL = 1e-4
SCORE_TOL = 1e-4


def _golden_workloads():
    import importlib.util

    spec = importlib.util.spec_from_file_location("make_fullsize_golden", os.path.join(GOLDEN, "make_fullsize_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod.workloads()


class _Frozen:
    """What a fixture holds of the oracle's run, under the names the checks use."""

    def __init__(self, z, D):
        self.fill, self.n_shrinks, self.rows_seen = int(z["fill"]), int(z["n_shrinks"]), int(z["rows_seen"])
        self.sum_delta, self.frob2 = float(z["sum_delta"]), float(z["frob2"])
        self.B = z["sketch_rows"].astype(np.float64) if "sketch_rows" in z else None
        self.sig2, self.alpha, self.u, self.selected = z["sig2"], z["alpha"], z["u"], z["selected"]
        self.V = None
        assert self.B is None or self.B.shape == (self.fill, D)


@pytest.mark.parametrize("name", ["cfg2_full", "ell256_cycles", "cfg3_full"])
def test_full_streams_match_the_oracle_fixture(name):
    """Sketch covariance, counters and squared singular values against what the oracle wrote for the same seeded
    stream; then the end-to-end check of the basis and the scores (the oracle scores the rows live on the GPU's basis),
    and the scores against the fixture's own as far as the conditioning of the top-k subspace lets them agree.
    The third workload's fixture holds no sketch rows (26 MB): there the covariance enters through the squared singular
    values of the frozen buffer (which move by at most the covariance error), sum(delta) and the scores, and the oracle
    projects a sample of the rows."""
    w = _golden_workloads()[name]
    z = np.load(os.path.join(GOLDEN, name + ".npz"))
    fz = _Frozen(z, w.D)
    G = inputs.generate_numpy(w)
    A = inputs.bf16_bits_to_f32(G) if G.dtype == np.uint16 else G
    assert abs(float(np.abs(A.astype(np.float64)).sum()) - float(z["input_checksum"])) <= 1e-9 * float(z["input_checksum"])
    fro = float((A.astype(np.float64) ** 2).sum())
    del A
    s, gidx = run_gpu(w, G)
    st = s.stats()
    assert st.n_shrinks == fz.n_shrinks and st.fill == fz.fill and st.rows_seen == fz.rows_seen == w.N
    assert st.n_unconverged * 100 <= st.n_shrinks     # (adaptive sweep count: see test_abrupt_spectrum_change)
    Bg = s.sketch().cpu().numpy()
    assert not Bg[st.fill:].any()
    sg = np.linalg.eigvalsh(Bg.astype(np.float64) @ Bg.astype(np.float64).T)[::-1]
    err = (cov_diff_spec_norm(Bg, fz.B) if fz.B is not None else float(np.abs(sg - fz.sig2).max())) / fro
    print("%s: covariance error %.3g, sum_delta %.6g vs %.6g" % (name, err, st.sum_delta / fro, fz.sum_delta / fro), flush=True)
    assert err <= COV_TOL, err
    assert abs(st.sum_delta - fz.sum_delta) <= 1e-5 * fro and abs(st.frob2 - fro) <= 1e-5 * fro
    assert abs(fz.frob2 - fro) <= 1e-9 * fro
    # squared singular values of the frozen buffer (Weyl: they move by at most the covariance error)
    assert np.abs(sg - fz.sig2).max() <= COV_TOL * fro
    del Bg

    # (the fixture holds sig2 and alpha, not the oracle's k x D basis)
    out = check_basis_and_scores(s, w, G, fz, fro, sample=48 if name == "cfg3_full" else None, cov_err=err)
    gap = (fz.sig2[w.k - 1] - fz.sig2[w.k]) / fro
    al = s.scores().cpu().numpy()
    err_fix = float(np.abs(al - fz.alpha).max())
    print("%s: max |alpha - fixture alpha| = %.3g, spectral gap %.3g" % (name, err_fix, gap), flush=True)
    # first-order bound on the rotation of the top-k subspace: covariance error over the gap
    assert err_fix <= max(SCORE_TOL, 4.0 * err / max(gap, 1e-300)), (err_fix, err, gap)
    if err_fix <= SCORE_TOL:
        gi, oi = set(gidx.cpu().numpy().tolist()), set(fz.selected.tolist())
        tau = float(np.min(fz.alpha[fz.selected]))
        for i in gi ^ oi:
            assert abs(float(fz.alpha[i]) - tau) <= SCORE_TOL
    assert out["err_same_basis"] <= SCORE_TOL


@pytest.mark.parametrize("ell,D,cycles,batch,dtype", [(64, 1024, 8, 300, "f32"), (128, 600, 5, 1000, "bf16")])
def test_sketch_matches_the_one_sided_jacobi_oracle(ell, D, cycles, batch, dtype):
    """Oracle mode 0 (Hestenes rotations of the buffer rows: no Gram matrix, no two-sided Jacobi) against the GPU's
    Gram + blocked two-sided Jacobi route, beyond the first workload: covariance, counters, then scores end to end."""
    w = inputs.WORKLOADS[3].scaled(name="hestenes_%d" % ell, N=ell * (cycles + 1) + 29, D=D, ell=ell, k=ell // 2,
                                   batch=batch, r=3 * ell // 2, dtype=dtype)
    G = inputs.generate_numpy(w)
    o, _ = run_oracle(w, G, mode=0)
    s, _ = run_gpu(w, G)
    st = s.stats()
    A64 = (inputs.bf16_bits_to_f32(G) if G.dtype == np.uint16 else G).astype(np.float64)
    fro = (A64 ** 2).sum()
    assert st.n_shrinks == o.n_shrinks == cycles and st.fill == o.fill and st.n_unconverged == 0 and st.last_sweeps < 100
    err = cov_diff_spec_norm(s.sketch().cpu().numpy(), o.B) / fro
    assert err <= COV_TOL, err
    assert abs(st.sum_delta - o.sum_delta) <= 1e-5 * fro and abs(st.frob2 - fro) <= 1e-5 * fro
    check_basis_and_scores(s, w, G, o, fro)


@pytest.mark.parametrize("all_sweeps", [True, False])
def test_abrupt_spectrum_change(all_sweeps):
    """The number of Jacobi sweeps a solve gets is chosen ahead of time from what earlier solves needed. A stream whose
    spectrum changes abruptly between cycles (flat noise, then a steep low-rank signal 1000 times larger, then rows
    that repeat, then noise again), with a wait after every phase so that the count has adapted to it before the next
    one starts. With SAGE_SWEEPS_ALL every solve must reach the tolerance; with the adaptive default a solve that runs
    out of sweeps must be counted, and the sketch must meet the covariance bar either way (a shrink from a not quite
    diagonalising rotation is still a valid step, and the Gram block taken as known includes what was left)."""
    from paper_2510_02470_amd.binding import Sage

    ell, D = 64, 900
    rng = np.random.default_rng(42)
    parts = [rng.standard_normal((5 * ell, D)) * 1e-2]
    steep = (rng.standard_normal((4 * ell, 6)) * (10.0 ** -np.arange(6))) @ rng.standard_normal((6, D)) * 10.0
    parts.append(steep + 1e-6 * rng.standard_normal(steep.shape))
    rep = np.repeat(rng.standard_normal((8, D)), ell // 2, axis=0)
    parts.append(rep[rng.permutation(rep.shape[0])])
    parts.append(rng.standard_normal((3 * ell + 11, D)) * 1e-3)
    G = np.concatenate(parts).astype(np.float32)
    o = Oracle(ell, D, 1)
    s = Sage(ell, D)
    s.set_sweep_policy(all_sweeps)
    Gd = torch.from_numpy(G).cuda()
    cuts = np.cumsum([0] + [p.shape[0] for p in parts])
    for a0, a1 in zip(cuts[:-1], cuts[1:]):
        for lo in range(a0, a1, 200):
            s.fd_update(Gd[lo:min(a1, lo + 200)])   # no wait between the calls: the host runs ahead of the solves
        s.sync()                                    # ... and one here, so that the sweep counts of this phase are known
    o.update(G)
    st = s.stats()
    fro = (G.astype(np.float64) ** 2).sum()
    print("abrupt change, all sweeps %s: %d of %d solves unconverged, last off-diagonal %.2g" %
          (all_sweeps, st.n_unconverged, st.n_shrinks, st.last_offdiag), flush=True)
    assert st.n_shrinks == o.n_shrinks and st.fill == o.fill
    if all_sweeps:
        assert st.n_unconverged == 0 and st.last_sweeps < 100 and st.last_offdiag <= 1e-7
    else:
        assert 0 <= st.n_unconverged <= st.n_shrinks
    assert cov_diff_spec_norm(s.sketch().cpu().numpy(), o.B) / fro <= COV_TOL
    assert abs(st.sum_delta - o.sum_delta) <= 1e-5 * fro


def test_same_cut_gives_the_same_bits_at_full_sketch_size():
    """Two runs of the same calls at ell = 256 (split-arithmetic kernels, look-ahead on the side stream, deferred
    shrinks): reductions are in a fixed order and nothing depends on timing, so sketch, scores and selection agree bit
    for bit."""
    w = inputs.WORKLOADS[5].scaled(N=256 * 9 + 77, D=3000, batch=1024, r=200, keep=0.1)
    G = inputs.generate_numpy(w)
    s1, i1 = run_gpu(w, G)
    s2, i2 = run_gpu(w, G)
    assert s1.stats().n_shrinks == 8
    assert torch.equal(s1.sketch(), s2.sketch())
    assert torch.equal(s1.basis(), s2.basis())
    assert torch.equal(s1.scores(), s2.scores()) and torch.equal(i1, i2)
    assert s1.stats().sum_delta == s2.stats().sum_delta


@pytest.mark.parametrize("ell,D,batch", [(256, 3000, 1024), (256, 2064, 700), (128, 1500, 2048)])
def test_one_part_shortcut_for_bf16_rows_changes_no_bit(ell, D, batch):
    """Rows of a bf16 stream have one bf16 part; the split-arithmetic kernels leave out the products with the other
    two (exact zeros). With the shortcut (mode 1, the default) and without it (mode 2): the same bits in the sketch, the
    basis, the scores and the selection. Batches that do and do not cut the stream at multiples of ell."""
    w = inputs.WORKLOADS[5].scaled(N=ell * 7 + 77, D=D, ell=ell, k=ell // 2, batch=batch, r=200, keep=0.1)
    G = inputs.generate_numpy(w)
    s1, i1 = run_gpu(w, G, arithmetic=1)
    s2, i2 = run_gpu(w, G, arithmetic=2)
    assert s1.stats().n_shrinks == s2.stats().n_shrinks == 6
    assert torch.equal(s1.sketch(), s2.sketch())
    assert torch.equal(s1.basis(), s2.basis())
    assert torch.equal(s1.scores(), s2.scores()) and torch.equal(i1, i2)
    assert s1.stats().sum_delta == s2.stats().sum_delta


def test_one_part_shortcut_is_dropped_for_rows_that_are_not_bf16_values():
    """A bf16 context that also receives fp32 rows (sage_fd_merge) and factored rows (stored rounded to bf16) between
    its bf16 batches: a half buffer that holds any fp32 row takes all three parts. Same bits as without the shortcut,
    and the covariance of the whole stream against the oracle."""
    from paper_2510_02470_amd.binding import Sage

    ell, C, dh = 256, 12, 171
    D = C * (dh + 1)
    rng = np.random.default_rng(5)
    w = inputs.WORKLOADS[5].scaled(N=ell * 4, D=D, ell=ell, k=64, batch=512, r=100)
    G = inputs.generate_numpy(w)                                    # bf16 bits
    Gd = to_dev(G, torch)
    F = torch.from_numpy((rng.standard_normal((300, D)) * 0.05).astype(np.float32)).cuda()
    E = torch.from_numpy(rng.standard_normal((200, C)).astype(np.float32)).cuda().bfloat16()
    H = torch.from_numpy((rng.standard_normal((200, dh)) * 0.05).astype(np.float32)).cuda().bfloat16()
    out = []
    for mode in (1, 2):
        s = Sage(ell, D, dtype="bf16")
        s.set_update_arithmetic(mode)
        s.fd_update(Gd[:700])          # fills the top half, 188 rows short of the first shrink
        s.fd_merge(F)                  # fp32 rows complete that buffer and start the next new half
        s.fd_update(Gd[700:])          # bf16 rows on top of them in the same half, then whole halves of bf16 rows
        s.fd_update_outer(E, H)
        s.fd_update(Gd[:400])
        s.fd_basis(64)
        out.append((s.sketch().clone(), s.basis().clone(), s.stats()))
    assert out[0][2].n_shrinks == out[1][2].n_shrinks and out[0][2].n_shrinks >= 5
    assert torch.equal(out[0][0], out[1][0]) and torch.equal(out[0][1], out[1][1])
    assert out[0][2].sum_delta == out[1][2].sum_delta
    # the oracle on the same rows, in the same order
    Eh, Hh = E.float().cpu().numpy().astype(np.float64), H.float().cpu().numpy().astype(np.float64)
    outer = np.concatenate([(Eh[:, :, None] * Hh[:, None, :]).reshape(200, C * dh), Eh], axis=1)
    outer = torch.from_numpy(outer).float().bfloat16().float().numpy().astype(np.float64)   # rounded as a stored row
    A = inputs.bf16_bits_to_f32(G).astype(np.float64)
    rows = np.concatenate([A[:700], F.cpu().numpy().astype(np.float64), A[700:], outer, A[:400]])
    o = Oracle(ell, D, 1)
    o.update(rows.astype(np.float32))      # (every one of them is an fp32 value)
    fro = (rows ** 2).sum()
    st = out[0][2]
    assert st.n_shrinks == o.n_shrinks and st.fill == o.fill
    assert cov_diff_spec_norm(out[0][0].cpu().numpy(), o.B) / fro <= COV_TOL
