"""The frozen worked example tests/golden/fd_tiny.json (written by tests/golden/make_golden.py from the oracle alone):
the oracle must still reproduce it, and the HIP path must match it to the parity bars."""
import importlib.util
import json
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def _golden():
    with open(os.path.join(HERE, "golden", "fd_tiny.json")) as f:
        return json.load(f)


def _maker():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    m = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(m)
    return m


def test_oracle_reproduces_the_frozen_example():
    g = _golden()
    m = _maker()
    assert g["recipe"] == json.loads(json.dumps(m.RECIPE))
    w, G, o, idx, cov = m.run()
    assert abs(float(np.abs(G.astype(np.float64)).sum()) - g["input_checksum"]) <= 1e-9 * g["input_checksum"]
    assert o.n_shrinks == g["n_shrinks"] and o.fill == g["fill"]
    assert abs(o.sum_delta - g["sum_delta"]) <= 1e-10 * g["frob2"] and abs(o.frob2 - g["frob2"]) <= 1e-10 * g["frob2"]
    assert np.abs(cov - np.array(g["sketch_covariance"])).max() <= 1e-10 * g["frob2"]
    assert np.abs(o.V.T @ o.V - np.array(g["projector"])).max() <= 1e-9
    assert np.abs(o.alpha - np.array(g["alpha"])).max() <= 1e-9
    assert idx.tolist() == g["selected"]


@pytest.mark.gpu
def test_hip_path_matches_the_frozen_example():
    torch = pytest.importorskip("torch")
    from paper_2510_02470_amd import inputs
    from paper_2510_02470_amd.binding import Sage

    g = _golden()
    w = _maker().workload()
    G = inputs.generate_numpy(w)
    assert abs(float(np.abs(G.astype(np.float64)).sum()) - g["input_checksum"]) <= 1e-9 * g["input_checksum"]
    s = Sage(w.ell, w.D, dtype=w.dtype)
    Gd = torch.from_numpy(G).cuda()
    for lo in range(0, w.N, w.batch):
        s.fd_update(Gd[lo:lo + w.batch])
    st = s.stats()
    assert st.n_shrinks == g["n_shrinks"] and st.fill == g["fill"]
    fro = g["frob2"]
    assert abs(st.sum_delta - g["sum_delta"]) <= 1e-5 * fro and abs(st.frob2 - fro) <= 1e-5 * fro
    Bg = s.sketch().cpu().numpy().astype(np.float64)
    diff = Bg.T @ Bg - np.array(g["sketch_covariance"])
    assert np.abs(np.linalg.eigvalsh(diff)).max() <= 1e-4 * fro
    s.fd_basis(w.k)
    Vg = s.basis().cpu().numpy().astype(np.float64)
    assert np.abs(Vg.T @ Vg - np.array(g["projector"])).max() <= 1e-4
    for lo in range(0, w.N, w.batch):
        s.score(Gd[lo:lo + w.batch])
    idx = s.select(w.keep).cpu().numpy()
    alpha = np.array(g["alpha"])
    assert np.abs(s.scores().cpu().numpy() - alpha).max() <= 1e-4
    want = set(g["selected"])
    tau = alpha[g["selected"]].min()
    assert len(idx) == len(want)
    for i in set(idx.tolist()) ^ want:
        assert abs(alpha[i] - tau) <= 1e-4


# ---------------------------------------------------------------- full-size fixtures (tests/golden/make_fullsize_golden.py)
def _fullsize():
    spec = importlib.util.spec_from_file_location("make_fullsize_golden",
                                                  os.path.join(HERE, "golden", "make_fullsize_golden.py"))
    m = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(m)
    return m


@pytest.mark.parametrize("name", ["cfg2_full", "cfg3_full", "ell256_cycles"])
def test_fullsize_fixtures_obey_what_holds_for_any_fd_run(name):
    """What the stored values must satisfy whatever the stream (Method, FD paragraph): the shrink count the schedule
    fixes, sum(delta) <= ||A||_F^2 / l, l * sum(delta) <= ||A||_F^2 - ||B||_F^2, the squared singular values are those of the
    stored rows, scores in [-1, 1] with mean ||zbar|| >= 0, a unit consensus direction, and the selection is the top m
    of the stored scores."""
    import oracle

    w = _fullsize().workloads()[name]
    z = np.load(os.path.join(HERE, "golden", name + ".npz"))
    fro, ell = float(z["frob2"]), w.ell
    assert int(z["rows_seen"]) == w.N and int(z["n_shrinks"]) == (w.N - 2 * ell) // ell + 1
    assert int(z["fill"]) == w.N - ell * int(z["n_shrinks"])
    assert 0.0 < float(z["sum_delta"]) <= fro / ell
    sig2 = z["sig2"]
    assert np.all(np.diff(sig2) <= 1e-12 * fro) and sig2.min() >= 0.0
    assert ell * float(z["sum_delta"]) <= fro - sig2.sum() + 1e-9 * fro          # ||B||_F^2 = sum of sigma_j^2
    if "sketch_rows" in z:
        B = z["sketch_rows"].astype(np.float64)
        assert B.shape == (int(z["fill"]), w.D)
        ev = np.linalg.eigvalsh(B @ B.T)[::-1]
        assert np.abs(ev - sig2[:len(ev)]).max() <= 1e-6 * fro                     # rows were stored as float32
        assert not sig2[len(ev):].any() or sig2[len(ev):].max() <= 1e-9 * fro
    al = z["alpha"]
    assert al.shape == (w.N,) and al.max() <= 1.0 and al.min() >= -1.0 and al.mean() >= 0.0
    assert abs(float(np.dot(z["u"][:w.k], z["u"][:w.k])) - 1.0) <= 1e-12
    m = oracle.keep_count(w.keep, w.N)
    assert z["selected"].tolist() == oracle.topm_f32(al.astype(np.float32), m).tolist()


def test_gram_route_reproduces_the_config2_fixture_of_the_one_sided_route():
    """The fixture of the second workload at full size was written by the oracle's one-sided Jacobi on the rows
    (mode 0, the definition; about eight minutes). The Gram route (mode 1), which the long GPU parity runs and the other
    fixtures rely on, must reproduce it over all 780 shrink cycles: covariance to 1e-9 ||A||_F^2 (the rows are stored
    as float32), sum(delta) and the squared singular values to 1e-10, scores to 1e-9, the same selection."""
    from oracle import Oracle
    from paper_2510_02470_amd import inputs

    m = _fullsize()
    w = m.workloads()["cfg2_full"]
    z = np.load(os.path.join(HERE, "golden", "cfg2_full.npz"))
    assert int(z["mode"]) == 0
    G = inputs.generate_numpy(w)
    assert abs(float(np.abs(G.astype(np.float64)).sum()) - float(z["input_checksum"])) <= 1e-9 * float(z["input_checksum"])
    o = Oracle(w.ell, w.D, 1)
    for lo in range(0, w.N, w.batch):
        o.update(G[lo:lo + w.batch])
    fro = float(z["frob2"])
    assert o.n_shrinks == int(z["n_shrinks"]) and o.fill == int(z["fill"])
    assert abs(o.sum_delta - float(z["sum_delta"])) <= 1e-10 * fro and abs(o.frob2 - fro) <= 1e-12 * fro
    B1 = o.B[:o.fill]
    B0 = z["sketch_rows"].astype(np.float64)
    W = np.vstack([B1, B0])
    J = np.concatenate([np.ones(B1.shape[0]), -np.ones(B0.shape[0])])
    assert np.abs(np.linalg.eigvals(J[:, None] * (W @ W.T))).max() <= 1e-6 * fro   # float32 storage of the fixture's rows
    o.basis(w.k)
    assert np.abs(o.sig2 - z["sig2"]).max() <= 1e-10 * fro
    for lo in range(0, w.N, w.batch):
        o.score(G[lo:lo + w.batch])
    idx = o.select(w.keep)
    assert np.abs(o.alpha - z["alpha"]).max() <= 1e-9
    assert idx.tolist() == z["selected"].tolist()
