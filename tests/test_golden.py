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
