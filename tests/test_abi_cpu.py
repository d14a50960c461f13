"""CPU-side checks of the boundary: the built library loads and exports every symbol the header declares."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "sage.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sage_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_five_calls():
    d = _declared()
    for name in ("sage_fd_create", "sage_fd_update", "sage_fd_basis", "sage_score", "sage_select"):
        assert name in d


def test_library_exports_every_declared_symbol():
    from paper_2510_02470_amd import binding

    if not os.path.exists(binding.LIB_PATH):
        pytest.fail("libsage_hip.so is not built: run __graft_entry__.build()")
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in _declared():
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == _declared()


def test_strerror_needs_no_gpu():
    from paper_2510_02470_amd import binding

    L = binding.lib()
    assert L.sage_strerror(0) == b"ok"
    assert L.sage_strerror(-5) == b"capacity exceeded"
    assert L.sage_strerror(-99) == b"unknown status"


def test_workload_recipes():
    """Host logic of the input module: sizes, the selection counts of the five workloads, bf16 rounding."""
    import numpy as np

    from paper_2510_02470_amd import inputs

    W = inputs.WORKLOADS
    assert [W[i].D for i in range(1, 6)] == [512, 5130, 51300, 1048576, 2049000]
    assert [W[i].ell for i in range(1, 6)] == [32, 64, 128, 256, 256]
    assert [int(np.floor(W[i].keep * W[i].N + 0.5)) for i in range(1, 6)] == [205, 2500, 5000, 10000, 10000]
    w = W[2].scaled(N=300, D=200)
    G = inputs.generate_numpy(w)
    assert G.shape == (300, 200) and G.dtype == np.float32
    assert np.array_equal(G, inputs.generate_numpy(w))  # seeded
    # noise share of total energy is eta (up to sampling error)
    s2 = float((w.spectrum() ** 2).sum())
    assert abs(w.noise_tau() ** 2 * w.N * w.D / (s2 + w.noise_tau() ** 2 * w.N * w.D) - w.eta) < 1e-12
    x = np.array([1.0, 1.00390625, 1.01171875, -3.0e-5], dtype=np.float32)
    h = inputs.f32_to_bf16_bits(x)
    assert h.tolist() == [0x3F80, 0x3F80, 0x3F82, 0xB7FC]  # ties to even, then plain rounding


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N > 1 exits with a message (this build runs on one GPU)."""
    import subprocess
    import sys

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and not r.stdout.strip()
