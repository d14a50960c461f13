"""sage_topm_static (the entry point that allocates nothing) against sage_topm, through the C ABI."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _scores(n, seed, torch):
    g = torch.Generator(device="cpu").manual_seed(seed)
    a = torch.rand(n, generator=g, dtype=torch.float32) * 2 - 1
    # heavy ties around the threshold, and both zeros
    a[::7] = 0.25
    a[3::1001] = -0.0
    a[5::1003] = 0.0
    return a.cuda()


def test_static_topm_matches_allocating_topm_on_two_calls_in_a_row():
    import torch

    from paper_2510_02470_amd import binding

    L = binding.lib()
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    # the second call is smaller: what the first left in the shared work space must not leak into it
    for n, m, seed in ((1_000_003, 100_000, 1), (70_001, 3_333, 2), (2_049, 2_049, 3), (5, 1, 4)):
        a = _scores(n, seed, torch)
        want = torch.empty(m, dtype=torch.int64, device="cuda")
        got = torch.full((m,), -1, dtype=torch.int64, device="cuda")
        print("topm_static case", n, m, flush=True)
        assert L.sage_topm(C.c_void_p(a.data_ptr()), n, m, C.c_void_p(want.data_ptr()), stream) == 0
        assert L.sage_topm_static(C.c_void_p(a.data_ptr()), n, m, C.c_void_p(got.data_ptr()), stream) == 0
        torch.cuda.synchronize()
        assert torch.equal(got, want)
        # and against a plain sort of (score descending, index ascending)
        ah = a.cpu().numpy()
        order = np.lexsort((np.arange(n), -(ah + np.float32(0.0))))[:m]
        assert np.array_equal(np.sort(order), got.cpu().numpy())


def test_static_topm_rejects_what_it_cannot_hold():
    import torch

    from paper_2510_02470_amd import binding

    L = binding.lib()
    a = torch.zeros(16, dtype=torch.float32, device="cuda")
    out = torch.zeros(16, dtype=torch.int64, device="cuda")
    p, q = C.c_void_p(a.data_ptr()), C.c_void_p(out.data_ptr())
    # sizes are checked before any pointer is used
    assert L.sage_topm_static(p, binding.TOPM_STATIC_MAX_N + 1, 1, q, None) == binding.SAGE_ERR_CAPACITY
    assert L.sage_topm_static(p, 16, 17, q, None) == binding.SAGE_ERR_ARG
    assert L.sage_topm_static(None, 16, 1, q, None) == binding.SAGE_ERR_ARG
    assert L.sage_topm_static(p, 16, 0, None, None) == 0
