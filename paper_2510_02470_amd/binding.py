"""Thin ctypes binding of the C ABI in ``include/sage.h`` (argument marshalling only).

Every step of the path runs in the HIP library; torch is used for device memory and the stream handle. If
the library has not been built, or cannot be loaded, importing a symbol from here raises: there is no fallback.
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsage_hip.so")

SAGE_F32, SAGE_BF16 = 0, 1
SAGE_OK, SAGE_ERR_ARG, SAGE_ERR_STATE, SAGE_ERR_ALLOC, SAGE_ERR_HIP, SAGE_ERR_CAPACITY = 0, -1, -2, -3, -4, -5
CB_PROPORTIONAL, CB_EQUAL = 0, 1  # sage_cb_rule

KERNEL_CLASSES = ("gram", "gram_reduce", "eigensolve", "coefficients", "rebuild", "insert", "project",
                  "score_finalize", "select")

# every symbol include/sage.h declares
EXPORTS = (
    "sage_fd_create", "sage_fd_create_ex", "sage_fd_update", "sage_fd_merge", "sage_set_update_arithmetic", "sage_probe_gram_split", "sage_fd_update_outer", "sage_score_outer", "sage_rescore_outer", "sage_set_score_store", "sage_rescore", "sage_fd_basis", "sage_fd_basis_weighted", "sage_score", "sage_select", "sage_score_labeled", "sage_select_cb", "sage_select_cb_ex",
    "sage_destroy", "sage_sync", "sage_set_projection_mode", "sage_fd_sketch_export", "sage_basis_export", "sage_set_basis", "sage_scores",
    "sage_scores_export", "sage_zhat_export", "sage_stats", "sage_topm", "sage_topm_static", "sage_probe_gram_eig", "sage_probe_eig_matrix",
    "sage_profile_enable", "sage_copy_probe", "sage_set_debug_checks", "sage_debug_fail_launch", "sage_set_sweep_policy",
    "sage_profile_read", "sage_strerror",
)


class SageStats(C.Structure):
    _fields_ = [("rows_seen", C.c_int64), ("n_shrinks", C.c_int64), ("n_scored", C.c_int64),
                ("sum_delta", C.c_double), ("frob2", C.c_double), ("last_delta", C.c_double),
                ("last_sweeps", C.c_int), ("fill", C.c_int), ("n_unconverged", C.c_int64),
                ("last_offdiag", C.c_double)]


class SageError(RuntimeError):
    def __init__(self, code, what):
        super().__init__("%s: %s (%d)" % (what, lib().sage_strerror(code).decode(), code))
        self.code = code


_lib = None


def lib():
    """Load libsage_hip.so (built by ``paper_2510_02470_amd.build``). Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("HIP library not built: %s is missing (run __graft_entry__.build())" % LIB_PATH)
    L = C.CDLL(LIB_PATH)
    vp, i64, i32, dbl = C.c_void_p, C.c_int64, C.c_int, C.c_double
    L.sage_fd_create.argtypes = [C.POINTER(vp), i32, i64]
    L.sage_fd_create_ex.argtypes = [C.POINTER(vp), i32, i64, i32, i64, vp]
    L.sage_fd_update.argtypes = [vp, vp, i64]
    L.sage_fd_merge.argtypes = [vp, vp, i64]
    L.sage_set_update_arithmetic.argtypes = [vp, C.c_int]
    L.sage_probe_gram_split.argtypes = [vp, vp, C.POINTER(C.c_int)]
    L.sage_fd_update_outer.argtypes = [vp, vp, vp, i64, i64, i64]
    L.sage_score_outer.argtypes = [vp, vp, vp, vp, i64, i64, i64]
    L.sage_rescore_outer.argtypes = [vp, vp, vp, i64, i64, i64]
    L.sage_set_score_store.argtypes = [vp, i32]
    L.sage_rescore.argtypes = [vp, vp, i64]
    L.sage_fd_basis.argtypes = [vp, i32]
    L.sage_fd_basis_weighted.argtypes = [vp, i32]
    L.sage_score.argtypes = [vp, vp, i64]
    L.sage_select.argtypes = [vp, dbl, vp, i64, C.POINTER(i64)]
    L.sage_score_labeled.argtypes = [vp, vp, vp, i64]
    L.sage_select_cb.argtypes = [vp, dbl, i32, vp, i64, C.POINTER(i64)]
    L.sage_select_cb_ex.argtypes = [vp, dbl, i32, i32, vp, i64, C.POINTER(i64)]
    L.sage_destroy.argtypes = [vp]
    L.sage_destroy.restype = None
    L.sage_sync.argtypes = [vp]
    L.sage_set_projection_mode.argtypes = [vp, i32]
    L.sage_fd_sketch_export.argtypes = [vp, vp]
    L.sage_basis_export.argtypes = [vp, vp]
    L.sage_set_basis.argtypes = [vp, vp, i32]
    L.sage_scores.argtypes = [vp, C.POINTER(vp), C.POINTER(i64)]
    L.sage_zhat_export.argtypes = [vp, vp]
    L.sage_scores_export.argtypes = [vp, vp]
    L.sage_stats.argtypes = [vp, C.POINTER(SageStats)]
    L.sage_topm.argtypes = [vp, i64, i64, vp, vp]
    L.sage_topm_static.argtypes = [vp, i64, i64, vp, vp]
    L.sage_probe_gram_eig.argtypes = [vp, vp, i32, vp, vp, C.POINTER(i32)]
    L.sage_probe_eig_matrix.argtypes = [vp, vp, vp, vp, vp]
    L.sage_copy_probe.argtypes = [vp, vp, i64, vp]
    L.sage_set_debug_checks.argtypes = [vp, i32]
    L.sage_set_sweep_policy.argtypes = [vp, i32]
    L.sage_debug_fail_launch.argtypes = [vp, i32]
    L.sage_profile_enable.argtypes = [vp, i32]
    L.sage_profile_read.argtypes = [vp, i32, C.POINTER(dbl), C.POINTER(i64)]
    L.sage_strerror.argtypes = [i32]
    L.sage_strerror.restype = C.c_char_p
    for name in EXPORTS:
        if name not in ("sage_destroy", "sage_strerror"):
            getattr(L, name).restype = i32
    _lib = L
    return L


def _check(rc, what):
    if rc != SAGE_OK:
        raise SageError(rc, what)


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None and t.numel() > 0 else C.c_void_p(0)


class Sage:
    """One sketch context on the current device and torch's current stream."""

    def __init__(self, ell, D, dtype="f32", max_rows=0):
        import torch

        self.torch = torch
        self.L = lib()
        self.ell, self.D = int(ell), int(D)
        self.dtype = dtype
        self.tdtype = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.h = C.c_void_p(0)
        stream = torch.cuda.current_stream().cuda_stream
        rc = self.L.sage_fd_create_ex(C.byref(self.h), self.ell, self.D, SAGE_BF16 if dtype == "bf16" else SAGE_F32,
                                      int(max_rows), C.c_void_p(stream))
        _check(rc, "sage_fd_create_ex")
        self.k = 0

    def close(self):
        if getattr(self, "h", None) and self.h.value:
            self.L.sage_destroy(self.h)
            self.h = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _rows(self, G):
        assert G.is_cuda and G.is_contiguous() and G.dtype == self.tdtype
        assert G.dim() == 2 and G.shape[1] == self.D
        return G

    def fd_update(self, G):
        G = self._rows(G)
        _check(self.L.sage_fd_update(self.h, _ptr(G), G.shape[0]), "sage_fd_update")

    def set_score_store(self, store_zhat=True):
        _check(self.L.sage_set_score_store(self.h, 1 if store_zhat else 0), "sage_set_score_store")

    def rescore(self, G):
        G = self._rows(G)
        _check(self.L.sage_rescore(self.h, _ptr(G), G.shape[0]), "sage_rescore")

    def fd_merge(self, B_other):
        """Feed the rows of another sketch (fp32 device tensor, rows x D) to this one."""
        assert B_other.is_cuda and B_other.is_contiguous() and B_other.dtype == self.torch.float32 and B_other.shape[1] == self.D
        _check(self.L.sage_fd_merge(self.h, _ptr(B_other), B_other.shape[0]), "sage_fd_merge")

    def set_update_arithmetic(self, split):
        """True / 1: the shrink's dense products run on the bf16 matrix cores with three-way split factors; False / 0:
        fp32 matrix cores; 2: split factors without the one-part shortcut for bf16 rows (same bits as 1)."""
        _check(self.L.sage_set_update_arithmetic(self.h, int(split)), "sage_set_update_arithmetic")

    def _factors(self, E, H):
        for t in (E, H):
            assert t.is_cuda and t.is_contiguous() and t.dtype == self.tdtype and t.dim() == 2
        assert E.shape[0] == H.shape[0]
        return E.shape[0], E.shape[1], H.shape[1]

    def fd_update_outer(self, E, H):
        """Rows e_i (x) [h_i; 1] given by their factors (E: rows x classes, H: rows x features)."""
        rows, ncls, nfeat = self._factors(E, H)
        _check(self.L.sage_fd_update_outer(self.h, _ptr(E), _ptr(H), rows, ncls, nfeat), "sage_fd_update_outer")

    def score_outer(self, E, H, labels=None):
        rows, ncls, nfeat = self._factors(E, H)
        if labels is not None:
            assert labels.is_cuda and labels.is_contiguous() and labels.dtype == self.torch.int32
            assert labels.numel() == rows
        _check(self.L.sage_score_outer(self.h, _ptr(E), _ptr(H), _ptr(labels), rows, ncls, nfeat), "sage_score_outer")

    def rescore_outer(self, E, H):
        rows, ncls, nfeat = self._factors(E, H)
        _check(self.L.sage_rescore_outer(self.h, _ptr(E), _ptr(H), rows, ncls, nfeat), "sage_rescore_outer")

    def fd_basis(self, k, weighted=False):
        if weighted:
            _check(self.L.sage_fd_basis_weighted(self.h, int(k)), "sage_fd_basis_weighted")
        else:
            _check(self.L.sage_fd_basis(self.h, int(k)), "sage_fd_basis")
        self.k = int(k)

    def set_basis(self, Vt):
        assert Vt.is_cuda and Vt.is_contiguous() and Vt.dtype == self.torch.float32 and Vt.shape[1] == self.D
        _check(self.L.sage_set_basis(self.h, _ptr(Vt), Vt.shape[0]), "sage_set_basis")
        self.k = int(Vt.shape[0])

    def set_projection_mode(self, mode):
        """0: bf16-split matrix cores when the rows allow it (default); 1: always fp32 matrix cores."""
        _check(self.L.sage_set_projection_mode(self.h, int(mode)), "sage_set_projection_mode")

    def score(self, G):
        G = self._rows(G)
        _check(self.L.sage_score(self.h, _ptr(G), G.shape[0]), "sage_score")

    def score_labeled(self, G, labels):
        G = self._rows(G)
        assert labels.is_cuda and labels.is_contiguous() and labels.dtype == self.torch.int32
        assert labels.numel() == G.shape[0]
        _check(self.L.sage_score_labeled(self.h, _ptr(G), _ptr(labels), G.shape[0]), "sage_score_labeled")

    def select_cb(self, keep_rate, n_classes, cap=None, rule="proportional"):
        """Class-balanced selection; rule: how the subset size is shared out ("proportional" or "equal")."""
        st = self.stats()
        cap = st.n_scored if cap is None else int(cap)
        out = self.torch.empty(max(cap, 1), dtype=self.torch.int64, device="cuda")
        m = C.c_int64(0)
        code = {"proportional": CB_PROPORTIONAL, "equal": CB_EQUAL}[rule]
        _check(self.L.sage_select_cb_ex(self.h, float(keep_rate), int(n_classes), code, _ptr(out), cap, C.byref(m)),
               "sage_select_cb_ex")
        return out[: m.value]

    def select(self, keep_rate, cap=None):
        st = self.stats()
        N = st.n_scored
        cap = N if cap is None else int(cap)
        out = self.torch.empty(max(cap, 1), dtype=self.torch.int64, device="cuda")
        m = C.c_int64(0)
        _check(self.L.sage_select(self.h, float(keep_rate), _ptr(out), cap, C.byref(m)), "sage_select")
        return out[: m.value]

    def sync(self):
        _check(self.L.sage_sync(self.h), "sage_sync")

    def sketch(self):
        out = self.torch.empty((2 * self.ell, self.D), dtype=self.torch.float32, device="cuda")
        _check(self.L.sage_fd_sketch_export(self.h, _ptr(out)), "sage_fd_sketch_export")
        return out

    def basis(self):
        out = self.torch.empty((self.k, self.D), dtype=self.torch.float32, device="cuda")
        _check(self.L.sage_basis_export(self.h, _ptr(out)), "sage_basis_export")
        return out

    def scores(self):
        st = self.stats()
        out = self.torch.empty(st.n_scored, dtype=self.torch.float32, device="cuda")
        _check(self.L.sage_scores_export(self.h, _ptr(out)), "sage_scores_export")
        return out

    def zhat(self):
        st = self.stats()
        out = self.torch.empty((st.n_scored, self.k), dtype=self.torch.float32, device="cuda")
        _check(self.L.sage_zhat_export(self.h, _ptr(out)), "sage_zhat_export")
        return out

    def stats(self):
        s = SageStats()
        _check(self.L.sage_stats(self.h, C.byref(s)), "sage_stats")
        return s

    def probe_gram_eig(self, eig=True):
        npad = C.c_int(0)
        self.L.sage_probe_gram_eig(self.h, C.c_void_p(0), 0, C.c_void_p(0), C.c_void_p(0), C.byref(npad))
        n = npad.value
        Cm = self.torch.empty((n, n), dtype=self.torch.float64, device="cuda")
        Y = self.torch.empty((n, n), dtype=self.torch.float64, device="cuda")
        lam = self.torch.empty((n,), dtype=self.torch.float64, device="cuda")
        _check(self.L.sage_probe_gram_eig(self.h, _ptr(Cm), 1 if eig else 0, _ptr(Y), _ptr(lam), C.byref(npad)),
               "sage_probe_gram_eig")
        return Cm, Y, lam

    def probe_gram_split(self):
        """The new x top and new x new Gram blocks from the split-arithmetic kernels (top x top block zero)."""
        npad = C.c_int(0)
        _check(self.L.sage_probe_gram_split(self.h, C.c_void_p(0), C.byref(npad)), "sage_probe_gram_split")
        n = npad.value
        Cm = self.torch.empty((n, n), dtype=self.torch.float64, device="cuda")
        _check(self.L.sage_probe_gram_split(self.h, _ptr(Cm), C.byref(npad)), "sage_probe_gram_split")
        return Cm

    def probe_eig_matrix(self, Cm):
        n = Cm.shape[0]
        assert Cm.is_cuda and Cm.dtype == self.torch.float64 and Cm.is_contiguous()
        Y = self.torch.empty((n, n), dtype=self.torch.float64, device="cuda")
        lam = self.torch.empty((n,), dtype=self.torch.float64, device="cuda")
        stat = self.torch.empty((18,), dtype=self.torch.float64, device="cuda")
        _check(self.L.sage_probe_eig_matrix(self.h, _ptr(Cm), _ptr(Y), _ptr(lam), _ptr(stat)), "sage_probe_eig_matrix")
        return Y, lam, stat

    def set_sweep_policy(self, all_sweeps):
        """True: every shrink's eigensolve gets all its sweeps; False (default): as many as recent solves needed, plus two."""
        _check(self.L.sage_set_sweep_policy(self.h, 1 if all_sweeps else 0), "sage_set_sweep_policy")

    def set_debug_checks(self, on=True):
        _check(self.L.sage_set_debug_checks(self.h, 1 if on else 0), "sage_set_debug_checks")

    def debug_fail_launch(self, nth):
        _check(self.L.sage_debug_fail_launch(self.h, int(nth)), "sage_debug_fail_launch")

    def profile_enable(self, on=True):
        _check(self.L.sage_profile_enable(self.h, 1 if on else 0), "sage_profile_enable")

    def profile_read(self):
        out = {}
        for i, name in enumerate(KERNEL_CLASSES):
            ms, n = C.c_double(0), C.c_int64(0)
            _check(self.L.sage_profile_read(self.h, i, C.byref(ms), C.byref(n)), "sage_profile_read")
            out[name] = (ms.value, n.value)
        return out


def copy_probe(dst, src):
    """Plain copy kernel src -> dst (same byte size, multiple of 16): the calibration kernel for traffic counters."""
    import torch

    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes and src.is_cuda and dst.is_cuda
    stream = torch.cuda.current_stream().cuda_stream
    _check(lib().sage_copy_probe(_ptr(dst), _ptr(src), nbytes, C.c_void_p(stream)), "sage_copy_probe")


def topm(alpha, m):
    """Stand-alone top-m of a float32 CUDA tensor: indices (int64, ascending) of the m greatest scores."""
    import torch

    assert alpha.is_cuda and alpha.dtype == torch.float32 and alpha.is_contiguous()
    out = torch.empty(max(int(m), 1), dtype=torch.int64, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    _check(lib().sage_topm(_ptr(alpha), alpha.numel(), int(m), _ptr(out), C.c_void_p(stream)), "sage_topm")
    return out[: int(m)]


TOPM_STATIC_MAX_N = 16777216  # SAGE_TOPM_STATIC_MAX_N


def topm_static(alpha, m, out):
    """sage_topm_static: as topm, into the caller's int64 tensor, without allocating and without waiting."""
    import torch

    assert alpha.is_cuda and alpha.dtype == torch.float32 and alpha.is_contiguous()
    assert out.is_cuda and out.dtype == torch.int64 and out.is_contiguous() and out.numel() >= int(m)
    stream = torch.cuda.current_stream().cuda_stream
    _check(lib().sage_topm_static(_ptr(alpha), alpha.numel(), int(m), _ptr(out), C.c_void_p(stream)),
           "sage_topm_static")
    return out[: int(m)]
