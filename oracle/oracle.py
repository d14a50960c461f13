"""ctypes front end of ``sage_oracle.c`` (fp64 CPU oracle; test infrastructure only).

Every function here only marshals arguments; the arithmetic lives in the C file, which cites the passages of
the paper (arxiv 2510.02470) it follows. The one exception is ``last_layer_rows``, which writes out the rows that
the factored entry points of the library are defined on (plain numpy, a few lines).
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sage_oracle.c")
_LIB = os.path.join(_HERE, "libsage_oracle.so")
_lib = None


def build_oracle(force=False):
    """Compile the oracle with gcc (no arch-specific flags: the library also runs on another host)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        # the sanitizer driver (tests build it again with -fsanitize): compiled here so that a build covers every C file
        os.makedirs(os.path.join(_HERE, "_build"), exist_ok=True)
        subprocess.run(["gcc", "-O2", "-fopenmp", "-std=c11", "-o", os.path.join(_HERE, "_build", "sanitize_check"),
                        os.path.join(_HERE, "sanitize_check.c"), _SRC, "-lm"], check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build_oracle()
    L = C.CDLL(_LIB)
    vp, i64, dbl, i32 = C.c_void_p, C.c_int64, C.c_double, C.c_int
    L.orc_create.restype = vp
    L.orc_create.argtypes = [i32, i64, i32]
    L.orc_destroy.argtypes = [vp]
    for name in ("orc_update_f32", "orc_update_bf16", "orc_score_f32", "orc_score_bf16"):
        getattr(L, name).argtypes = [vp, vp, i64]
        getattr(L, name).restype = i32
    L.orc_basis.argtypes = [vp, i32]
    L.orc_basis_weighted.argtypes = [vp, i32]
    L.orc_set_basis.argtypes = [vp, vp, i32]
    L.orc_select.argtypes = [vp, dbl, vp, i64, vp]
    L.orc_topm_f32.argtypes = [vp, i64, i64, vp]
    L.orc_keep_count.argtypes = [dbl, i64]
    L.orc_keep_count.restype = i64
    L.orc_hestenes_rows.argtypes = [vp, i32, i64, vp]
    L.orc_sym_jacobi.argtypes = [vp, i32, vp, vp]
    for name in ("orc_B", "orc_V", "orc_sig2", "orc_alpha", "orc_zhat", "orc_u", "orc_ssum"):
        getattr(L, name).argtypes = [vp]
        getattr(L, name).restype = C.POINTER(C.c_double)
    for name in ("orc_fill", "orc_n_shrinks", "orc_last_sweeps"):
        getattr(L, name).argtypes = [vp]
        getattr(L, name).restype = i32
    for name in ("orc_n_scored", "orc_rows_seen"):
        getattr(L, name).argtypes = [vp]
        getattr(L, name).restype = i64
    for name in ("orc_sum_delta", "orc_last_delta", "orc_frob2"):
        getattr(L, name).argtypes = [vp]
        getattr(L, name).restype = dbl
    L.orc_threads.restype = i32
    L.orc_row_dot.argtypes = [vp, vp, i64]
    L.orc_row_dot.restype = dbl
    _lib = L
    return L


def oracle_threads():
    return int(_load().orc_threads())


def _as_rows(G):
    """Accept float32 rows, or bf16 rows given as uint16 bit patterns. Returns (array, is_bf16)."""
    G = np.ascontiguousarray(G)
    if G.dtype == np.uint16:
        return G, True
    if G.dtype != np.float32:
        raise TypeError("rows must be float32, or uint16 holding bf16 bit patterns")
    return G, False


class Oracle:
    """The four calls of the path on the CPU in fp64. mode 0 = Hestenes on rows, mode 1 = Gram route."""

    def __init__(self, ell, D, mode=0):
        self.L = _load()
        self.ell, self.n, self.D, self.mode = int(ell), 2 * int(ell), int(D), int(mode)
        self.h = self.L.orc_create(self.ell, self.D, self.mode)
        if not self.h:
            raise ValueError("bad ell / D / mode")
        self.k = 0

    def __del__(self):
        if getattr(self, "h", None):
            self.L.orc_destroy(self.h)
            self.h = None

    def update(self, G):
        G, bf = _as_rows(G)
        assert G.ndim == 2 and G.shape[1] == self.D
        fn = self.L.orc_update_bf16 if bf else self.L.orc_update_f32
        rc = fn(self.h, G.ctypes.data, G.shape[0])
        assert rc == 0

    def basis(self, k, weighted=False):
        """weighted: rows sqrt(sigma_j^2 - delta) v_j^T (the sketch rows a shrink would write) instead of v_j^T."""
        rc = (self.L.orc_basis_weighted if weighted else self.L.orc_basis)(self.h, int(k))
        if rc != 0:
            raise ValueError("basis: need 1 <= k <= ell-1")
        self.k = int(k)

    def set_basis(self, Vt):
        Vt = np.ascontiguousarray(Vt, dtype=np.float64)
        assert Vt.ndim == 2 and Vt.shape[1] == self.D
        rc = self.L.orc_set_basis(self.h, Vt.ctypes.data, Vt.shape[0])
        assert rc == 0
        self.k = Vt.shape[0]

    def score(self, G):
        G, bf = _as_rows(G)
        assert G.ndim == 2 and G.shape[1] == self.D
        fn = self.L.orc_score_bf16 if bf else self.L.orc_score_f32
        rc = fn(self.h, G.ctypes.data, G.shape[0])
        if rc != 0:
            raise RuntimeError("score before basis")

    def select(self, keep_rate):
        N = self.n_scored
        out = np.empty(max(N, 1), dtype=np.int64)
        m = C.c_int64(0)
        rc = self.L.orc_select(self.h, float(keep_rate), out.ctypes.data, N, C.byref(m))
        if rc != 0:
            raise RuntimeError("select failed rc=%d" % rc)
        return out[: m.value].copy()

    def select_cb(self, keep_rate, labels, n_classes, rule="proportional"):
        """Class-balanced selection (Algorithm 1, "if class balance required"): per class c the unit centroid u_c of the
        stored zhat of its rows, alpha_i = <zhat_i, u_c(i)> clamped, and the k_c (cb_budgets: they sum to the plain
        selection's m) rows of the class greatest under (alpha as float32 descending, index ascending). Returns (alpha float64, indices ascending)."""
        return cb_scores_and_selection(self.zhat, labels, n_classes, keep_rate, rule)

    # ---- views (copies) ----
    def _arr(self, ptr, shape):
        n = int(np.prod(shape))
        if n == 0:
            return np.zeros(shape)
        return np.ctypeslib.as_array(ptr, shape=(n,)).reshape(shape).copy()

    @property
    def B(self):
        return self._arr(self.L.orc_B(self.h), (self.n, self.D))

    @property
    def V(self):
        return self._arr(self.L.orc_V(self.h), (self.k, self.D))

    @property
    def sig2(self):
        return self._arr(self.L.orc_sig2(self.h), (self.n,))

    @property
    def alpha(self):
        return self._arr(self.L.orc_alpha(self.h), (self.n_scored,))

    @property
    def zhat(self):
        return self._arr(self.L.orc_zhat(self.h), (self.n_scored, self.k))

    @property
    def u(self):
        return self._arr(self.L.orc_u(self.h), (self.k,))

    @property
    def ssum(self):
        return self._arr(self.L.orc_ssum(self.h), (self.k,))

    @property
    def fill(self):
        return int(self.L.orc_fill(self.h))

    @property
    def n_scored(self):
        return int(self.L.orc_n_scored(self.h))

    @property
    def rows_seen(self):
        return int(self.L.orc_rows_seen(self.h))

    @property
    def sum_delta(self):
        return float(self.L.orc_sum_delta(self.h))

    @property
    def last_delta(self):
        return float(self.L.orc_last_delta(self.h))

    @property
    def frob2(self):
        return float(self.L.orc_frob2(self.h))

    @property
    def n_shrinks(self):
        return int(self.L.orc_n_shrinks(self.h))

    @property
    def last_sweeps(self):
        return int(self.L.orc_last_sweeps(self.h))


def hestenes_rows(A):
    """One-sided Jacobi on the rows of A. Returns (rows = sigma_j v_j^T sorted descending, sigma^2, sweeps)."""
    L = _load()
    A = np.array(A, dtype=np.float64, order="C", copy=True)
    n, D = A.shape
    s2 = np.zeros(n)
    sweeps = L.orc_hestenes_rows(A.ctypes.data, n, D, s2.ctypes.data)
    return A, s2, int(sweeps)


def sym_jacobi(Cm):
    """Cyclic two-sided Jacobi of a symmetric matrix. Returns (lam descending, Y with eigenvectors in columns)."""
    L = _load()
    Cm = np.array(Cm, dtype=np.float64, order="C", copy=True)
    n = Cm.shape[0]
    Y = np.zeros((n, n))
    lam = np.zeros(n)
    L.orc_sym_jacobi(Cm.ctypes.data, n, Y.ctypes.data, lam.ctypes.data)
    return lam, Y


def row_dot(a, b):
    """<a, b> in fp64, summed in index order: one entry of the Gram matrix the Gram route forms."""
    a = np.ascontiguousarray(a, dtype=np.float64)
    b = np.ascontiguousarray(b, dtype=np.float64)
    assert a.ndim == 1 and a.shape == b.shape
    return float(_load().orc_row_dot(a.ctypes.data, b.ctypes.data, a.shape[0]))


def topm_f32(alpha, m):
    L = _load()
    alpha = np.ascontiguousarray(alpha, dtype=np.float32)
    out = np.empty(max(int(m), 1), dtype=np.int64)
    rc = L.orc_topm_f32(alpha.ctypes.data, alpha.shape[0], int(m), out.ctypes.data)
    if rc != 0:
        raise ValueError("need 0 <= m <= N")
    return out[: int(m)].copy()


def cb_alpha(zhat, labels, n_classes):
    """alpha_i = clamp(<zhat_i, u_c(i)>, -1, 1) with u_c = sum of the class's zhat, normalised (0 if the sum is 0)."""
    zhat = np.asarray(zhat, dtype=np.float64)
    labels = np.asarray(labels)
    alpha = np.zeros(zhat.shape[0])
    for c in range(int(n_classes)):
        rows = np.nonzero(labels == c)[0]
        if rows.size == 0:
            continue
        s = np.zeros(zhat.shape[1])
        for i in rows:               # plain ordered sum, as the definition reads
            s += zhat[i]
        nrm = float(np.sqrt(np.dot(s, s)))
        u = s / nrm if nrm > 0.0 else np.zeros_like(s)
        alpha[rows] = np.clip(zhat[rows] @ u, -1.0, 1.0)
    return alpha


def cb_budgets(counts, keep_rate, rule="proportional"):
    """The class budgets k_c (Algorithm 1, class-balanced branch: "sum_c k_c = k"; the paper leaves the k_c open). The
    subset size is that of the plain selection, m = floor(keep*N + 0.5). Returns an int64 array with sum m.
    rule "proportional": class c gets floor(keep*N_c), and the rows still missing from m go one each to the classes
    with the largest fractional part keep*N_c - floor(keep*N_c) (equal parts: the lower class first) that are not yet
    full (largest-remainder rule).
    rule "equal": the m rows are dealt one at a time to the classes in turn, lowest class first, a class that has
    none left to give being passed over: every class ends with the same budget, up to one row and up to its size."""
    counts = np.asarray(counts, dtype=np.int64)
    m = keep_count(keep_rate, int(counts.sum()))
    if rule == "equal":
        kc = np.zeros(counts.size, dtype=np.int64)
        left = m
        while left > 0:
            for c in range(counts.size):
                if left == 0:
                    break
                if kc[c] < counts[c]:
                    kc[c] += 1
                    left -= 1
        return kc
    if rule != "proportional":
        raise ValueError("rule must be 'proportional' or 'equal'")
    q = float(keep_rate) * counts.astype(np.float64)
    kc = np.minimum(np.floor(q).astype(np.int64), counts)
    frac = q - np.floor(q)
    rem = m - int(kc.sum())
    open_classes = [c for c in range(counts.size) if kc[c] < counts[c]]
    for c in sorted(open_classes, key=lambda c: (-frac[c], c))[:max(rem, 0)]:
        kc[c] += 1
    return kc


def cb_select_from_alpha(alpha, labels, n_classes, keep_rate, rule="proportional"):
    """Per class the k_c (cb_budgets) rows greatest under (float32 alpha descending, index ascending); all kept indices
    ascending."""
    a32 = np.asarray(alpha).astype(np.float32)
    a32 = np.where(a32 == 0, np.float32(0), a32)     # -0 -> +0
    labels = np.asarray(labels)
    budgets = cb_budgets([int((labels == c).sum()) for c in range(int(n_classes))], keep_rate, rule)
    kept = []
    for c in range(int(n_classes)):
        rows = np.nonzero(labels == c)[0]
        kc = int(budgets[c])
        if kc == 0:
            continue
        order = sorted(rows.tolist(), key=lambda i: (-float(a32[i]), i))
        kept.extend(order[:kc])
    return np.array(sorted(kept), dtype=np.int64)


def cb_scores_and_selection(zhat, labels, n_classes, keep_rate, rule="proportional"):
    alpha = cb_alpha(zhat, labels, n_classes)
    return alpha, cb_select_from_alpha(alpha, labels, n_classes, keep_rate, rule)


def keep_count(keep_rate, N):
    return int(_load().orc_keep_count(float(keep_rate), int(N)))


def _round_to_bf16(x):
    """float64 values rounded to the nearest bf16 value (8 significant bits), ties to even; normal range only."""
    m, ex = np.frexp(np.asarray(x, dtype=np.float64))
    return np.ldexp(np.rint(np.ldexp(m, 8)), ex - 8)


def last_layer_rows(E, H):
    """The rows behind a batch given by factors (Method, definition of g_i, for a linear last layer of C x dh weights
    followed by C biases with a loss on the logits): g_i = [vec(e_i h_i^T) ; e_i], i.e. column c*dh + t is
    e_i[c] * h_i[t] and column C*dh + c is e_i[c], each value as a stored row of the factors' type holds it
    (float32: the product rounded to float32; bf16 bit patterns: the exact product rounded to bf16).
    E: N x C, H: N x dh, both float32 or both uint16 (bf16 bits). Returns N x C*(dh+1) of the same type."""
    E = np.ascontiguousarray(E)
    H = np.ascontiguousarray(H)
    assert E.dtype == H.dtype and E.ndim == 2 and H.ndim == 2 and E.shape[0] == H.shape[0]
    bf = E.dtype == np.uint16
    if bf:
        e = (E.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        h = (H.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    else:
        assert E.dtype == np.float32
        e, h = E.astype(np.float64), H.astype(np.float64)
    N, Cn = e.shape
    W = e[:, :, None] * h[:, None, :]          # N x C x dh, exact in float64 for both types
    rows = np.concatenate([W.reshape(N, -1), e], axis=1)
    if bf:
        r32 = _round_to_bf16(rows).astype(np.float32)  # exact: bf16 values
        return (r32.view(np.uint32) >> 16).astype(np.uint16)
    return rows.astype(np.float32)
