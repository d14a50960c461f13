"""Pins for the CPU oracle: it is checked against numpy's LAPACK SVD, closed forms and invariants that the
paper (arxiv 2510.02470) and the FD literature fix, never against itself or the HIP path.
"""
import itertools

import numpy as np
import pytest

import oracle
from oracle import Oracle
from paper_2510_02470_amd import inputs


def spec_norm_sym(M):
    return float(np.abs(np.linalg.eigvalsh((M + M.T) / 2)).max())


def lowrank_rows(rng, N, D, r, noise=0.0):
    A = rng.standard_normal((N, r)) @ (rng.standard_normal((r, D)) * (np.arange(1, r + 1)[:, None] ** -0.7))
    if noise:
        A = A + noise * rng.standard_normal((N, D))
    return A.astype(np.float32)


# ---------------------------------------------------------------- SVD routines vs LAPACK
@pytest.mark.parametrize("n,D,rank", [(8, 40, None), (9, 33, None), (16, 16, None), (12, 64, 5), (24, 10, None)])
def test_hestenes_matches_lapack(n, D, rank):
    rng = np.random.default_rng(n * 100 + D)
    A = rng.standard_normal((n, D))
    if rank:
        A = rng.standard_normal((n, rank)) @ rng.standard_normal((rank, D))
    R, s2, sweeps = oracle.hestenes_rows(A)
    sv = np.linalg.svd(A, compute_uv=False)
    full = np.zeros(n)
    full[: len(sv)] = sv
    assert sweeps < 30
    assert np.abs(np.sqrt(s2) - full).max() <= 1e-12 * sv[0]
    # rows are sigma_j v_j^T: covariance kept, rows orthogonal, projector of the leading rows matches LAPACK's
    assert np.abs(R.T @ R - A.T @ A).max() <= 1e-11 * sv[0] ** 2
    Gm = R @ R.T
    assert np.abs(Gm - np.diag(np.diag(Gm))).max() <= 1e-12 * sv[0] ** 2
    rk = int((full > 1e-9 * sv[0]).sum())
    kk = max(1, rk // 2)
    _, s_l, Vt = np.linalg.svd(A, full_matrices=False)
    if s_l[kk - 1] - s_l[kk] > 1e-3 * s_l[0]:
        Vo = R[:kk] / np.sqrt(s2[:kk])[:, None]
        assert np.abs(Vo.T @ Vo - Vt[:kk].T @ Vt[:kk]).max() <= 1e-9


@pytest.mark.parametrize("n", [2, 7, 16, 33])
def test_sym_jacobi_matches_lapack(n):
    rng = np.random.default_rng(n)
    X = rng.standard_normal((n, n + 3))
    Cm = X @ X.T
    lam, Y = oracle.sym_jacobi(Cm)
    ref = np.linalg.eigvalsh(Cm)[::-1]
    assert np.abs(lam - ref).max() <= 1e-12 * ref[0]
    assert np.abs(Y.T @ Y - np.eye(n)).max() <= 1e-13
    assert np.abs(Y @ np.diag(lam) @ Y.T - Cm).max() <= 1e-12 * ref[0]
    assert np.all(np.diff(lam) <= 0)


# ---------------------------------------------------------------- FD: closed forms
@pytest.mark.parametrize("mode", [0, 1])
def test_no_shrink_regime_is_exact(mode):
    """N < 2*ell: nothing is shrunk, B^T B = A^T A, the basis is the top-k right singular space of A and the
    scores and selection follow from the plain definitions (Method, 'Two-pass scoring')."""
    rng = np.random.default_rng(3)
    ell, D, N, k = 8, 24, 13, 4
    A = rng.standard_normal((N, D)).astype(np.float32) * np.linspace(3, 0.2, N)[:, None].astype(np.float32)
    o = Oracle(ell, D, mode)
    o.update(A[:5])
    o.update(A[5:])
    assert o.n_shrinks == 0 and o.fill == N and o.sum_delta == 0.0
    A64 = A.astype(np.float64)
    assert np.abs(o.B.T @ o.B - A64.T @ A64).max() == 0.0
    assert abs(o.frob2 - (A64 ** 2).sum()) <= 1e-12 * (A64 ** 2).sum()
    o.basis(k)
    _, sv, Vt = np.linalg.svd(A64, full_matrices=False)
    P = Vt[:k].T @ Vt[:k]
    assert np.abs(o.V.T @ o.V - P).max() <= 1e-10
    o.score(A)
    idx = o.select(0.3)
    Z = A64 @ Vt[:k].T
    Zh = Z / np.linalg.norm(Z, axis=1, keepdims=True)
    zbar = Zh.mean(0)
    u = zbar / np.linalg.norm(zbar)
    alpha = Zh @ u
    assert np.abs(o.alpha - alpha).max() <= 1e-10
    m = int(np.floor(0.3 * N + 0.5))
    expect = np.sort(np.argsort(-alpha.astype(np.float32), kind="stable")[:m])
    assert idx.tolist() == expect.tolist()


@pytest.mark.parametrize("mode", [0, 1])
def test_one_shrink_closed_form(mode):
    """N = 2*ell: exactly one shrink, B^T B = V max(Sigma^2 - sigma_ell^2, 0) V^T (Method, FD paragraph)."""
    rng = np.random.default_rng(5)
    ell, D = 6, 20
    A = rng.standard_normal((2 * ell, D)).astype(np.float32)
    o = Oracle(ell, D, mode)
    o.update(A)
    A64 = A.astype(np.float64)
    _, sv, Vt = np.linalg.svd(A64, full_matrices=False)
    delta = sv[ell - 1] ** 2
    want = Vt.T @ np.diag(np.maximum(sv ** 2 - delta, 0.0)) @ Vt
    assert o.n_shrinks == 1 and o.fill == ell
    assert abs(o.sum_delta - delta) <= 1e-12 * sv[0] ** 2
    assert np.abs(o.B.T @ o.B - want).max() <= 1e-11 * sv[0] ** 2
    # at least ell+1 rows are exactly zero after the shrink: rows ell-1 .. n-1
    assert np.all(o.B[ell - 1:] == 0.0)
    # the kept rows are mutually orthogonal with squared norms sigma_j^2 - delta
    Gm = o.B[: ell - 1] @ o.B[: ell - 1].T
    assert np.abs(Gm - np.diag(sv[: ell - 1] ** 2 - delta)).max() <= 1e-11 * sv[0] ** 2


@pytest.mark.parametrize("mode", [0, 1])
def test_low_rank_exact_recovery(mode):
    """rank(A) <= ell-1: every delta is 0 and the sketch reproduces A^T A."""
    rng = np.random.default_rng(7)
    ell, D, N, r = 8, 40, 100, 6
    A = lowrank_rows(rng, N, D, r)
    o = Oracle(ell, D, mode)
    for lo in range(0, N, 17):
        o.update(A[lo:lo + 17])
    A64 = A.astype(np.float64)
    cov = A64.T @ A64
    assert o.n_shrinks == (N - 2 * ell) // ell + 1
    assert o.sum_delta <= 1e-12 * np.trace(cov)
    assert spec_norm_sym(o.B.T @ o.B - cov) <= 1e-10 * np.trace(cov)


@pytest.mark.parametrize("mode", [0, 1])
def test_fd_invariants(mode):
    """0 <= A^T A - B^T B, ||A^T A - B^T B||_2 <= sum(delta) <= ||A||_F^2 / ell, and
    ell * sum(delta) <= ||A||_F^2 - ||B||_F^2 (Method, FD guarantee; Liberty's argument for the 2*ell buffer)."""
    rng = np.random.default_rng(11)
    ell, D, N = 8, 48, 203
    A = lowrank_rows(rng, N, D, 20, noise=0.3)
    o = Oracle(ell, D, mode)
    seen = 0
    for lo in range(0, N, 29):
        o.update(A[lo:lo + 29])
        seen = min(N, lo + 29)
        A64 = A[:seen].astype(np.float64)
        diff = A64.T @ A64 - o.B.T @ o.B
        ev = np.linalg.eigvalsh(diff)
        fro = (A64 ** 2).sum()
        assert ev.min() >= -1e-10 * fro
        assert ev.max() <= o.sum_delta + 1e-10 * fro
        assert o.sum_delta <= fro / ell + 1e-10 * fro
        assert ell * o.sum_delta <= fro - (o.B ** 2).sum() + 1e-9 * fro
        assert abs(o.frob2 - fro) <= 1e-12 * fro
        assert np.all(o.B[o.fill:] == 0.0)
    assert o.rows_seen == N and o.n_shrinks == (N - 2 * ell) // ell + 1
    # the paper's form of the bound with k = ell/2: (2/ell) * ||A - A_k||_F^2
    sv = np.linalg.svd(A.astype(np.float64), compute_uv=False)
    assert o.sum_delta <= (2.0 / ell) * (sv[ell // 2:] ** 2).sum() + 1e-10 * (sv ** 2).sum()


def test_modes_agree_on_cfg1_shape():
    """Hestenes route and Gram route give the same sketch covariance, scores and selection."""
    w = inputs.WORKLOADS[1].scaled(N=512)
    G = inputs.generate_numpy(w)
    res = []
    for mode in (0, 1):
        o = Oracle(w.ell, w.D, mode)
        for lo in range(0, w.N, w.batch):
            o.update(G[lo:lo + w.batch])
        o.basis(w.k)
        o.score(G)
        idx = o.select(w.keep)
        res.append((o.B.T @ o.B, o.alpha, idx, o.sum_delta))
    fro = (G.astype(np.float64) ** 2).sum()
    assert np.abs(res[0][0] - res[1][0]).max() <= 1e-10 * fro
    assert abs(res[0][3] - res[1][3]) <= 1e-10 * fro
    assert np.abs(res[0][1] - res[1][1]).max() <= 1e-7
    assert res[0][2].tolist() == res[1][2].tolist()


def test_row_dot_is_the_plain_dot_product():
    """The Gram entry the Gram route forms: exact on integer vectors, and equal to the correctly rounded sum
    (math.fsum) to a few ulp on random ones."""
    import math

    rng = np.random.default_rng(2)
    a = rng.integers(-1000, 1000, size=5000).astype(np.float64)
    b = rng.integers(-1000, 1000, size=5000).astype(np.float64)
    assert oracle.row_dot(a, b) == float(int(a.astype(np.int64) @ b.astype(np.int64)))
    x, y = rng.standard_normal(20000), rng.standard_normal(20000)
    exact = math.fsum((x * y).tolist())     # each product rounded once, then summed exactly
    assert abs(oracle.row_dot(x, y) - exact) <= 1e-13 * float(np.abs(x * y).sum())
    assert oracle.row_dot(x, x) > 0 and oracle.row_dot(x, y) == oracle.row_dot(y, x)


@pytest.mark.parametrize("ell,D,cycles,dtype", [(64, 1024, 4, "f32"), (128, 600, 3, "bf16")])
def test_modes_agree_at_larger_sketch_sizes(ell, D, cycles, dtype):
    """The Gram route (mode 1), which the long GPU parity runs and the full-size fixtures use, against the one-sided
    Jacobi on the rows (mode 0, the definition) at ell = 64 and ell = 128, on slowly decaying spectra like those of the
    second and third workload: the same sketch covariance and sum(delta) to 1e-10 relative, and the same top-k energy."""
    w = inputs.WORKLOADS[3].scaled(N=ell * (cycles + 1) + 29, D=D, ell=ell, k=ell // 2, batch=300, r=3 * ell // 2, dtype=dtype)
    G = inputs.generate_numpy(w)
    A = inputs.bf16_bits_to_f32(G) if G.dtype == np.uint16 else G
    fro = (A.astype(np.float64) ** 2).sum()
    res = []
    for mode in (0, 1):
        o = Oracle(w.ell, w.D, mode)
        for lo in range(0, w.N, w.batch):
            o.update(G[lo:lo + w.batch])
        o.basis(w.k)
        res.append((o.B.T @ o.B, o.sum_delta, o.sig2.copy(), o.n_shrinks))
    assert res[0][3] == res[1][3] == cycles
    assert np.abs(res[0][0] - res[1][0]).max() <= 1e-10 * fro
    assert abs(res[0][1] - res[1][1]) <= 1e-10 * fro
    assert np.abs(res[0][2] - res[1][2]).max() <= 1e-10 * fro


def test_orthogonal_invariance():
    """Right-multiplying every row by an orthogonal Q leaves sum(delta), the scores and the selection unchanged."""
    rng = np.random.default_rng(13)
    ell, D, N, k = 4, 12, 37, 2
    A = lowrank_rows(rng, N, D, 8, noise=0.2).astype(np.float64)
    Q, _ = np.linalg.qr(rng.standard_normal((D, D)))
    # rows must be exactly representable on both sides: round the rotated rows to fp32 and rotate back in fp64
    A1 = A.astype(np.float32)
    A2 = (A1.astype(np.float64) @ Q).astype(np.float32)
    outs = []
    for rows in (A1, A2):
        o = Oracle(ell, D, 0)
        o.update(rows)
        o.basis(k)
        o.score(rows)
        idx = o.select(0.25)
        outs.append((o.sum_delta, o.alpha, idx))
    assert abs(outs[0][0] - outs[1][0]) <= 1e-5 * outs[0][0]
    assert np.abs(outs[0][1] - outs[1][1]).max() <= 1e-4


# ---------------------------------------------------------------- scoring identities
def _scored(rng, N=60, D=16, ell=6, k=3):
    A = lowrank_rows(rng, N, D, 5, noise=0.1)
    A[:, :] += 0.5 * rng.standard_normal(D).astype(np.float32)  # common mean so the consensus is not tiny
    o = Oracle(ell, D, 0)
    o.update(A)
    o.basis(k)
    o.score(A)
    return o, A


def test_score_range_mean_and_lemma():
    """alpha in [-1,1]; mean(alpha) = ||zbar||_2; the consensus-direction energy identity and the mean-alignment
    bound (Method, Lemma 'Consensus-direction energy' and its corollary)."""
    rng = np.random.default_rng(17)
    o, A = _scored(rng)
    idx = o.select(0.2)
    al = o.alpha
    N = len(al)
    assert np.all(al <= 1.0) and np.all(al >= -1.0)
    zbar = o.zhat.mean(0)
    assert abs(al.mean() - np.linalg.norm(zbar)) <= 1e-12
    assert abs(np.linalg.norm(o.u) - 1.0) <= 1e-12
    V = o.V
    Z = A.astype(np.float64) @ V.T
    T = idx
    lhs = ((Z[T] @ o.u) ** 2).sum()
    mid = ((np.linalg.norm(Z[T], axis=1) ** 2) * al[T] ** 2).sum()
    xi = al[T].min()
    assert abs(lhs - mid) <= 1e-10 * max(lhs, 1e-300)
    if xi > 0:
        assert mid >= xi ** 2 * (np.linalg.norm(Z[T], axis=1) ** 2).sum() - 1e-12
        assert np.linalg.norm(Z[T].mean(0)) >= xi * np.linalg.norm(Z[T], axis=1).mean() - 1e-12
    assert len(T) == int(np.floor(0.2 * N + 0.5))


def test_rank_one_basis_gives_signs():
    """k = 1: zhat is +-1 (or 0), so alpha is +1 for the majority sign, -1 for the minority, 0 for null rows."""
    rng = np.random.default_rng(19)
    D, ell = 10, 4
    v = rng.standard_normal(D)
    v /= np.linalg.norm(v)
    coef = np.array([3, 2, -1, 4, 5, -2, 1, 6, 0], dtype=np.float64)
    A = (coef[:, None] * v[None, :]).astype(np.float32)
    o = Oracle(ell, D, 0)
    o.set_basis(v[None, :])
    o.score(A)
    o.select(0.5)
    want = np.sign(coef)
    got = o.alpha
    # fp32 rounding of the rows cannot flip a sign here
    assert np.all(np.abs(got - want) <= 1e-12)


def test_identical_and_opposed_rows():
    rng = np.random.default_rng(23)
    D, ell, k = 12, 4, 2
    g = rng.standard_normal(D).astype(np.float32)
    h = rng.standard_normal(D).astype(np.float32)
    o = Oracle(ell, D, 0)
    o.update(np.stack([g, h, g + h]))
    o.basis(k)
    o.score(np.stack([g] * 5))
    o.select(1.0)
    assert np.abs(o.alpha - 1.0).max() <= 1e-12
    o.basis(k)
    o.score(np.stack([g, g, g, -g, 2 * g, -3 * g, g]))
    o.select(1.0)
    assert np.abs(o.alpha - np.array([1, 1, 1, -1, 1, -1, 1.0])).max() <= 1e-12


def test_zero_rows_and_zero_consensus():
    """zhat = 0 when z = 0 (still counted in N); u = 0 when zbar = 0, then every alpha is 0."""
    D, ell = 8, 4
    V = np.eye(D)[:2]
    rows = np.zeros((4, D), dtype=np.float32)
    rows[0, 0] = 2.0
    rows[1, 0] = -2.0
    rows[2, 5] = 1.0  # orthogonal to the basis: z = 0
    o = Oracle(ell, D, 0)
    o.set_basis(V)
    o.score(rows)
    idx = o.select(0.5)
    assert o.n_scored == 4
    assert np.all(o.zhat[2] == 0.0) and np.all(o.zhat[3] == 0.0)
    assert np.all(o.u == 0.0) and np.all(o.alpha == 0.0)
    assert not np.any(np.signbit(o.alpha))
    assert idx.tolist() == [0, 1]  # all tied: lowest indices win


def test_metamorphic_scaling_permutation_rotation():
    rng = np.random.default_rng(29)
    N, D, ell, k = 40, 14, 6, 3
    A = lowrank_rows(rng, N, D, 5, noise=0.1) + 0.3
    V, _ = np.linalg.qr(rng.standard_normal((D, k)))
    V = V.T

    def run(rows, basis):
        o = Oracle(ell, D, 0)
        o.set_basis(basis)
        o.score(rows.astype(np.float32))
        o.select(0.3)
        return o.alpha

    base = run(A, V)
    scale = (2.0 ** rng.integers(-3, 4, size=N)).astype(np.float32)  # exact in fp32
    assert np.abs(run(A * scale[:, None], V) - base).max() <= 1e-12
    perm = rng.permutation(N)
    assert np.abs(run(A[perm], V) - base[perm]).max() <= 1e-12
    Rk, _ = np.linalg.qr(rng.standard_normal((k, k)))
    assert np.abs(run(A, Rk @ V) - base).max() <= 1e-12
    assert np.abs(run(A, -V) - base).max() <= 1e-12


def test_rank_deficient_basis_zeroes_direction():
    """A direction with sigma_j^2 <= n 2^-23 sigma_1^2 is returned as the zero vector and the call succeeds."""
    rng = np.random.default_rng(31)
    D, ell, k = 16, 6, 4
    A = lowrank_rows(rng, 9, D, 2)
    o = Oracle(ell, D, 0)
    o.update(A)
    o.basis(k)
    V = o.V
    nz = np.linalg.norm(V, axis=1)
    assert np.all(np.abs(nz[:2] - 1.0) <= 1e-12) and np.all(nz[2:] == 0.0)


# ---------------------------------------------------------------- selection
def test_topm_exhaustive_small():
    vals = [-1.0, 0.0, 0.5]
    for N in range(0, 6):
        for combo in itertools.product(vals, repeat=N):
            a = np.array(combo, dtype=np.float32)
            for m in range(0, N + 1):
                got = oracle.topm_f32(a, m).tolist()
                order = sorted(range(N), key=lambda i: (-float(a[i]), i))[:m]
                assert got == sorted(order)


def test_topm_random_with_ties_and_keep_count():
    rng = np.random.default_rng(37)
    a = np.round(rng.standard_normal(5000), 1).astype(np.float32)
    for m in (0, 1, 17, 2500, 4999, 5000):
        got = oracle.topm_f32(a, m)
        order = np.lexsort((np.arange(len(a)), -a))[:m]
        assert got.tolist() == sorted(order.tolist())
    assert oracle.keep_count(0.1, 2048) == 205
    assert oracle.keep_count(0.05, 50000) == 2500
    assert oracle.keep_count(0.0, 10) == 0 and oracle.keep_count(1.0, 10) == 10
    assert oracle.keep_count(0.25, 10) == 3 and oracle.keep_count(0.24, 10) == 2
    with pytest.raises(ValueError):
        oracle.topm_f32(a, len(a) + 1)


def test_bf16_rows_are_widened_exactly():
    rng = np.random.default_rng(41)
    A = rng.standard_normal((10, 12)).astype(np.float32)
    h = inputs.f32_to_bf16_bits(A)
    back = inputs.bf16_bits_to_f32(h)
    assert np.abs(back - A).max() <= 2.0 ** -8 * np.abs(A).max()
    assert np.array_equal(inputs.f32_to_bf16_bits(back), h)
    o1, o2 = Oracle(6, 12, 0), Oracle(6, 12, 0)
    o1.update(h)
    o2.update(back)
    assert np.array_equal(o1.B, o2.B)
    o1.basis(2)
    o2.basis(2)
    o1.score(h)
    o2.score(back)
    assert np.array_equal(o1.zhat, o2.zhat)


# ---------------------------------------------------------------- sketch-weighted basis (the paper's z = S g)
@pytest.mark.parametrize("mode", [0, 1])
def test_weighted_basis_is_the_sketch_a_shrink_would_write(mode):
    """Method, "Two-pass scoring": z = S g with S = Sigma' V^T. Pins: (1) against LAPACK, the rows are
    sqrt(sigma_j^2 - sigma_ell^2) v_j^T of the buffer as it stands; (2) taken right after a shrink they are the
    sketch rows themselves; (3) scores are then the plain definition on S g."""
    rng = np.random.default_rng(11 + mode)
    ell, D, k = 8, 40, 5
    A = lowrank_rows(rng, 3 * ell + 5, D, 12, noise=0.05)   # buffer ends partly filled
    o = Oracle(ell, D, mode)
    o.update(A)
    Bbuf = o.B.copy()
    o.basis(k, weighted=True)
    S = o.V
    U, sv, Vt = np.linalg.svd(Bbuf, full_matrices=False)
    delta = sv[ell - 1] ** 2
    wgt = np.sqrt(np.maximum(sv[:k] ** 2 - delta, 0.0))
    want = (wgt[:, None] * Vt[:k])
    assert np.abs(S.T @ S - want.T @ want).max() <= 1e-10 * sv[0] ** 2          # sign-free comparison
    assert np.abs(np.abs(np.sum(S * want, axis=1)) - wgt ** 2).max() <= 1e-10 * sv[0] ** 2
    assert np.array_equal(o.B, Bbuf)                                             # the sketch is untouched
    # (3) scores from the plain definition on S g
    o.score(A)
    idx = o.select(0.25)
    Z = A.astype(np.float64) @ S.T
    Zh = Z / np.linalg.norm(Z, axis=1, keepdims=True)
    u = Zh.sum(0) / np.linalg.norm(Zh.sum(0))
    al = np.clip(Zh @ u, -1, 1)
    assert np.abs(o.alpha - al).max() <= 1e-12
    assert idx.tolist() == sorted(np.lexsort((np.arange(len(al)), -al))[: len(idx)].tolist())
    # (2) right after a shrink (exactly 2*ell + m*ell rows) the weighted basis is the sketch
    o2 = Oracle(ell, D, mode)
    o2.update(A[: 3 * ell])
    assert o2.fill == ell
    Bs = o2.B.copy()
    o2.basis(k, weighted=True)
    S2 = o2.V
    for j in range(k):
        sgn = np.sign(np.dot(S2[j], Bs[j])) or 1.0
        assert np.abs(S2[j] - sgn * Bs[j]).max() <= 1e-9 * np.abs(Bs).max()


# ---------------------------------------------------------------- class-balanced selection (CB-SAGE)
def test_cb_selection_matches_per_class_plain_selection():
    """Algorithm 1, "if class balance required". Pins: (1) with one class it is the plain selection; (2) class by class
    the scores equal the plain (already pinned) scoring run on that class's rows alone with the same basis, and the kept
    rows are the plain top-m of those scores with m = the class budget; (3) the budgets sum to the plain selection's m;
    (4) renaming the classes leaves every score unchanged."""
    rng = np.random.default_rng(77)
    ell, D, k, N, Cn = 8, 30, 4, 90, 5
    A = lowrank_rows(rng, N, D, 6, noise=0.1)
    A[17] = A[3]                     # ties inside a class
    A[40] = 0.0                      # a zero row
    labels = rng.integers(0, Cn - 1, size=N)    # class Cn-1 stays empty
    labels[17] = labels[3]
    o = Oracle(ell, D, 1)
    o.update(A)
    o.basis(k)
    V = o.V.copy()
    o.score(A)
    plain_idx = o.select(0.3)
    plain_alpha = o.alpha.copy()
    # (1) one class
    al1, idx1 = o.select_cb(0.3, np.zeros(N, dtype=np.int64), 1)
    assert np.abs(al1 - plain_alpha).max() <= 1e-12 and idx1.tolist() == plain_idx.tolist()
    # (2), (3) class by class through the plain path
    al, idx = o.select_cb(0.3, labels, Cn)
    got = set(idx.tolist())
    budgets = oracle.cb_budgets([int((labels == c).sum()) for c in range(Cn)], 0.3)
    assert budgets.sum() == len(plain_idx) == len(idx)
    for c in range(Cn):
        rows = np.nonzero(labels == c)[0]
        if rows.size == 0:
            assert budgets[c] == 0
            continue
        oc = Oracle(ell, D, 1)
        oc.set_basis(V)
        oc.score(A[rows])
        oc.select(0.3)
        assert np.abs(oc.alpha - al[rows]).max() <= 1e-12
        sub = oracle.topm_f32(oc.alpha.astype(np.float32), int(budgets[c]))
        assert sorted(rows[sub].tolist()) == sorted(i for i in got if labels[i] == c)
    assert idx.tolist() == sorted(idx.tolist())
    assert (al <= 1).all() and (al >= -1).all()
    # (4) renaming classes
    perm = rng.permutation(Cn)
    al2, idx2 = o.select_cb(0.3, perm[labels], Cn)
    assert np.array_equal(al2, al) and len(idx2) == len(idx)


def test_cb_budgets_sum_to_the_subset_size():
    """Algorithm 1, class-balanced branch: "sum_c k_c = k". The largest-remainder budgets against an exact rational
    re-statement of the rule (keep rates that are dyadic, so that keep * N_c is exact in fp64 too), and the properties
    that hold for any rate: the sum is the plain m, every class is within one row of its share, none above its size."""
    from fractions import Fraction

    rng = np.random.default_rng(5)
    for keep in (0.25, 0.375, 0.0625, 0.5, 1.0, 0.0):
        for trial in range(20):
            Cn = int(rng.integers(1, 40))
            counts = rng.integers(0, 30, size=Cn)
            got = oracle.cb_budgets(counts, keep)
            kf = Fraction(keep)
            N = int(counts.sum())
            m = min(N, max(0, int(kf * N + Fraction(1, 2))))          # floor(keep N + 1/2), exactly
            base = [int(kf * int(n)) for n in counts]
            frac = [kf * int(n) - b for n, b in zip(counts, base)]
            order = sorted((c for c in range(Cn) if base[c] < counts[c]), key=lambda c: (-frac[c], c))
            for c in order[: m - sum(base)]:
                base[c] += 1
            assert got.tolist() == base and got.sum() == m
    for keep in (0.01, 0.05, 0.1, 0.3, 0.77):
        counts = rng.integers(0, 200, size=300)
        got = oracle.cb_budgets(counts, keep)
        assert got.sum() == oracle.keep_count(keep, int(counts.sum()))
        assert (got <= counts).all() and (np.abs(got - keep * counts) < 1.0).all()
    # many small classes at a low rate: rounding every class on its own would keep nothing at all
    counts = np.full(1000, 20)
    counts[:480] += 1                                                   # 20,480 rows
    got = oracle.cb_budgets(counts, 0.01)
    assert got.sum() == 205 and got.max() == 1
    assert got[:480].sum() == 205                                       # the larger classes have the larger remainders


def test_cb_equal_budgets_are_the_most_even_split():
    """Rule "equal" of the class budgets. Against brute force on tiny inputs: among all integer vectors with
    0 <= k_c <= N_c and sum m, the budgets are the one with the smallest sum of squares (the most even split), and
    among those of that sum of squares the lexicographically greatest (spare rows go to the lower classes). Then the
    closed form for classes that are all large enough, and the properties that hold for any input."""
    import itertools

    rng = np.random.default_rng(17)
    for trial in range(60):
        Cn = int(rng.integers(1, 5))
        counts = rng.integers(0, 6, size=Cn)
        N = int(counts.sum())
        for keep in (0.0, 0.2, 0.5, 0.8, 1.0):
            m = oracle.keep_count(keep, N)
            got = oracle.cb_budgets(counts, keep, "equal")
            feas = [v for v in itertools.product(*[range(int(n) + 1) for n in counts]) if sum(v) == m]
            best = min(sum(x * x for x in v) for v in feas)
            want = max(v for v in feas if sum(x * x for x in v) == best)
            assert tuple(got.tolist()) == want, (counts, keep, got, want)
    # every class large enough: floor(m / C) each, the m mod C spare rows to the first classes
    counts = np.full(7, 1000)
    got = oracle.cb_budgets(counts, 0.0147, "equal")             # m = 103
    assert got.tolist() == [15, 15, 15, 15, 15, 14, 14]
    for keep in (0.01, 0.1, 0.33, 0.9):
        counts = rng.integers(0, 120, size=200)
        got = oracle.cb_budgets(counts, keep, "equal")
        assert got.sum() == oracle.keep_count(keep, int(counts.sum())) and (got <= counts).all() and (got >= 0).all()
        open_c = got < counts                                     # classes that could have given more
        if open_c.any():
            lvl = got[open_c]
            assert lvl.max() - lvl.min() <= 1
            assert (got[~open_c] <= lvl.max()).all()              # a class is full only at or below the common level
            hi = np.nonzero(open_c & (got == lvl.max()))[0]
            lo = np.nonzero(open_c & (got == lvl.min()))[0]
            if lvl.max() > lvl.min():
                assert hi.max() < lo.min()                        # the spare rows went to the lower classes
    # the two rules differ where class sizes do: proportional follows the sizes, equal does not
    counts = np.array([1000, 100, 10])
    assert oracle.cb_budgets(counts, 0.1, "proportional").tolist() == [100, 10, 1]
    assert oracle.cb_budgets(counts, 0.1, "equal").tolist() == [51, 50, 10]
    with pytest.raises(ValueError):
        oracle.cb_budgets(counts, 0.1, "other")


def test_sketches_merge_with_added_bounds():
    """Mergeability (a property of Frequent Directions, the sketch the Method section uses): feeding the rows of the
    sketch of A2 to the sketch of A1 as data gives B with 0 <= A^T A - B^T B and
    ||A^T A - B^T B||_2 <= sum_delta(merged context) + sum_delta(second sketch), A = [A1; A2]."""
    rng = np.random.default_rng(23)
    ell, D = 8, 40
    A1 = lowrank_rows(rng, 120, D, 12, noise=0.2)
    A2 = lowrank_rows(rng, 95, D, 12, noise=0.2)
    o1, o2 = Oracle(ell, D, 0), Oracle(ell, D, 0)
    o1.update(A1)
    o2.update(A2)
    B2 = o2.B[:o2.fill].astype(np.float32)  # what a merge sends: fp32 rows
    o1.update(B2)
    A = np.vstack([A1, A2]).astype(np.float64)
    diff = A.T @ A - o1.B.T @ o1.B
    ev = np.linalg.eigvalsh(diff)
    fro = (A ** 2).sum()
    assert ev.min() >= -1e-6 * fro  # fp32 rounding of the rows sent
    assert ev.max() <= o1.sum_delta + o2.sum_delta + 1e-6 * fro
    assert o1.sum_delta + o2.sum_delta <= fro / ell + 1e-6 * fro



# ---------------------------------------------------------------- factored last-layer rows
def test_last_layer_rows_are_the_autograd_gradient():
    """Layout and sign of oracle.last_layer_rows against torch's autograd: the gradient of the cross-entropy of a linear
    layer (weights C x dh row-major, then biases) for one example is (softmax - onehot) (x) [h; 1]."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(41)
    Cn, dh, N = 5, 7, 6
    W = torch.tensor(rng.standard_normal((Cn, dh)), dtype=torch.float64, requires_grad=True)
    b = torch.tensor(rng.standard_normal(Cn), dtype=torch.float64, requires_grad=True)
    Hm = rng.standard_normal((N, dh))
    y = rng.integers(0, Cn, size=N)
    logits = Hm @ W.detach().numpy().T + b.detach().numpy()
    P = np.exp(logits - logits.max(axis=1, keepdims=True))
    P /= P.sum(axis=1, keepdims=True)
    E = P.copy()
    E[np.arange(N), y] -= 1.0
    rows = oracle.last_layer_rows(E.astype(np.float32), Hm.astype(np.float32))
    assert rows.shape == (N, Cn * (dh + 1))
    for i in range(N):
        loss = torch.nn.functional.cross_entropy((torch.tensor(Hm[i]) @ W.T + b)[None, :], torch.tensor([int(y[i])]))
        gW, gb = torch.autograd.grad(loss, [W, b])
        ref = np.concatenate([gW.numpy().reshape(-1), gb.numpy()])
        assert np.abs(rows[i] - ref).max() <= 2e-7 * max(1.0, np.abs(ref).max())


def test_last_layer_rows_gram_closed_form_and_bf16_rounding():
    """<g_i, g_j> = <e_i, e_j> (<h_i, h_j> + 1): exact for small-integer factors in both row types. The bf16 rounding
    of the products against torch's own float32 -> bfloat16 conversion on random factors."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(42)
    E = rng.integers(-3, 4, size=(9, 4)).astype(np.float32)
    Hm = rng.integers(-3, 4, size=(9, 6)).astype(np.float32)
    want = (E.astype(np.float64) @ E.T) * (Hm.astype(np.float64) @ Hm.T + 1.0)
    R32 = oracle.last_layer_rows(E, Hm).astype(np.float64)
    assert np.array_equal(R32 @ R32.T, want)
    Rb = oracle.last_layer_rows(inputs.f32_to_bf16_bits(E), inputs.f32_to_bf16_bits(Hm))
    Rb = inputs.bf16_bits_to_f32(Rb).astype(np.float64)
    assert np.array_equal(Rb @ Rb.T, want)
    # random bf16 factors: products need rounding
    Eb = inputs.f32_to_bf16_bits(rng.standard_normal((16, 8)).astype(np.float32))
    Hb = inputs.f32_to_bf16_bits(rng.standard_normal((16, 32)).astype(np.float32))
    got = oracle.last_layer_rows(Eb, Hb)
    e = torch.from_numpy(inputs.bf16_bits_to_f32(Eb))
    h = torch.from_numpy(inputs.bf16_bits_to_f32(Hb))
    prod = (e[:, :, None] * h[:, None, :]).reshape(16, -1)  # exact in float32
    ref = torch.cat([prod, e], dim=1).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, ref)


# ---------------------------------------------------------------- host-side sanitizer run
def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """oracle/sanitize_check.c drives every entry point of the oracle (both SVD routes, shrink cycles, bases, scoring of
    fp32 and bf16 rows, selection, error returns) in a build with -fsanitize=address,undefined: an out-of-bounds
    access, a leak or an undefined operation anywhere in it ends the run with a non-zero status."""
    import os
    import subprocess

    src = os.path.join(os.path.dirname(os.path.abspath(oracle.__file__)))
    exe = str(tmp_path / "sanitize_check")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-o", exe, os.path.join(src, "sanitize_check.c"), os.path.join(src, "sage_oracle.c"), "-lm"]
    b = subprocess.run(cmd, capture_output=True, text=True)
    if b.returncode != 0 and "asan" in b.stderr.lower():
        pytest.skip("this gcc has no AddressSanitizer runtime: " + b.stderr.strip().splitlines()[-1])
    assert b.returncode == 0, b.stderr
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "sanitize_check ok" in r.stdout, r.stdout + r.stderr
