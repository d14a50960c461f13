"""Shared checks for the parity tests (no method arithmetic: only comparison metrics)."""
import numpy as np


def cov_diff_spec_norm(B1, B2):
    """||B1^T B1 - B2^T B2||_2 without forming D x D: the non-zero eigenvalues of W^T J W (W = [B1; B2],
    J = diag(I, -I)) are those of J W W^T, a small matrix."""
    B1 = np.asarray(B1, dtype=np.float64)
    B2 = np.asarray(B2, dtype=np.float64)
    W = np.vstack([B1, B2])
    K = W @ W.T
    J = np.concatenate([np.ones(B1.shape[0]), -np.ones(B2.shape[0])])
    ev = np.linalg.eigvals(J[:, None] * K)
    return float(np.abs(ev).max())


def run_oracle(w, G, mode=1, k=None, keep=None, score=True):
    """The whole path on the CPU oracle. Returns the Oracle (scored and selected) and the selected indices."""
    from oracle import Oracle

    o = Oracle(w.ell, w.D, mode)
    for lo in range(0, G.shape[0], w.batch):
        o.update(G[lo:lo + w.batch])
    idx = None
    if score:
        o.basis(k or w.k)
        for lo in range(0, G.shape[0], w.batch):
            o.score(G[lo:lo + w.batch])
        idx = o.select(w.keep if keep is None else keep)
    return o, idx


def to_dev(G, torch):
    """Host rows (float32, or uint16 bf16 bit patterns) -> device tensor of the matching dtype."""
    if G.dtype == np.uint16:
        return torch.from_numpy(G.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(G).cuda()


def run_gpu(w, G, k=None, keep=None, score=True, arithmetic=None):
    import torch
    from paper_2510_02470_amd.binding import Sage

    s = Sage(w.ell, w.D, dtype=w.dtype)
    if arithmetic is not None:
        s.set_update_arithmetic(arithmetic)
    Gd = to_dev(G, torch)
    for lo in range(0, G.shape[0], w.batch):
        s.fd_update(Gd[lo:lo + w.batch])
    idx = None
    if score:
        s.fd_basis(k or w.k)
        for lo in range(0, G.shape[0], w.batch):
            s.score(Gd[lo:lo + w.batch])
        idx = s.select(w.keep if keep is None else keep)
    return s, idx


def check_basis_and_scores(s, w, G, o, fro, keep=None, score_tol=1e-4, sample=None, cov_err=None):
    """End-to-end check that does not depend on how well conditioned the top-k subspace is.

    s: the GPU context after sage_fd_basis, a full scoring pass over G and sage_select; o: the oracle after the same
    stream and basis(k) (its sig2 = squared singular values of its frozen buffer), or a fixture holding sig2 and alpha;
    fro = ||A||_F^2.
    The top-k subspace of a slowly decaying spectrum moves by far more than 1e-4 under a covariance change of 1e-7,
    so the two bases need not agree; what must hold is that the GPU's basis is *a* correct top-k basis of the GPU's
    own sketch and that its scores are the scores of that basis:
      1. V V^T = I to 1e-5;
      2. span(V) is invariant under the GPU sketch's covariance: ||B^T B V - V (V^T B^T B V)||_2 <= 1e-6 ||A||_F^2;
      3. it captures the top-k energy: tr(V^T B^T B V) equals the sum of the k largest eigenvalues of the GPU sketch's
         own B B^T (LAPACK) to 1e-6 ||A||_F^2 -- an invariant subspace with the top-k energy is a top-k subspace -- and
         the oracle's sum_{j<=k} sigma_j^2 to 1e-6 ||A||_F^2, or, when the measured covariance error between the two
         sketches is given (long streams, where it exceeds 1e-7), to k times that error (Weyl's inequality);
      4. scores within score_tol of the oracle scoring the same rows on the GPU's exported basis, and the selection equal
         to the oracle's outside the band round its threshold. With sample = n (wide or long streams, where the oracle
         cannot project every row in a test) the oracle projects n sampled rows on that basis (zhat to 1e-5) and then
         runs its consensus / cosine / selection on the GPU's stored zhat, taken as rows of a k-column problem with
         the identity as basis.
    Returns a dict of the measured figures (also printed), including the gap to the oracle's own scores and the largest
    principal angle between the two bases."""
    from oracle import Oracle

    keep = w.keep if keep is None else keep
    Vg = s.basis().cpu().numpy().astype(np.float64)          # k x D
    Bg = s.sketch().cpu().numpy().astype(np.float64)         # 2 ell x D
    k = Vg.shape[0]
    ortho = float(np.abs(Vg @ Vg.T - np.eye(k)).max())
    BV = Bg @ Vg.T
    H = BV.T @ BV
    res = float(np.linalg.norm(Bg.T @ BV - Vg.T @ H, 2)) / fro
    energy_gap = float(abs(np.trace(H) - o.sig2[:k].sum())) / fro
    own = np.linalg.eigvalsh(Bg @ Bg.T)[::-1]
    energy_own = float(abs(np.trace(H) - own[:k].sum())) / fro
    del Bg
    al = s.scores().cpu().numpy()
    if sample is None:
        o2 = Oracle(w.ell, w.D, 1)
        o2.set_basis(Vg)
        for lo in range(0, G.shape[0], w.batch):
            o2.score(G[lo:lo + w.batch])
        zhat_err = float(np.abs(s.zhat().cpu().numpy() - o2.zhat).max())
    else:
        rows = np.sort(np.random.default_rng(G.shape[0] + k).choice(G.shape[0], size=min(sample, G.shape[0]), replace=False))
        o1 = Oracle(w.ell, w.D, 1)
        o1.set_basis(Vg)
        o1.score(np.ascontiguousarray(G[rows]))
        zg = s.zhat().cpu().numpy()
        zhat_err = float(np.abs(zg[rows] - o1.zhat).max())
        o2 = Oracle(2, k, 1)
        o2.set_basis(np.eye(k))
        o2.score(zg)                                          # unit rows (or zero rows): normalising changes <= 1e-7
    oidx = o2.select(keep)
    err_same = float(np.abs(al - o2.alpha).max())
    sin_max = float("nan")                                   # (a fixture does not hold the oracle's k x D basis)
    if getattr(o, "V", None) is not None:
        sv = np.linalg.svd(Vg @ o.V.T, compute_uv=False)
        sin_max = float(np.sqrt(max(0.0, 1.0 - sv.min() ** 2)))
    err_own = float(np.abs(al - o.alpha).max()) if o.alpha.shape == al.shape else float("nan")
    gap = float(o.sig2[k - 1] - o.sig2[k]) / fro
    out = dict(ortho=ortho, residual=res, energy_own=energy_own, energy_gap=energy_gap, zhat_err=zhat_err, err_same_basis=err_same,
               err_oracle_basis=err_own, sin_max=sin_max, spectral_gap=gap)
    print("end-to-end %s: %s" % (w.name, ", ".join("%s=%.3g" % kv for kv in out.items())), flush=True)
    assert ortho <= 1e-5, out
    assert res <= 1e-6, out
    assert energy_own <= 1e-6, out
    assert energy_gap <= (1e-6 if cov_err is None else max(1e-6, k * cov_err)), out
    assert zhat_err <= 1e-5, out
    assert err_same <= score_tol, out
    gidx = s.select(keep).cpu().numpy()
    gi, oi = set(gidx.tolist()), set(oidx.tolist())
    assert len(gi) == len(oi)
    if oi:
        tau = float(np.min(o2.alpha[list(oi)]))
        for i in gi ^ oi:
            assert abs(float(o2.alpha[i]) - tau) <= score_tol, (i, o2.alpha[i], tau)
    return out
