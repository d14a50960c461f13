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


def run_gpu(w, G, k=None, keep=None, score=True):
    import torch
    from paper_2510_02470_amd.binding import Sage

    s = Sage(w.ell, w.D, dtype=w.dtype)
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
