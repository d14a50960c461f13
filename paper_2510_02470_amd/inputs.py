"""Seeded synthetic gradient-row generators (inputs only; none of the method's arithmetic lives here).

The paper (arxiv 2510.02470, Experiments) feeds per-example gradients of a ResNet-18 on public image sets;
none of that data is used. The five workloads below stand in for it: low-rank signal + isotropic noise,
log-normal row norms, a fraction of sign-disturbed rows, at last-layer-gradient widths (512*C + C).

Row i:   g_i = c_i * ( f_i * sum_j a_ij s_j w_j  +  tau * nu_i )
  s_j   signal spectrum (scale * j^-power), j = 1..r
  a_i   row of U: exact orthonormal columns (QR) when ``u_orth`` else iid N(0, 1/N)
  w_j   column of W: orthonormal (QR) when ``w_orth`` else iid N(0, 1/D)
  nu_i  iid N(0, 1) noise; tau from ``tau`` or from the noise share eta of total energy:
        N*D*tau^2 = eta/(1-eta) * sum_j s_j^2
  c_i   exp(sigma_norm * xi_i), xi_i ~ N(0, 1)
  f_i   +1, or with probability flip_prob: -1 (``flip='neg'``) or a random sign (``flip='random'``)

Two back ends produce rows of the same recipe (not the same bytes): numpy on the host for the small and medium
workloads, torch on the device for the wide streamed ones. Parity tests always hand both sides the same bytes.
"""
from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    N: int
    D: int
    dtype: str          # "f32" | "bf16"
    ell: int
    k: int
    batch: int
    keep: float
    r: int
    s_scale: float
    s_power: float
    eta: float          # noise share of total energy (ignored when tau is given)
    tau: float          # < 0: derive from eta
    sigma_norm: float
    flip_prob: float
    flip: str           # "neg" | "random"
    u_orth: bool
    w_orth: bool
    seed: int = 0

    def scaled(self, **kw):
        """Same recipe at another size (used by tests)."""
        return replace(self, **kw)

    def spectrum(self):
        j = np.arange(1, self.r + 1, dtype=np.float64)
        return self.s_scale * j ** (-self.s_power)

    def noise_tau(self):
        if self.tau >= 0:
            return self.tau
        e = float(np.sum(self.spectrum() ** 2))
        return float(np.sqrt(self.eta / (1.0 - self.eta) * e / (self.N * self.D)))


WORKLOADS = {
    1: Workload("cfg1_tiny", 2048, 512, "f32", 32, 16, 256, 0.10, 16, 10.0, 1.0, 0.0, 0.01 / np.sqrt(512.0),
                0.5, 0.05, "neg", True, True),
    2: Workload("cfg2_last10", 50_000, 5_130, "f32", 64, 32, 1024, 0.05, 64, 1.0, 0.8, 0.05, -1.0,
                0.7, 0.10, "random", False, True),
    3: Workload("cfg3_last100", 50_000, 51_300, "f32", 128, 64, 2048, 0.10, 256, 1.0, 0.6, 0.10, -1.0,
                0.7, 0.20, "neg", False, True),
    4: Workload("cfg4_wide", 100_000, 1_048_576, "f32", 256, 128, 512, 0.10, 512, 1.0, 0.5, 0.20, -1.0,
                1.0, 0.0, "neg", False, False),
    5: Workload("cfg5_head", 1_000_000, 2_049_000, "bf16", 256, 128, 1024, 0.01, 1024, 1.0, 0.5, 0.30, -1.0,
                1.0, 0.15, "neg", False, False),
}


def f32_to_bf16_bits(x):
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(h):
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed, stream):
    return np.random.default_rng([int(seed), int(stream)])


def generate_numpy(w: Workload):
    """All N rows on the host. float32 array, or uint16 bf16 bit patterns when w.dtype == 'bf16'."""
    N, D, r = w.N, w.D, w.r
    s = w.spectrum()
    U = _rng(w.seed, 1).standard_normal((N, r))
    if w.u_orth:
        U, _ = np.linalg.qr(U)
    else:
        U /= np.sqrt(N)
    Wm = _rng(w.seed, 2).standard_normal((D, r))
    if w.w_orth:
        Wm, _ = np.linalg.qr(Wm)
    else:
        Wm /= np.sqrt(D)
    xi = _rng(w.seed, 4).standard_normal(N)
    c = np.exp(w.sigma_norm * xi)
    fr = _rng(w.seed, 5)
    hit = fr.random(N) < w.flip_prob
    if w.flip == "neg":
        f = np.where(hit, -1.0, 1.0)
    else:
        f = np.where(hit, np.where(fr.random(N) < 0.5, -1.0, 1.0), 1.0)
    tau = w.noise_tau()
    G = np.empty((N, D), dtype=np.float32)
    nr = _rng(w.seed, 3)
    step = max(1, (1 << 24) // max(D, 1))
    SW = (Wm * s[None, :]).T  # r x D
    for lo in range(0, N, step):
        hi = min(N, lo + step)
        blk = (U[lo:hi] * f[lo:hi, None]) @ SW
        blk += tau * nr.standard_normal((hi - lo, D))
        blk *= c[lo:hi, None]
        G[lo:hi] = blk.astype(np.float32)
    if w.dtype == "bf16":
        return f32_to_bf16_bits(G)
    return G


class DeviceStream:
    """Rows of a wide workload made batch by batch on the GPU with torch (input synthesis, never timed).

    Every batch is a pure function of (seed, batch index), so both passes see the same stream. W (r x D) is
    materialised once and reused.
    """

    def __init__(self, w: Workload, device="cuda", w_dtype=None):
        import torch

        self.torch = torch
        self.w = w
        self.device = torch.device(device)
        g = torch.Generator(device=self.device)
        g.manual_seed(w.seed * 1_000_003 + 2)
        wd = w_dtype or torch.float32
        self.SW = torch.empty((w.r, w.D), dtype=wd, device=self.device)
        s = torch.tensor(w.spectrum(), dtype=torch.float32, device=self.device)
        rows_per = max(1, (1 << 26) // w.D)
        for lo in range(0, w.r, rows_per):
            hi = min(w.r, lo + rows_per)
            blk = torch.randn((hi - lo, w.D), generator=g, device=self.device, dtype=torch.float32)
            blk *= (s[lo:hi] / np.sqrt(w.D))[:, None]
            self.SW[lo:hi] = blk.to(wd)
        self.tau = w.noise_tau()

    def n_batches(self):
        return (self.w.N + self.w.batch - 1) // self.w.batch

    def batch(self, b, rows=None, out=None):
        """Rows [b*batch, b*batch + rows) as a (rows x D) device tensor (float32 or bfloat16)."""
        torch, w = self.torch, self.w
        R = rows if rows is not None else min(w.batch, w.N - b * w.batch)
        g = torch.Generator(device=self.device)
        g.manual_seed((w.seed * 1_000_003 + 7) * 1_000_003 + b)
        A = torch.randn((R, w.r), generator=g, device=self.device, dtype=torch.float32) / np.sqrt(w.N)
        xi = torch.randn((R,), generator=g, device=self.device, dtype=torch.float32)
        c = torch.exp(w.sigma_norm * xi)
        hit = torch.rand((R,), generator=g, device=self.device) < w.flip_prob
        if w.flip == "neg":
            f = torch.where(hit, -1.0, 1.0)
        else:
            coin = torch.rand((R,), generator=g, device=self.device) < 0.5
            f = torch.where(hit & coin, -1.0, 1.0)
        G = torch.randn((R, w.D), generator=g, device=self.device, dtype=torch.float32)
        G *= self.tau
        G.addmm_((A * f[:, None]).to(self.SW.dtype), self.SW) if self.SW.dtype == torch.float32 else G.add_(
            ((A * f[:, None]).to(self.SW.dtype) @ self.SW).float())
        G *= c[:, None]
        if w.dtype == "bf16":
            G = G.to(torch.bfloat16)
        if out is not None:
            out[:R].copy_(G)
            return out[:R]
        return G


# ---- factored last-layer rows ------------------------------------------------------------------------------
# For a linear last layer under softmax cross-entropy the per-example gradient is (p_i - y_i) (x) [h_i; 1]. The
# generators below make the two factors of such rows (never the rows): features h_i = relu(class mean + noise) of a
# C-class mixture, logits from a fixed random classifier that partly knows the class means, a share of wrong labels.
# E = softmax(logits) - onehot(label) (rows x C), H = features (rows x dh), labels (rows, int32).

def _factor_params(C, dh, seed):
    rng = _rng(seed, 11)
    means = rng.standard_normal((C, dh)) * 0.7
    Wc = (means * 0.6 + rng.standard_normal((C, dh)) * 0.4) / np.sqrt(dh) * 4.0  # a half-trained classifier
    bc = rng.standard_normal(C) * 0.1
    return means, Wc, bc


def generate_factors_numpy(N, C, dh, dtype="f32", seed=0, wrong_labels=0.1):
    """(E, H, labels): float32 arrays, or uint16 bf16 bit patterns when dtype == 'bf16'; labels int32."""
    means, Wc, bc = _factor_params(C, dh, seed)
    rng = _rng(seed, 12)
    cls = rng.integers(0, C, size=N)
    Hm = np.maximum(means[cls] + rng.standard_normal((N, dh)), 0.0)
    logits = Hm @ Wc.T + bc
    logits -= logits.max(axis=1, keepdims=True)
    P = np.exp(logits)
    P /= P.sum(axis=1, keepdims=True)
    labels = np.where(rng.random(N) < wrong_labels, rng.integers(0, C, size=N), cls)
    E = P.copy()
    E[np.arange(N), labels] -= 1.0
    E = E.astype(np.float32)
    Hm = Hm.astype(np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(E), f32_to_bf16_bits(Hm), labels.astype(np.int32)
    return E, Hm, labels.astype(np.int32)


class DeviceFactors:
    """The same recipe batch by batch on the GPU with torch (input synthesis, never timed); a batch is a pure function
    of (seed, batch index)."""

    def __init__(self, C, dh, dtype="bf16", seed=0, wrong_labels=0.1, device="cuda"):
        import torch

        self.torch, self.C, self.dh, self.dtype, self.seed = torch, int(C), int(dh), dtype, int(seed)
        self.wrong = float(wrong_labels)
        self.device = torch.device(device)
        means, Wc, bc = _factor_params(self.C, self.dh, self.seed)
        self.means = torch.from_numpy(means.astype(np.float32)).to(self.device)
        self.Wc = torch.from_numpy(Wc.astype(np.float32)).to(self.device)
        self.bc = torch.from_numpy(bc.astype(np.float32)).to(self.device)

    def batch(self, b, rows):
        torch = self.torch
        g = torch.Generator(device=self.device)
        g.manual_seed((self.seed * 1_000_003 + 13) * 1_000_003 + int(b))
        cls = torch.randint(0, self.C, (rows,), generator=g, device=self.device)
        Hm = torch.relu(self.means[cls] + torch.randn((rows, self.dh), generator=g, device=self.device))
        P = torch.softmax(Hm @ self.Wc.T + self.bc, dim=1)
        wrong = torch.rand((rows,), generator=g, device=self.device) < self.wrong
        other = torch.randint(0, self.C, (rows,), generator=g, device=self.device)
        labels = torch.where(wrong, other, cls)
        E = P
        E[torch.arange(rows, device=self.device), labels] -= 1.0
        td = torch.bfloat16 if self.dtype == "bf16" else torch.float32
        return E.to(td).contiguous(), Hm.to(td).contiguous(), labels.to(torch.int32)
