"""Synthetic feature trajectories F_t in R^{N x D} for one cached DiT block.

The paper measures on real FLUX.1-dev / HunyuanVideo hidden states (Sec. 4,
DrawBench / VBench prompts).  Those are not available, so the tests and the
benchmark use stand-ins that keep only what the paper says about such
features (Sec. 1, Fig. 1a): a smooth, high-energy low-rank principal part and
a low-energy residual that oscillates from step to step.

    F_t = U diag(s * a(t)) V^T + E_t

  * U (N x m), V (D x m): random matrices with orthonormal columns,
  * s_i = c * i^(-gamma): power-law spectrum; c makes the mean-square entry
    of the signal (1 - rho),
  * a_i(t) = 1 + 0.3 cos(2 pi f_i t / T + phi_i), f_i ~ U[0.5, 1.5]: smooth
    per-direction drift,
  * E_t: residual.  "iid": noise_sigma * N(0,1) redrawn every step.
    "alternating": (-1)^t E_0 + 0.1 * fresh_t, rescaled to carry a fraction
    rho of the total energy (a sign-flipping, hard-to-forecast residual).

Everything is drawn from torch generators seeded from (config, block, t), so
``at(t)`` is random-access and reproducible on a given device.  CPU and GPU
generators give different draws; a test therefore generates once and hands the
same bytes to both sides.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    config_id: int
    B: int            # blocks batched into one launch
    N: int            # tokens (rows of F)
    D: int            # hidden size (columns of F)
    k: int            # rank of the principal subspace
    dtype: str        # storage type of F / R / Fhat: "f32" or "bf16"
    T: int            # timesteps in a trajectory
    interval: int     # a full-compute step every `interval` steps
    alpha: float      # EMA weight on the NEW coefficients (= 1 - beta of Eq. 11)
    gamma: float      # spectrum exponent
    signal_rank: int  # m
    rho: float        # residual energy fraction ("alternating" residual)
    noise_sigma: float  # std of the i.i.d. residual ("iid" residual)
    residual: str     # "iid" | "alternating"

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4


# The five configurations the benchmark description names.
WORKLOADS = {
    # 2 blocks, 256 x 64, k = 8, fp32, 10 steps, every 3rd full.
    "tiny": Workload("tiny", 1, 2, 256, 64, 8, "f32", 10, 3, 0.5, 1.5, 64, 0.0, 0.02, "iid"),
    # FLUX-shaped single block (4096 image + 512 text tokens).
    "flux1": Workload("flux1", 2, 1, 4608, 3072, 32, "bf16", 50, 5, 0.5, 1.2, 256, 0.05, 0.0, "alternating"),
    # FLUX-shaped whole model: 19 double-stream + 38 single-stream blocks.
    "flux57": Workload("flux57", 3, 57, 4608, 3072, 32, "bf16", 50, 6, 0.5, 1.2, 256, 0.05, 0.0, "alternating"),
    # HunyuanVideo-shaped 720p x 129 frames: 33*45*80 latent + 256 text tokens.
    "hyv60": Workload("hyv60", 4, 60, 33 * 45 * 80 + 256, 3072, 64, "bf16", 50, 6, 0.5, 1.0, 256, 0.08, 0.0, "alternating"),
    # Rank / precision sweep: 4 prompts stacked along N with one shared basis.
    "sweep": Workload("sweep", 5, 1, 4 * 4608, 3072, 32, "bf16", 50, 5, 0.5, 1.2, 256, 0.05, 0.0, "alternating"),
}


def is_full_step(t: int, interval: int) -> bool:
    """Schedule used by every test and by the benchmark: step t is a
    full-compute step iff t mod interval == 0 (so t = 0 always is)."""
    return t % interval == 0


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def _seed(config_id: int, block: int, t: int = -1) -> int:
    return 0x5DC0000 + config_id * 1_000_003 + block * 1009 + (t + 1) * 7_919_111


def _orthonormal(n: int, m: int, gen: torch.Generator, device, work) -> torch.Tensor:
    g = torch.randn(n, m, generator=gen, device=device, dtype=work)
    q, _ = torch.linalg.qr(g, mode="reduced")
    return q


class FeatureStream:
    """Feature trajectory of one block of one workload.

    ``work`` is the dtype the generator computes in (float64 on the CPU for
    small cases, float32 on the GPU for the full-size ones); the returned F_t
    is rounded once to the workload's storage dtype.
    """

    def __init__(self, wl: Workload, block: int = 0, device="cpu", work: torch.dtype | None = None,
                 N: int | None = None):
        self.wl = wl
        self.block = block
        self.device = torch.device(device)
        self.work = work if work is not None else (torch.float64 if self.device.type == "cpu" else torch.float32)
        self.N = wl.N if N is None else N
        m = min(wl.signal_rank, wl.D, self.N)
        self.m = m
        gen = torch.Generator(device=self.device)
        gen.manual_seed(_seed(wl.config_id, block))
        self.U = _orthonormal(self.N, m, gen, self.device, self.work)
        self.V = _orthonormal(wl.D, m, gen, self.device, self.work)
        i = torch.arange(1, m + 1, device=self.device, dtype=self.work)
        s = i.pow(-wl.gamma)
        # unit mean-square signal (times 1 - rho): sum s_i^2 = N D (1 - rho)
        s = s * math.sqrt(self.N * wl.D * (1.0 - wl.rho)) / s.norm()
        self.s = s
        self.f = 0.5 + torch.rand(m, generator=gen, device=self.device, dtype=self.work)
        self.phi = 2.0 * math.pi * torch.rand(m, generator=gen, device=self.device, dtype=self.work)
        self.E0 = None
        if wl.residual == "alternating":
            self.E0 = torch.randn(self.N, wl.D, generator=gen, device=self.device, dtype=self.work)

    def coeff_scale(self, t: int) -> torch.Tensor:
        """a_i(t): the smooth multiplicative drift of direction i."""
        wl = self.wl
        return 1.0 + 0.3 * torch.cos(2.0 * math.pi * self.f * (t / wl.T) + self.phi)

    def signal(self, t: int) -> torch.Tensor:
        """Noise-free part U diag(s a(t)) V^T in the working dtype."""
        return (self.U * (self.s * self.coeff_scale(t))) @ self.V.T

    def residual(self, t: int, signal_energy: float) -> torch.Tensor:
        wl = self.wl
        gen = torch.Generator(device=self.device)
        gen.manual_seed(_seed(wl.config_id, self.block, t))
        fresh = torch.randn(self.N, wl.D, generator=gen, device=self.device, dtype=self.work)
        if wl.residual == "iid":
            return wl.noise_sigma * fresh
        e = (1.0 if t % 2 == 0 else -1.0) * self.E0 + 0.1 * fresh
        target = wl.rho / (1.0 - wl.rho) * signal_energy
        return e * math.sqrt(target) / e.norm()

    def at(self, t: int, noise: bool = True) -> torch.Tensor:
        """F_t rounded to the storage dtype, shape [N, D]."""
        sig = self.signal(t)
        if noise:
            energy = float(((self.s * self.coeff_scale(t)) ** 2).sum())
            sig = sig + self.residual(t, energy)
        return sig.to(torch_dtype(self.wl.dtype))
