"""Seeded synthetic inputs for the sketched-AMSGrad step.

This module is the only code shared by the HIP path's tests/benchmark and the CPU
oracle's tests.  It holds none of the method's arithmetic: it only draws random
gradients, initial parameters and hash parameters, with the shapes and value
distributions of the five workloads (flat parameter vectors of ResNet/GPT-2 size
split into layer segments of very different scale, light- and heavy-tailed
per-worker noise, a small set of heavy coordinates shared by all workers).  These
stand in for the gradient streams of the paper's ResNet-50/CIFAR and LeNet-5/MNIST
runs (Sec. V), which need datasets and a training stack that are not available.

Everything is generated with torch on the requested device from an explicit seed,
so the same call on the same device type gives the same bits; parity tests always
hand the *same tensor* (downloaded) to both sides.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np
import torch

P31 = 2147483647  # 2^31 - 1, modulus of the hash family


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    d: int
    n: int
    r: int
    c: int
    k: int
    steps: int
    noise: str = "normal"        # "normal" | "laplace" | "student3"
    nseg: int = 1                # layer segments with sizes ~ 10^U(0,3)
    lo: float = -3.0             # per-segment std = 10^U(lo, hi)
    hi: float = -3.0
    heavy_frac: float = 0.0      # fraction of coordinates that are heavy (shared by all workers)
    heavy_count: int = 0         # or an absolute count
    heavy: str = "none"          # "uniform": U(a,b)*scale ; "pareto": Pareto(alpha)*sigma
    heavy_a: float = 0.5
    heavy_b: float = 1.5
    heavy_scale: float = 1.0     # for "uniform": multiplies sigma unless heavy_abs
    heavy_abs: bool = False      # magnitude independent of the segment's sigma
    heavy_alpha: float = 1.5
    beta1: float = 0.9
    beta2: float = 0.99
    eps: float = 1e-8            # v_0 = vhat_0
    lr: float = 1e-3
    seed: int = 0

    def scaled(self, d: int, c: int | None = None, k: int | None = None, n: int | None = None,
               name: str | None = None) -> "Workload":
        """Same recipe at a smaller size (d/c and k/d kept unless given)."""
        f = d / self.d
        c2 = c if c is not None else max(16, int(round(self.c * f)))
        k2 = k if k is not None else max(1, int(round(self.k * f)))
        hc = max(1, int(round(self.heavy_count * f))) if self.heavy_count else 0
        return dataclasses.replace(self, d=d, c=c2, k=k2, n=n or self.n, heavy_count=hc,
                                   nseg=max(1, min(self.nseg, d // 64)),
                                   name=name or f"{self.name}@d={d}")


WORKLOADS = {
    "C1": Workload("C1-tiny", d=65_536, n=4, r=5, c=2_048, k=256, steps=10, noise="normal",
                   lo=-3.0, hi=-3.0, heavy="uniform", heavy_count=256, heavy_abs=True),
    "C2": Workload("C2-resnet18", d=11_200_000, n=8, r=5, c=262_144, k=50_000, steps=20,
                   noise="laplace", nseg=60, lo=-4.0, hi=-1.0),
    "C3": Workload("C3-resnet50", d=25_600_000, n=16, r=7, c=1_048_576, k=100_000, steps=20,
                   noise="student3", nseg=100, lo=-5.0, hi=-1.0, heavy="uniform", heavy_frac=0.005,
                   heavy_scale=10.0),
    "C4": Workload("C4-gpt2small", d=124_000_000, n=8, r=5, c=4_194_304, k=1_240_000, steps=10,
                   noise="normal", nseg=150, lo=-5.0, hi=-2.0, heavy="pareto", heavy_frac=0.01,
                   heavy_alpha=1.5),
    "C5": Workload("C5-stress", d=1_300_000_000, n=4, r=5, c=16_777_216, k=1_300_000, steps=3,
                   noise="normal", nseg=1, lo=-3.0, hi=-3.0, heavy="pareto", heavy_frac=0.001,
                   heavy_alpha=1.2),
    # The sketch shapes of the paper's own experiments (Sec. V): ResNet-50 (roughly 25M parameters, 16 workers,
    # 10 rows x 100,000 columns, k = 50,000) and LeNet-5 (roughly 60k parameters, 50 and 100 workers, 5 rows x
    # 400 columns, k = 500).  Even row count, column counts that are not powers of two.  The gradient recipe is
    # synthetic as above (the paper's come from CIFAR / MNIST training).
    "P1": Workload("P1-paper-resnet50", d=25_000_000, n=16, r=10, c=100_000, k=50_000, steps=5,
                   noise="student3", nseg=100, lo=-5.0, hi=-1.0, heavy="uniform", heavy_frac=0.005,
                   heavy_scale=10.0),
    "P2a": Workload("P2-paper-lenet5-n50", d=60_000, n=50, r=5, c=400, k=500, steps=10, noise="normal",
                    nseg=8, lo=-3.0, hi=-1.0, heavy="uniform", heavy_count=100, heavy_abs=True),
    "P2b": Workload("P2-paper-lenet5-n100", d=60_000, n=100, r=5, c=400, k=500, steps=10, noise="normal",
                    nseg=8, lo=-3.0, hi=-1.0, heavy="uniform", heavy_count=100, heavy_abs=True),
}


def hash_params(r: int, seed: int = 0) -> np.ndarray:
    """[r][4] uint32 = (a_h, b_h, a_s, b_s) per row; a in [1, p-1], b in [0, p-1]."""
    rng = np.random.default_rng(seed + 0x5A15)
    hp = np.empty((r, 4), dtype=np.uint32)
    hp[:, 0] = rng.integers(1, P31, size=r)
    hp[:, 1] = rng.integers(0, P31, size=r)
    hp[:, 2] = rng.integers(1, P31, size=r)
    hp[:, 3] = rng.integers(0, P31, size=r)
    return hp


def identity_hash_params(r: int, seed: int = 0) -> np.ndarray:
    """Bucket hash h_j(l) = l (a=1, b=0: collision-free when c >= d); random sign hashes."""
    hp = hash_params(r, seed)
    hp[:, 0] = 1
    hp[:, 1] = 0
    return hp


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


class GradientStream:
    """Per-step, per-worker synthetic gradients for one workload.

    ``sigma`` ([d]) is the per-coordinate noise scale (constant inside a segment);
    the heavy set (indices, signed magnitudes) is drawn once and added to every
    worker's gradient at every step; the noise is redrawn for each (step, worker).
    """

    def __init__(self, w: Workload, device="cpu", seed: int | None = None):
        self.w = w
        self.device = torch.device(device)
        self.seed = w.seed if seed is None else seed
        rng = np.random.default_rng(self.seed + 0x9E37)
        d = w.d
        # segment sizes ~ 10^U(0,3), rescaled to sum to d; per-segment std 10^U(lo,hi)
        raw = 10.0 ** rng.uniform(0.0, 3.0, size=w.nseg)
        sizes = np.maximum(1, np.floor(raw / raw.sum() * d).astype(np.int64))
        sizes[-1] += d - sizes.sum()
        if sizes[-1] < 1:  # only for tiny d: fall back to equal segments
            sizes = np.full(w.nseg, d // w.nseg, dtype=np.int64)
            sizes[-1] += d - sizes.sum()
        self.seg_sizes = sizes
        self.seg_sigma = (10.0 ** rng.uniform(w.lo, w.hi, size=w.nseg)).astype(np.float32)
        sig = torch.from_numpy(self.seg_sigma).to(self.device)
        self.sigma = torch.repeat_interleave(sig, torch.from_numpy(sizes).to(self.device))
        assert self.sigma.numel() == d
        # heavy coordinates, shared by all workers and steps
        nh = w.heavy_count if w.heavy_count else int(round(w.heavy_frac * d))
        self.heavy_idx = None
        if w.heavy != "none" and nh > 0:
            hidx = np.sort(rng.choice(d, size=nh, replace=False)) if d < (1 << 26) else \
                np.unique(rng.integers(0, d, size=nh))
            sgn = rng.integers(0, 2, size=hidx.size) * 2.0 - 1.0
            if w.heavy == "uniform":
                mag = rng.uniform(w.heavy_a, w.heavy_b, size=hidx.size) * w.heavy_scale
            else:  # pareto, x_m = 1
                mag = (1.0 - rng.uniform(0.0, 1.0, size=hidx.size)) ** (-1.0 / w.heavy_alpha)
            self.heavy_idx = torch.from_numpy(hidx.astype(np.int64)).to(self.device)
            hv = torch.from_numpy((sgn * mag).astype(np.float32)).to(self.device)
            if not w.heavy_abs:
                hv = hv * self.sigma[self.heavy_idx]
            self.heavy_val = hv

    def _noise(self, gen: torch.Generator, numel: int) -> torch.Tensor:
        w, dev = self.w, self.device
        if w.noise == "normal":
            return torch.randn(numel, generator=gen, device=dev, dtype=torch.float32)
        if w.noise == "laplace":  # std 1: scale b = 1/sqrt(2)
            uu = torch.rand(numel, generator=gen, device=dev, dtype=torch.float32) - 0.5
            return -(1.0 / math.sqrt(2.0)) * torch.sign(uu) * torch.log1p(-2.0 * uu.abs()).clamp_(min=-80.0)
        if w.noise == "student3":  # z / sqrt(chi2_3 / 3)
            z = torch.randn(numel, generator=gen, device=dev, dtype=torch.float32)
            q = torch.zeros(numel, device=dev, dtype=torch.float32)
            for _ in range(3):
                t = torch.randn(numel, generator=gen, device=dev, dtype=torch.float32)
                q.addcmul_(t, t)
            return z / torch.sqrt(q / 3.0).clamp_(min=1e-6)
        raise ValueError(w.noise)

    def worker(self, step: int, i: int, out: torch.Tensor | None = None) -> torch.Tensor:
        """Gradient of worker ``i`` at step ``step`` ([d], float32)."""
        gen = _gen(self.device, (self.seed * 1_000_003 + step) * 4099 + i + 17)
        g = self._noise(gen, self.w.d).mul_(self.sigma)
        if self.heavy_idx is not None:
            g.index_add_(0, self.heavy_idx, self.heavy_val)
        if out is not None:
            out.copy_(g)
            return out
        return g

    def step(self, step: int, out: torch.Tensor | None = None) -> torch.Tensor:
        """All workers' gradients at ``step``: [n][d] float32 on the stream's device."""
        w = self.w
        if out is None:
            out = torch.empty((w.n, w.d), device=self.device, dtype=torch.float32)
        for i in range(w.n):
            self.worker(step, i, out=out[i])
        return out

    def x1(self) -> torch.Tensor:
        """Initial parameters x_1 ~ N(0, 0.02^2)."""
        gen = _gen(self.device, self.seed * 7919 + 5)
        return torch.randn(self.w.d, generator=gen, device=self.device, dtype=torch.float32) * 0.02


def integer_vectors(n: int, d: int, amax: int = 64, seed: int = 0, device="cpu") -> torch.Tensor:
    """[n][d] float32 with small integer values (every partial sum stays exact in fp32)."""
    gen = _gen(device, seed + 31)
    return torch.randint(-amax, amax + 1, (n, d), generator=gen, device=device).to(torch.float32)
