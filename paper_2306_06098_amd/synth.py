"""Seeded synthetic gradient streams shared by the oracle tests, the GPU parity
tests and the benchmark.  This module holds input generation only: none of
the method's arithmetic (no error feedback, no Top-k, no scalar products).

The streams stand in for the gradient sequences of the models whose sizes the
workloads borrow (d = 272,474 / 11.2M / 110M / 340M); no dataset or trained
weight is involved.

Recipe (one stream = one ``GradientStream``):
  s_j   = exp(n_j), n_j ~ N(0,1)            fixed per coordinate (heavy tail)
  z_1   = eps_1;  z_t = rho * z_{t-1} + eps_t,  eps ~ N(0,1) i.i.d.
  g_t   = float32(s_j * z_t[j])
so consecutive gradients are strongly correlated and a small set of
coordinates carries most of the energy, as with real gradients.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    d: int
    m: int
    k: int
    lam: float
    T: int
    rho: float
    seed: int


# The five workloads of the benchmark definition.
WORKLOADS = {
    "tiny": Workload("tiny", 65_536, 32, 655, 1e-4, 200, 0.9, 0),
    "resnet20": Workload("resnet20", 272_474, 1024, 2_725, 1e-5, 500, 0.9, 1),
    "resnet18": Workload("resnet18", 11_200_000, 1024, 112_000, 1e-5, 300, 0.8, 2),
    "bert_base": Workload("bert_base", 110_000_000, 1024, 1_100_000, 1e-6, 100, 0.9, 3),
    "bert_large": Workload("bert_large", 340_000_000, 1024, 3_400_000, 1e-6, 50, 0.9, 4),
}


class GradientStream:
    """CPU (numpy, Philox counter-based) stream; the same float32 bytes are
    handed to the oracle and copied to the GPU."""

    def __init__(self, d: int, rho: float, seed: int):
        self.d, self.rho = int(d), np.float32(rho)
        self._rng = np.random.Generator(np.random.Philox(key=int(seed)))
        self.scale = np.exp(self._rng.standard_normal(self.d, dtype=np.float32))
        self._z = None

    def next(self) -> np.ndarray:
        eps = self._rng.standard_normal(self.d, dtype=np.float32)
        if self._z is None:
            self._z = eps
        else:
            self._z = self.rho * self._z + eps
        return (self.scale * self._z).astype(np.float32)


class TorchGradientStream:
    """Same recipe generated on a torch device (used by the benchmark to fill
    a 1024-row window at d = 110M quickly).  Its bits differ from the numpy
    stream; it is never compared against the oracle bit for bit."""

    def __init__(self, d: int, rho: float, seed: int, device):
        import torch
        self._torch = torch
        self.d, self.rho = int(d), float(rho)
        self._gen = torch.Generator(device=device)
        self._gen.manual_seed(int(seed))
        self.device = device
        self.scale = torch.randn(self.d, generator=self._gen, device=device,
                                 dtype=torch.float32).exp_()
        self._z = None

    def next_into(self, out) -> None:
        """Write g_t into the preallocated float32 tensor ``out``."""
        torch = self._torch
        if self._z is None:
            self._z = torch.randn(self.d, generator=self._gen, device=self.device,
                                  dtype=torch.float32)
        else:
            self._z.mul_(self.rho)
            out.normal_(generator=self._gen)
            self._z.add_(out)
        torch.mul(self.scale, self._z, out=out)


def integer_stream(d: int, seed: int, lo: int = -8, hi: int = 8):
    """Generator of small-integer-valued float32 gradients: every float32 sum
    is exact and magnitudes collide constantly, so the tie rule of the
    selection is exercised at the threshold on every step."""
    rng = np.random.Generator(np.random.Philox(key=int(seed)))
    while True:
        yield rng.integers(lo, hi + 1, size=d).astype(np.float32)


def random_sparse_row(d: int, k: int, rng: np.random.Generator):
    """k distinct ascending indices in [0, d) and N(0,1) float32 values (used
    to preload a window when only timing matters)."""
    if k * 4 < d:
        idx = np.unique(rng.integers(0, d, size=int(k * 1.2) + 16))
        while idx.size < k:
            idx = np.unique(np.concatenate([idx, rng.integers(0, d, size=k)]))
        idx = np.sort(rng.choice(idx, size=k, replace=False))
    else:
        idx = np.sort(rng.choice(d, size=k, replace=False))
    val = rng.standard_normal(k, dtype=np.float32)
    return idx.astype(np.int32), val
