"""Seeded synthetic workloads shared by the GPU path, the oracle's tests and bench.py.

This module only *describes* inputs: sizes, hyper-parameters, the diagonal of
the quadratic loss, its optimum, the initial model and the order in which
workers arrive.  It contains none of the method's arithmetic (no update rule,
no gradient, no noise generator) and imports neither the GPU binding nor the
oracle, so both sides can be fed the same bits from here.

The sizes stand in for the models of the paper's experiments (Section 6:
ResNet-20 on CIFAR-10 with M = 4 and 8, ResNet-50 on ImageNet with M = 16);
lambda_0 = 0.04 (constant), lambda_0 = 2 with m = 0.95 (adaptive) and
eps = 1e-7 are the values Section 6 reports.  The loss itself is synthetic:
0.5 * sum_i h_i (w_i - wstar_i)^2.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

MODE_C = 0   # DC-ASGD-c: lambda_t = lambda_0
MODE_A = 1   # DC-ASGD-a: lambda_t = lambda_0 / sqrt(MeanSquare(t) + eps)

_CHUNK = 1 << 24


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    d: int                 # number of parameters
    M: int                 # number of workers
    T: int                 # number of pushes
    mode: int              # MODE_C or MODE_A
    eta: float
    lambda0: float
    ema_m: float           # the constant m of Eq. 18 (unused in MODE_C)
    eps: float
    h_lo: float            # h_i log-uniform in [h_lo, h_hi]
    h_hi: float
    wstar_sigma: float     # wstar_i ~ N(0, wstar_sigma^2)
    sigma: float           # gradient-noise standard deviation
    order: str             # "round_robin" | "iid" | "queues"
    K: int = 1             # queue length for push_batch ("queues" only)
    grad_bf16: bool = False
    seed: int = 0

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)

    # ---- inputs -----------------------------------------------------------
    def _rng(self, stream: int) -> np.random.Generator:
        return np.random.Generator(np.random.Philox(key=[self.seed, stream]))

    def hdiag(self) -> np.ndarray:
        """Diagonal of the quadratic loss, log-uniform, float32[d]."""
        rng = self._rng(1)
        lo, hi = math.log(self.h_lo), math.log(self.h_hi)
        out = np.empty(self.d, dtype=np.float32)
        for a in range(0, self.d, _CHUNK):
            b = min(self.d, a + _CHUNK)
            out[a:b] = np.exp(lo + rng.random(b - a) * (hi - lo)).astype(np.float32)
        return out

    def wstar(self) -> np.ndarray:
        """Optimum of the quadratic loss, float32[d]."""
        rng = self._rng(2)
        out = np.empty(self.d, dtype=np.float32)
        for a in range(0, self.d, _CHUNK):
            b = min(self.d, a + _CHUNK)
            out[a:b] = (self.wstar_sigma * rng.standard_normal(b - a)).astype(np.float32)
        return out

    def w0(self) -> np.ndarray:
        return np.zeros(self.d, dtype=np.float32)

    def arrivals(self) -> np.ndarray:
        """Worker id of every push, int32[T].

        round_robin: t mod M (constant delay M-1).
        iid:         independent uniform draws (delays vary).
        queues:      consecutive blocks of K holding K distinct workers each
                     (a worker has one gradient in flight, Algorithm 1), every
                     block a fresh random choice and order.
        """
        if self.order in ("round_robin", "sync"):
            return (np.arange(self.T) % self.M).astype(np.int32)
        rng = self._rng(3)
        if self.order == "iid":
            return rng.integers(0, self.M, size=self.T).astype(np.int32)
        if self.order == "queues":
            assert 1 <= self.K <= self.M and self.T % self.K == 0
            blocks = [rng.permutation(self.M)[: self.K] for _ in range(self.T // self.K)]
            return np.concatenate(blocks).astype(np.int32)
        raise ValueError(self.order)

    def sample_indices(self, count: int, edge: int = 1024) -> np.ndarray:
        """Sorted element indices for spot checks at full size: both ends of
        the vector (first/last tiles and the ragged tail) plus a seeded
        uniform sample of the interior."""
        if self.d <= count + 2 * edge:
            return np.arange(self.d, dtype=np.uint64)
        rng = self._rng(4)
        mid = rng.integers(edge, self.d - edge, size=count)
        idx = np.concatenate([np.arange(edge), mid, np.arange(self.d - edge, self.d)])
        return np.unique(idx).astype(np.uint64)


_BASE_SEED = 160908326

CONFIGS = (
    Workload("cfg0_resnet20_M4_c", d=272_474, M=4, T=2000, mode=MODE_C, eta=0.1,
             lambda0=0.04, ema_m=0.0, eps=0.0, h_lo=1e-3, h_hi=1.0, wstar_sigma=1.0,
             sigma=0.01, order="round_robin", seed=_BASE_SEED + 0),
    Workload("cfg1_resnet20_M8_a", d=272_474, M=8, T=4000, mode=MODE_A, eta=0.1,
             lambda0=2.0, ema_m=0.95, eps=1e-7, h_lo=1e-3, h_hi=1.0, wstar_sigma=1.0,
             sigma=0.01, order="iid", seed=_BASE_SEED + 1),
    Workload("cfg2_resnet50_M16_a", d=25_557_032, M=16, T=200, mode=MODE_A, eta=0.05,
             lambda0=2.0, ema_m=0.95, eps=1e-7, h_lo=1e-4, h_hi=1.0, wstar_sigma=0.05,
             sigma=0.001, order="iid", seed=_BASE_SEED + 2),
    Workload("cfg3_resnet50_M16_a_K16", d=25_557_032, M=16, T=320, mode=MODE_A, eta=0.05,
             lambda0=2.0, ema_m=0.95, eps=1e-7, h_lo=1e-4, h_hi=1.0, wstar_sigma=0.05,
             sigma=0.001, order="queues", K=16, seed=_BASE_SEED + 3),
    Workload("cfg4_vgg16_M32_a_bf16", d=138_357_544, M=32, T=64, mode=MODE_A, eta=0.02,
             lambda0=2.0, ema_m=0.95, eps=1e-7, h_lo=1e-4, h_hi=1.0, wstar_sigma=0.05,
             sigma=0.001, order="iid", grad_bf16=True, seed=_BASE_SEED + 4),
)


# Beyond the five asynchronous configurations: the supplement's synchronous
# variant, 16 same-snapshot gradients folded per step (eta_hat = K * eta).
EXTRA = (
    Workload("fold_resnet50_J16_a", d=25_557_032, M=1, T=320, mode=MODE_A, eta=0.05,
             lambda0=2.0, ema_m=0.95, eps=1e-7, h_lo=1e-4, h_hi=1.0, wstar_sigma=0.05,
             sigma=0.001, order="sync", K=16, seed=_BASE_SEED + 5),
)


def get(name_or_index) -> Workload:
    if isinstance(name_or_index, int):
        return CONFIGS[name_or_index]
    for wl in CONFIGS + EXTRA:
        if wl.name == name_or_index or wl.name.startswith(str(name_or_index)):
            return wl
    raise KeyError(name_or_index)
