"""Seeded synthetic model-update vectors and workload descriptions.

This module serves both the CPU oracle's tests and the GPU library's tests and
benchmark.  It holds no arithmetic of the compression method: it only draws
update vectors and names, per workload, the planner inputs (number of groups,
code lengths, fractions or bit budget).  Plans themselves are computed by
whichever side is under test.

The vectors stand in for the CNN updates the paper trains on CIFAR-10/100 and
FEMNIST (Sec. V), which are not available here; their skewed magnitude
distribution (Sec. IV-A, Fig. 1) is imitated by heavy-tailed and
layer-structured draws.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Sequence

import numpy as np

# ResNet-18 (CIFAR-style) parameter layout: 20 convolutions and 20 (scale, shift)
# pairs in network order; the last block is enlarged to stand in for the
# classifier so that the total is 11 200 000.
_RESNET18_BLOCKS = (
    [1728, 64, 64]
    + [36864, 64, 64, 36864, 64, 64] * 2
    + [73728, 128, 128, 147456, 128, 128, 8192, 128, 128]
    + [147456, 128, 128, 147456, 128, 128]
    + [294912, 256, 256, 589824, 256, 256, 32768, 256, 256]
    + [589824, 256, 256, 589824, 256, 256]
    + [1179648, 512, 512, 2359296, 512, 512, 131072, 512, 512]
    + [2359296, 512, 512, 2359296, 512, 31680]
)
assert len(_RESNET18_BLOCKS) == 60 and sum(_RESNET18_BLOCKS) == 11_200_000


@dataclass(frozen=True)
class Workload:
    """One benchmark/parity configuration (planner inputs only)."""

    cfg: int                      # 1-based configuration number
    name: str
    n_clients: int
    d: int
    n_coded: int                  # R: coded groups; the 0-bit tail is implicit
    mode: str                     # "fractions" | "budget" | "alg1"
    code_len: Optional[Sequence[int]] = None     # y_r for modes fractions/budget
    fractions: Optional[Sequence[float]] = None  # share of d per coded group
    bits_per_coord: Optional[float] = None       # budget for modes budget/alg1
    quant_seed: int = field(default=0)

    def budget_bits(self, client: int = 0) -> int:
        """Communication budget of one client in bits."""
        if self.cfg == 5:  # per-client budget, uniform in [0.25, 2] bit/coord
            rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([2402, 3770, 5, client, 99])))
            return int(self.d * rng.uniform(0.25, 2.0))
        if self.bits_per_coord is None:  # plan fixed by fractions: no budget
            return 0
        return int(self.d * self.bits_per_coord)


WORKLOADS = {
    1: Workload(1, "laplace-65k", 1, 65_536, 3, "fractions", code_len=(8, 4, 2),
                fractions=(0.10, 0.15, 0.25), quant_seed=2402037701),
    2: Workload(2, "gauss-1.2M-x8", 8, 1_200_000, 7, "alg1", bits_per_coord=1.5,
                quant_seed=2402037702),
    3: Workload(3, "resnet18-t3-x32", 32, 11_200_000, 15, "alg1", bits_per_coord=1.0,
                quant_seed=2402037703),
    4: Workload(4, "sparse-mix-x32", 32, 11_200_000, 7, "budget", code_len=(16, 8, 6, 4, 3, 2, 1),
                bits_per_coord=0.5, quant_seed=2402037704),
    5: Workload(5, "resnet50-mixed-x100", 100, 25_600_000, 31, "alg1", quant_seed=2402037705),
}


def _rng(cfg: int, client: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([2402, 3770, cfg, client])))


def update_vector(cfg: int, client: int, d: Optional[int] = None) -> np.ndarray:
    """The fp32 update vector of one client of configuration `cfg`.

    `d` overrides the configuration's length (for reduced-size parity cases);
    for the layer-structured configuration the block list is scaled with it.
    """
    w = WORKLOADS[cfg]
    d = w.d if d is None else int(d)
    rng = _rng(cfg, client)
    if cfg == 1:
        x = rng.laplace(0.0, 1e-3, size=d)
    elif cfg == 2:
        sigma = 10.0 ** rng.uniform(-4.0, -2.0)
        x = rng.normal(0.0, sigma, size=d)
    elif cfg == 3:
        sizes = np.asarray(_RESNET18_BLOCKS, dtype=np.float64)
        edges = np.floor(np.cumsum(sizes) * (d / sizes.sum())).astype(np.int64)
        edges[-1] = d
        factor = 10.0 ** rng.uniform(-5.0, -2.0, size=len(sizes))
        x = rng.standard_t(3.0, size=d)
        start = 0
        for e, f in zip(edges, factor):
            x[start:e] *= f
            start = int(e)
    elif cfg == 4:
        big = rng.random(d) < 0.05
        x = rng.normal(0.0, 1.0, size=d)
        x *= np.where(big, 1e-1, 1e-3)  # variances 1e-2 and 1e-6
    elif cfg == 5:
        if rng.random() < 0.5:
            x = rng.laplace(0.0, 1e-3, size=d)
        else:
            x = rng.normal(0.0, 1e-3, size=d)
    else:
        raise ValueError(f"unknown configuration {cfg}")
    return np.ascontiguousarray(x, dtype=np.float32)


def tie_heavy_vector(kind: str, d: int, seed: int = 0) -> np.ndarray:
    """Crafted vectors whose magnitudes collide, to exercise the tie rule."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([2402, 3770, 77, seed])))
    if kind == "all_equal":
        x = np.full(d, 0.5, dtype=np.float32)
    elif kind == "all_equal_mixed_sign":
        x = np.full(d, 0.5, dtype=np.float32) * rng.choice(np.array([-1.0, 1.0], dtype=np.float32), size=d)
    elif kind == "two_valued":
        x = rng.choice(np.array([0.25, -1.0], dtype=np.float32), size=d)
    elif kind == "few_levels":
        x = rng.integers(-4, 5, size=d).astype(np.float32) * np.float32(0.125)
    elif kind == "zeros_and_denormals":
        x = np.zeros(d, dtype=np.float32)
        x[::3] = np.float32(-0.0)
        den = rng.integers(1, 200, size=d).astype(np.uint32)
        mask = rng.random(d) < 0.3
        x = np.where(mask, den.view(np.float32) * rng.choice(np.array([-1.0, 1.0], dtype=np.float32), size=d), x)
    elif kind == "all_zero":
        x = np.zeros(d, dtype=np.float32)
    else:
        raise ValueError(kind)
    return np.ascontiguousarray(x, dtype=np.float32)
