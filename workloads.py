"""Seeded synthetic gradients for the five benchmark configurations.

This module serves both the CPU reference and the HIP library and therefore contains none
of the method's arithmetic (no hashing, no sketching, no selection): it only draws numbers.
A gradient is a pure function of (config, step t, worker w): every call re-seeds a
torch.Generator from those three integers, so "generated on the fly from the seed" means
that a worker's vector can be re-created at any time, on the device it will be consumed on,
and copied to the host for the reference, which then sees bit-identical fp32 values.

The vectors stand in for the gradients of the paper's transformer / LSTM (Sec. 5.3) and
residual-network (Sec. 5.4) experiments, whose datasets are not available here: only the
sizes, the number of workers and a heavy-tailed value structure are mimicked.

N(0, 1e-4) is read as variance 1e-4 (standard deviation 0.01).  Planted heavy coordinates
(index set, magnitudes, signs) are drawn once per configuration and are identical for all
workers and steps; noise is redrawn per (step, worker).
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np
import torch

BASE_SEED = 190304488


@dataclasses.dataclass(frozen=True)
class Config:
    cfg: int          # 1..5, which value recipe to use
    d: int            # gradient length
    W: int            # simulated workers
    r: int            # sketch rows
    c: int            # sketch columns
    k: int            # coordinates selected per step
    steps: int        # steps of the configuration (1 = stateless)
    rho: float | None  # momentum (None = no sketch-space state)
    n_heavy: int      # planted / heavy-subset size
    name: str = ""
    P: int = 1        # candidates asked of the sketch per selected coordinate (Sec. 5.1)
    recipe: int = 0   # value recipe when it is not the one numbered `cfg` (0: use cfg)

    @property
    def hash_seed(self) -> int:
        return BASE_SEED + self.cfg

    @property
    def data_seed(self) -> int:
        return (BASE_SEED + self.cfg) ^ 0xD47A

    @property
    def stateful(self) -> bool:
        return self.rho is not None


CONFIGS = {
    1: Config(1, 1 << 20, 4, 5, 1 << 15, 1000, 1, None, 1000, "planted-1M"),
    2: Config(2, 6_500_000, 8, 5, 1 << 17, 5000, 1, None, 5000, "student-t-6.5M"),
    3: Config(3, 11_000_000, 16, 5, 1 << 18, 50_000, 1, None, 0, "log-uniform-scale-11M"),
    4: Config(4, 100_000_000, 32, 5, 1 << 20, 100_000, 10, 0.9, 100_000, "transformer-100M"),
    5: Config(5, 25_000_000, 256, 7, 1 << 19, 20_000, 20, 0.9, 20_000, "many-workers-25M"),
}

# The sketch shapes the paper itself trains with (Sec. 5.3, Table 1 and its footnotes: W = 4
# workers, k = 100 000, about 90 M parameters for the transformer and 73 M for the LSTM), as extra
# workloads for bench.py.  They are no part of the benchmark definition's five configurations;
# the values follow recipe 4 (Gaussian body, 0.1 % Laplace), the gradients of the paper's models
# not being available.
PAPER_SHAPES = {
    6: Config(6, 90_000_000, 4, 5, 1_000_000, 100_000, 10, 0.9, 90_000, "paper-transformer-5x1M-P36", P=36, recipe=4),
    7: Config(7, 90_000_000, 4, 15, 180_000, 100_000, 10, 0.9, 90_000, "paper-transformer-15x180k-P16", P=16, recipe=4),
    8: Config(8, 73_000_000, 4, 5, 180_000, 100_000, 10, 0.9, 73_000, "paper-lstm-5x180k-P26", P=26, recipe=4),
}
ALL_CONFIGS = {**CONFIGS, **PAPER_SHAPES}


def scaled(cfg: int, **overrides) -> Config:
    """A configuration with the same value recipe but other sizes (tests use small ones)."""
    return dataclasses.replace(CONFIGS[cfg], **overrides)


def _mix(seed: int, t: int, w: int) -> int:
    return (seed * 0x9E3779B1 + (t + 1) * 1000003 + (w + 1) * 7919) & 0x7FFFFFFFFFFFFFFF


class Workload:
    """Draws worker gradients for one configuration on `device` ("cpu" or "cuda:0")."""

    def __init__(self, config: Config, device="cpu"):
        self.config = config
        self.device = torch.device(device)
        c = config
        self.recipe = c.recipe or c.cfg
        rng = np.random.default_rng(c.data_seed)
        self.heavy_idx = None
        self.heavy_val = None
        self.tau = None
        if self.recipe in (1, 2, 5) and c.n_heavy > 0:
            lo = 0.1 if self.recipe == 2 else 0.5
            idx = np.sort(rng.choice(c.d, size=c.n_heavy, replace=False)).astype(np.int64)
            mag = rng.uniform(lo, 1.0, size=c.n_heavy)
            sgn = rng.integers(0, 2, size=c.n_heavy) * 2 - 1
            self.heavy_idx = torch.from_numpy(idx).to(self.device)
            self.heavy_val = torch.from_numpy((mag * sgn).astype(np.float32)).to(self.device)
        elif self.recipe == 4 and c.n_heavy > 0:
            idx = np.sort(rng.choice(c.d, size=c.n_heavy, replace=False)).astype(np.int64)
            self.heavy_idx = torch.from_numpy(idx).to(self.device)
        if self.recipe == 3:
            gen = torch.Generator(device=self.device)
            gen.manual_seed(_mix(c.data_seed, -1, -1))
            e = torch.empty(c.d, dtype=torch.float32, device=self.device)
            e.uniform_(-6.0, -1.0, generator=gen)
            self.tau = torch.pow(10.0, e)

    def gradient(self, t: int, w: int, out: torch.Tensor | None = None) -> torch.Tensor:
        """fp32[d] gradient of worker w at step t (written into `out` when given)."""
        c = self.config
        gen = torch.Generator(device=self.device)
        gen.manual_seed(_mix(c.data_seed, t, w))
        g = out if out is not None else torch.empty(c.d, dtype=torch.float32, device=self.device)
        assert g.shape == (c.d,) and g.dtype == torch.float32
        if self.recipe in (1, 5):
            g.normal_(0.0, 0.01, generator=gen)
            if self.heavy_idx is not None:
                g[self.heavy_idx] += self.heavy_val
        elif self.recipe == 2:
            # Student-t, 3 degrees of freedom: Z / sqrt((Z1^2 + Z2^2 + Z3^2) / 3)
            g.normal_(0.0, 1.0, generator=gen)
            chi = torch.zeros_like(g)
            tmp = torch.empty_like(g)
            for _ in range(3):
                tmp.normal_(0.0, 1.0, generator=gen)
                chi.addcmul_(tmp, tmp)
            g.div_(torch.sqrt(chi / 3.0)).mul_(1e-3)
            if self.heavy_idx is not None:
                g[self.heavy_idx] += self.heavy_val
        elif self.recipe == 3:
            g.normal_(0.0, 1.0, generator=gen)
            g.mul_(self.tau)
        elif self.recipe == 4:
            g.normal_(0.0, 0.01, generator=gen)
            if self.heavy_idx is not None:
                n = self.heavy_idx.numel()
                u = torch.empty(n, dtype=torch.float32, device=self.device)
                u.uniform_(-0.5, 0.5, generator=gen)
                # Laplace(0, b) by inverse CDF: -b sign(u) ln(1 - 2|u|)
                lap = -0.1 * torch.sign(u) * torch.log1p(-2.0 * u.abs().clamp(max=0.4999999))
                g[self.heavy_idx] = lap
        else:
            raise ValueError(f"unknown recipe {self.recipe}")
        return g

    def all_workers(self, t: int) -> list:
        return [self.gradient(t, w) for w in range(self.config.W)]


def describe(config: Config) -> str:
    c = config
    tbl = 4 * c.r * c.c
    return (f"cfg{c.cfg} {c.name}: d={c.d} W={c.W} r={c.r} c={c.c} k={c.k} steps={c.steps} "
            f"rho={c.rho} table={tbl / 1e6:.2f} MB gradients={4 * c.d * c.W / 1e9:.3f} GB "
            f"d/c={c.d / c.c:.1f} log2(c)={math.log2(c.c):.2f}")
