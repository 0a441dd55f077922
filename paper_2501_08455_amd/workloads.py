"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds input generation only (no signature arithmetic) so that the
fp64 oracle and the HIP path can be fed the identical float32 buffers.  The
paper's own benchmark inputs are unspecified synthetic tensors (Section 4.2
says only "synthetic"); the shapes and distributions below are the five
benchmark configurations of this build.

Paths are generated in float64 with numpy's PCG64 and rounded once to float32;
both implementations receive that float32 array.
"""
from collections import namedtuple

import numpy as np

Config = namedtuple("Config", "name B L d depth stream dist")

BASE_SEED = 250108455

CONFIGS = {
    # name        B    L     d   N  stream  increment law
    "C1": Config("C1", 4, 16, 2, 3, False, "normal"),
    "C2": Config("C2", 128, 100, 5, 4, False, "normal"),
    "C3": Config("C3", 128, 2000, 5, 4, False, "normal"),
    "C4": Config("C4", 64, 256, 4, 4, True, "normal"),
    "C5": Config("C5", 16, 128, 10, 6, False, "uniform"),
}
_ORDER = ["C1", "C2", "C3", "C4", "C5"]


def brownian_paths(B, L, d, seed):
    """Paths starting at 0 whose L-1 increments are i.i.d. N(0, 1/L); float32 [B, L, d]."""
    rng = np.random.default_rng(seed)
    xi = rng.normal(0.0, np.sqrt(1.0 / L), size=(B, L - 1, d))
    x = np.zeros((B, L, d), dtype=np.float64)
    np.cumsum(xi, axis=1, out=x[:, 1:, :])
    return x.astype(np.float32)


def uniform_paths(B, L, d, seed, half_width=0.1):
    """Paths starting at 0 whose increments are i.i.d. U(-half_width, half_width); float32 [B, L, d]."""
    rng = np.random.default_rng(seed)
    xi = rng.uniform(-half_width, half_width, size=(B, L - 1, d))
    x = np.zeros((B, L, d), dtype=np.float64)
    np.cumsum(xi, axis=1, out=x[:, 1:, :])
    return x.astype(np.float32)


def make_paths(cfg, B=None, seed=None):
    """Input of a named configuration; `B` overrides the batch (batch-saturated variants)."""
    if isinstance(cfg, str):
        cfg = CONFIGS[cfg]
    if seed is None:
        seed = BASE_SEED + _ORDER.index(cfg.name)
    B = cfg.B if B is None else B
    if cfg.dist == "normal":
        return brownian_paths(B, cfg.L, cfg.d, seed)
    return uniform_paths(B, cfg.L, cfg.d, seed)


def sig_size(d, depth):
    """Row length of a depth-`depth` signature in d channels: d + d^2 + ... + d^depth."""
    return sum(d ** n for n in range(1, depth + 1))


def fused_fma_per_step(d, depth):
    """FMAs of one fused multiply-by-exponential step in Horner form: sum_m (depth-m+1) d^m."""
    return sum((depth - m + 1) * d ** m for m in range(1, depth + 1))
