"""Solves the degree scale `ell` of each configuration for its stated mean degree.

The degree law is deg(v) = clamp(floor(ell / x_v^(p4/4)), 1, d_max) with x_v the
hashed uniform of node v (see workload/synth.py).  The mean over the nodes grows
with ell, so bisection finds the ell whose realised mean is the configuration's;
the value is then frozen in workload/configs.py (a change of ell changes every
graph, so it is data, not something to recompute at run time).

    python -m workload.calibrate [tiny medium ...]

prints the solved ell beside the frozen one.
"""
from __future__ import annotations

import sys

import numpy as np

from .configs import CONFIGS
from .synth import TAGS, U64, hash_chain


def inverse_scale(seed: int, n: int, p4: int, chunk: int = 1 << 24) -> np.ndarray:
    """1 / x_v^(p4/4) per node, with the generator's own operations (sqrt, multiply, divide)."""
    out = np.empty(n, dtype=np.float64)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        h = hash_chain(seed, TAGS["DEG"], np.arange(lo, hi, dtype=U64))
        x = ((h >> U64(32)).astype(np.float64) + 1.0) / 4294967296.0
        q = np.sqrt(np.sqrt(x))
        y = q.copy()
        for _ in range(p4 - 1):
            y = y * q
        out[lo:hi] = y
    return out


def mean_degree(ell: float, y: np.ndarray, d_max: int) -> float:
    total = 0
    for lo in range(0, len(y), 1 << 24):
        d = np.floor(ell / y[lo:lo + (1 << 24)])
        total += float(np.clip(d, 1, d_max).sum())
    return total / len(y)


def solve(name: str) -> float:
    cfg = CONFIGS[name]
    y = inverse_scale(cfg.seed, cfg.n_nodes, cfg.p4)
    lo, hi = 1e-3, 64.0
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        if mean_degree(mid, y, cfg.d_max) < cfg.mean_degree:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


if __name__ == "__main__":
    for name in (sys.argv[1:] or ["tiny", "medium"]):
        cfg = CONFIGS[name]
        ell = solve(name)
        y = inverse_scale(cfg.seed, cfg.n_nodes, cfg.p4)
        print(f"{name}: solved ell = {ell!r} (mean {mean_degree(ell, y, cfg.d_max):.4f}); frozen ell = {cfg.ell!r} "
              f"(mean {mean_degree(cfg.ell, y, cfg.d_max):.4f}, target {cfg.mean_degree})")
