"""The benchmark configurations (graph, sampling, cache) as plain data."""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

MiB = 1 << 20
GiB = 1 << 30


@dataclass(frozen=True)
class Config:
    name: str
    seed: int
    n_nodes: int
    zipf_a: float       # degree law: tail exponent a - 1 = 4 / p4
    p4: int
    ell: float          # degree scale, solved once for the stated mean degree and frozen
    mean_degree: float
    index_dtype: str    # CSR / ID dtype: "int32" or "int64"
    dim: int
    feat_dtype: str     # "float32" or "float16"
    fanouts: tuple
    n_seeds: int
    n_batches: int
    cache_lines: int
    ways: int
    line_bytes: int
    cpu_rows: int       # rows pinned in the constant CPU buffer
    window: int
    seed_zipf_s: float | None = None

    @property
    def row_bytes(self) -> int:
        return self.dim * np.dtype(self.feat_dtype).itemsize

    @property
    def id_bytes(self) -> int:
        return np.dtype(self.index_dtype).itemsize

    @property
    def n_sets(self) -> int:
        return self.cache_lines // self.ways

    @property
    def d_max(self) -> int:
        return min(self.n_nodes - 1, 65535)


def _cfg(**kw) -> Config:
    return Config(**kw)


# `ell` values come from workload/calibrate.py (bisection on the realised mean degree).
CONFIGS = {
    "tiny": _cfg(name="tiny", seed=0x6A1D5_0001, n_nodes=10_000, zipf_a=2.0, p4=4, ell=1.0360073614865544,
                 mean_degree=10, index_dtype="int32", dim=128, feat_dtype="float32", fanouts=(10, 5),
                 n_seeds=256, n_batches=20, cache_lines=1024, ways=4, line_bytes=512, cpu_rows=500, window=4),
    "medium": _cfg(name="medium", seed=0x6A1D5_0002, n_nodes=1_000_000, zipf_a=2.0, p4=4, ell=1.2602475821040573,
                   mean_degree=15, index_dtype="int64", dim=1024, feat_dtype="float16", fanouts=(15, 10),
                   n_seeds=1024, n_batches=200, cache_lines=256 * MiB // 2048, ways=8, line_bytes=2048,
                   cpu_rows=20_000, window=8),
    "large": _cfg(name="large", seed=0x6A1D5_0003, n_nodes=50_000_000, zipf_a=1.8, p4=5, ell=0.19718919227573953,
                  mean_degree=12, index_dtype="int64", dim=1024, feat_dtype="float16", fanouts=(10, 10, 10),
                  n_seeds=4096, n_batches=500, cache_lines=16 * GiB // 2048, ways=8, line_bytes=2048,
                  cpu_rows=4 * GiB // 2048, window=8),
    "skew": _cfg(name="skew", seed=0x6A1D5_0003, n_nodes=50_000_000, zipf_a=1.8, p4=5, ell=0.19718919227573953,
                 mean_degree=12, index_dtype="int64", dim=1024, feat_dtype="float16", fanouts=(25, 10),
                 n_seeds=2048, n_batches=300, cache_lines=32 * GiB // 2048, ways=16, line_bytes=2048,
                 cpu_rows=4 * GiB // 2048, window=4, seed_zipf_s=0.8),
    "resident": _cfg(name="resident", seed=0x6A1D5_0005, n_nodes=10_000_000, zipf_a=2.0, p4=4, ell=1.7909835150931028,
                     mean_degree=20, index_dtype="int64", dim=768, feat_dtype="float32", fanouts=(20, 15, 10),
                     n_seeds=8192, n_batches=1000, cache_lines=40 * GiB // 4096, ways=16, line_bytes=4096,
                     cpu_rows=0, window=8),
}


def scaled(cfg: Config, n_nodes: int) -> Config:
    """The same configuration at another node count, every ratio kept
    (cache : store, CPU buffer : store); sets stay a whole number."""
    f = n_nodes / cfg.n_nodes
    n_sets = max(1, round(cfg.n_sets * f))
    return replace(cfg, name=f"{cfg.name}@{n_nodes}", n_nodes=n_nodes, cache_lines=n_sets * cfg.ways,
                   cpu_rows=int(round(cfg.cpu_rows * f)))
