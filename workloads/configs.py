"""The five synthetic MoE-shaped workloads and their group-size draws.

Group sizes are drawn on the CPU with NumPy's PCG64 `default_rng`, so they are
bit-reproducible everywhere.  seed = 20250816 + index of the config.
The paper's own experiments are synthetic as well (Sec. 3.1 and App. C.1); no
dataset is involved, these draws stand in for MoE routing traces.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 20250816


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    index: int
    G: int
    K: int
    N: int
    M_total: int          # 0 => defined by the draw (tiny)
    sizes: str            # which group-size law
    bound: str            # roofline that bounds it on MI355X: "mfma" | "hbm" | "latency"

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index


CONFIGS = {
    "tiny":       WorkloadConfig("tiny",       0, 4,   256,  256,  0,     "uniform300", "latency"),
    "gate_up":    WorkloadConfig("gate_up",    1, 8,   7168, 4096, 8192,  "dirichlet1", "mfma"),
    "down":       WorkloadConfig("down",       2, 32,  2048, 7168, 16384, "zipf1.1",    "mfma"),
    "many_small": WorkloadConfig("many_small", 3, 256, 7168, 4096, 32768, "poisson128", "hbm"),
    "decode":     WorkloadConfig("decode",     4, 64,  7168, 4096, 2048,  "dirichlet0.3", "hbm"),
}


def paper_group_sizes(M: int, G: int, rng: np.random.Generator) -> np.ndarray:
    """The paper's M^g generator (App. C.1): uniform integers in [0, 2*floor(M/G)],
    rescaled by M / sum and floored, the last entry absorbing the remainder."""
    v = rng.integers(0, 2 * (M // G) + 1, size=G).astype(np.int64)
    if v.sum() == 0:
        v[:] = 1
    v = np.floor(v * (M / v.sum())).astype(np.int64)
    v[-1] += M - v.sum()
    return v


def group_sizes(cfg: WorkloadConfig, seed: int | None = None) -> np.ndarray:
    """int64[G] rows per group for a config (sums to cfg.M_total when that is set)."""
    rng = np.random.default_rng(cfg.seed if seed is None else seed)
    G, M = cfg.G, cfg.M_total
    if cfg.sizes == "uniform300":
        s = rng.integers(0, 301, size=G).astype(np.int64)
        i0, i1 = rng.choice(G, size=2, replace=False)
        s[i0], s[i1] = 0, 1
    elif cfg.sizes.startswith("dirichlet"):
        alpha = float(cfg.sizes[len("dirichlet"):])
        p = rng.dirichlet(np.full(G, alpha))
        s = rng.multinomial(M, p).astype(np.int64)
    elif cfg.sizes.startswith("zipf"):
        # expert popularity ~ rank^-s, ranks assigned to experts at random; every
        # group gets a residual r_g uniform in [0,128) and the rest of the rows is
        # dealt out in whole 128-row blocks by that popularity.
        sexp = float(cfg.sizes[len("zipf"):])
        p = np.arange(1, G + 1, dtype=np.float64) ** (-sexp)
        p = rng.permutation(p / p.sum())
        r = rng.integers(0, 128, size=G).astype(np.int64)
        r[-1] = (r[-1] + (M - r.sum())) % 128          # make (M - sum r) a multiple of 128
        assert (M - r.sum()) % 128 == 0 and M >= r.sum()
        q = rng.multinomial((M - r.sum()) // 128, p).astype(np.int64)
        s = 128 * q + r
    elif cfg.sizes.startswith("poisson"):
        lam = float(cfg.sizes[len("poisson"):])
        v = rng.poisson(lam, size=G).astype(np.int64)
        s = np.floor(v * (M / v.sum())).astype(np.int64)   # same renormalisation as App. C.1
        s[-1] += M - s.sum()
    else:
        raise ValueError(cfg.sizes)
    assert np.all(s >= 0)
    if M:
        assert s.sum() == M
    return s
