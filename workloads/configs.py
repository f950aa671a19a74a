"""The five synthetic workloads and reduced-size variants of each.

Every entry describes one CoCoA training job (Section 5.1 "CoCoA" of the paper names the
hyper-parameters: K tasks, sigma = K, lambda, H = all local samples, L = 1).  The real
datasets of Table 1 are not reproduced; `dense_ridge` borrows the 28-feature dense shape of
the first row of Table 1 and `sparse_zipf` the one-million sparse feature shape of the second.

`size` selects "full" (the size throughput is reported on) or "mini" (a size the CPU oracle
finishes in about a second, still spanning several chunks, several solvers and a ragged
last chunk).
"""
from __future__ import annotations
import copy

CONFIGS = {
    # 1: dense hinge SVM
    "dense_hinge": {
        "kind": "dense_hinge", "loss": "hinge", "lam": 1e-3, "seed": 0, "flip": 0.10,
        "full": dict(n=4096, d=256, K=4, chunk_rows=1024, rounds=10),
        "mini": dict(n=1000, d=48, K=4, chunk_rows=256, rounds=6),
    },
    # 2: dense ridge regression
    "dense_ridge": {
        "kind": "dense_ridge", "loss": "squared", "lam": 1e-4, "seed": 0, "noise": 0.1,
        "full": dict(n=500_000, d=28, K=16, chunk_rows=4096, rounds=50),
        "mini": dict(n=9000, d=28, K=5, chunk_rows=512, rounds=12),
    },
    # 3: sparse hinge SVM, Zipf column popularity
    "sparse_zipf": {
        "kind": "sparse_zipf", "loss": "hinge", "lam": 1e-5, "seed": 0, "flip": 0.05,
        "zipf_a": 1.1, "nnz_row": 40, "wstar_density": 0.01,
        "full": dict(n=2_000_000, d=1_000_000, K=32, chunk_rows=4096, rounds=20),
        "mini": dict(n=30_000, d=20_000, K=6, chunk_rows=1024, rounds=6),
    },
    # 4: sparse long-row hinge SVM
    "sparse_longrow": {
        "kind": "sparse_longrow", "loss": "hinge", "lam": 1e-6, "seed": 0, "flip": 0.05,
        "median_len": 800, "sigma_len": 0.668, "max_len": 20_000, "wstar_density": 0.01,
        "full": dict(n=100_000, d=20_000_000, K=64, chunk_rows=1024, rounds=10),
        "mini": dict(n=1500, d=200_000, K=7, chunk_rows=128, rounds=4,
                     median_len=300, max_len=3000),
    },
    # 5: elastic schedule on the data of workload 3
    "elastic": {
        "kind": "sparse_zipf", "loss": "hinge", "lam": 1e-5, "seed": 0, "flip": 0.05,
        "zipf_a": 1.1, "nnz_row": 40, "wstar_density": 0.01,
        # (first round, K) pairs; rounds are 0-based; reassignment happens before that round
        "full": dict(n=2_000_000, d=1_000_000, K=32, chunk_rows=4096, rounds=20,
                     schedule=[(0, 32), (5, 8), (10, 64), (15, 16)]),
        "mini": dict(n=30_000, d=20_000, K=6, chunk_rows=1024, rounds=8,
                     schedule=[(0, 6), (2, 2), (4, 9), (6, 4)]),
        # relative solver speeds, alternating by solver index, as integer weights (1.0 -> 2, 0.5 -> 1)
        "speed_q": (2, 1),
    },
}


def get_config(name: str, size: str = "full") -> dict:
    """Flat dict for one workload: common keys merged with the `size` keys."""
    base = copy.deepcopy(CONFIGS[name])
    sized = base.pop(size)
    for other in ("full", "mini"):
        base.pop(other, None)
    base.update(sized)
    base["name"] = name
    base["size"] = size
    if "schedule" not in base:
        base["schedule"] = [(0, base["K"])]
    return base


def k_for_round(cfg: dict, r: int) -> int:
    """Number of solvers in force during round r (0-based)."""
    k = cfg["schedule"][0][1]
    for start, kk in cfg["schedule"]:
        if r >= start:
            k = kk
    return k


def speeds_for(cfg: dict, K: int):
    """Integer speed weight per solver, or None when all solvers are equally fast."""
    sq = cfg.get("speed_q")
    if sq is None:
        return None
    return [sq[k % len(sq)] for k in range(K)]
