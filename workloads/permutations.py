"""Per-(round, solver) coordinate orders for the local solvers.

Each local solver makes one pass over its rows without replacement in a fresh random order
every round (H = all local samples, L = 1 in the paper's Section 2.2 / 5.1 notation).  The
orders are inputs: they are generated here once and handed, as int32 arrays, to the oracle
and to the GPU library alike.

A permutation is numpy's `Generator.permutation` driven by the counter-based Philox
generator keyed with (seed, round, solver), so any (round, solver) order can be produced
independently of the others.
"""
from __future__ import annotations

import numpy as np


def solver_permutation(seed: int, rnd: int, solver: int, n_local: int) -> np.ndarray:
    """Permutation of [0, n_local) for one solver in one round, int32."""
    key = np.array([np.uint64(seed), (np.uint64(rnd) << np.uint64(32)) | np.uint64(solver)],
                   dtype=np.uint64)
    g = np.random.Generator(np.random.Philox(key=key))
    return g.permutation(n_local).astype(np.int32)


def round_permutations(seed: int, rnd: int, rows_per_solver) -> list:
    """One permutation per solver for round `rnd`; `rows_per_solver[k]` = rows solver k owns."""
    return [solver_permutation(seed, rnd, k, int(nk)) for k, nk in enumerate(rows_per_solver)]


def chunk_draws(seed: int, rnd: int, n_chunks: int) -> np.ndarray:
    """One random 32-bit word per chunk for a scaling step before round `rnd` (input to the
    random chunk picks of the scale-out policy), uint32."""
    key = np.array([np.uint64(seed) ^ np.uint64(0x5CA1E), np.uint64(rnd)], dtype=np.uint64)
    g = np.random.Generator(np.random.Philox(key=key))
    return g.integers(0, 2 ** 32, n_chunks, dtype=np.uint64).astype(np.uint32)
