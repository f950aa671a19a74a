"""Seeded generators for the synthetic training sets.

Output is plain numpy arrays: fp32 values, int32 column indices, int64 row offsets, fp32
labels or targets, and the row boundaries of the fixed-row-count data chunks (the paper's
chunks, Section 4.4, hold a variable number of samples in a fixed number of bytes; here the
row count is fixed and the last chunk is ragged).  Nothing here computes any part of the
training method.

Generation is blocked over rows and every block draws from its own child of one
`numpy.random.SeedSequence`, so the result does not depend on the number of worker threads.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

_BLOCK = 32768  # rows per generation block (one RNG stream each)


@dataclass
class Problem:
    """One training set plus its chunking.  Either `X` (dense) or (`row_ptr`, `col`, `val`)."""
    name: str
    loss: str                      # "hinge" or "squared"
    n: int
    d: int
    lam: float                     # normalised regulariser: P(w) = lam/2 |w|^2 + 1/n sum loss
    y: np.ndarray                  # fp32 [n]
    chunk_bounds: np.ndarray       # int64 [n_chunks + 1], row offsets
    X: Optional[np.ndarray] = None         # fp32 [n, d] row-major
    row_ptr: Optional[np.ndarray] = None   # int64 [n + 1]
    col: Optional[np.ndarray] = None       # int32 [nnz], ascending inside a row
    val: Optional[np.ndarray] = None       # fp32 [nnz]
    meta: dict = field(default_factory=dict)

    @property
    def dense(self) -> bool:
        return self.X is not None

    @property
    def n_chunks(self) -> int:
        return len(self.chunk_bounds) - 1

    @property
    def nnz(self) -> int:
        return self.n * self.d if self.dense else int(self.row_ptr[-1])

    def chunk_rows(self, c: int):
        return int(self.chunk_bounds[c]), int(self.chunk_bounds[c + 1])

    def chunk_nnz(self) -> np.ndarray:
        """Stored entries per chunk (rows x d for dense chunks), int64."""
        b = self.chunk_bounds
        if self.dense:
            return (b[1:] - b[:-1]).astype(np.int64) * self.d
        return (self.row_ptr[b[1:]] - self.row_ptr[b[:-1]]).astype(np.int64)

    def chunk_csr(self, c: int):
        """(row_ptr int32 chunk-local, col, val, y) views/copies of chunk c."""
        r0, r1 = self.chunk_rows(c)
        p0, p1 = int(self.row_ptr[r0]), int(self.row_ptr[r1])
        rp = (self.row_ptr[r0:r1 + 1] - p0).astype(np.int32)
        return rp, self.col[p0:p1], self.val[p0:p1], self.y[r0:r1]

    def chunk_dense(self, c: int):
        r0, r1 = self.chunk_rows(c)
        return self.X[r0:r1], self.y[r0:r1]


def _bounds(n: int, chunk_rows: int) -> np.ndarray:
    b = np.arange(0, n, chunk_rows, dtype=np.int64)
    return np.concatenate([b, np.array([n], dtype=np.int64)])


def _n_threads() -> int:
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit():
        return max(1, min(int(env), 16))
    return max(1, min(os.cpu_count() or 1, 16))


def _blocks(n: int, block: int):
    return [(s, min(n, s + block)) for s in range(0, n, block)]


def _run_blocks(fn, n: int, seed_seq: np.random.SeedSequence, block: int = _BLOCK):
    blocks = _blocks(n, block)
    seeds = seed_seq.spawn(len(blocks))
    args = [(b, np.random.Generator(np.random.PCG64(s))) for b, s in zip(blocks, seeds)]
    nt = _n_threads()
    if nt == 1 or len(blocks) == 1:
        return [fn(b, g) for b, g in args]
    with ThreadPoolExecutor(max_workers=nt) as ex:
        return list(ex.map(lambda a: fn(*a), args))


# --------------------------------------------------------------------------- dense

def _dense_hinge(cfg) -> Problem:
    n, d = cfg["n"], cfg["d"]
    root = np.random.SeedSequence([cfg["seed"], 1])
    s_x, s_w, s_f = root.spawn(3)
    wstar = np.random.Generator(np.random.PCG64(s_w)).standard_normal(d)

    def blk(b, g):
        x = g.standard_normal((b[1] - b[0], d)).astype(np.float32)
        nrm = np.sqrt((x.astype(np.float64) ** 2).sum(axis=1))
        x = (x / nrm[:, None]).astype(np.float32)
        return x

    X = np.concatenate(_run_blocks(blk, n, s_x), axis=0)
    z = X.astype(np.float64) @ wstar
    y = np.where(z >= 0, 1.0, -1.0)
    flip = np.random.Generator(np.random.PCG64(s_f)).random(n) < cfg["flip"]
    y[flip] *= -1.0
    return Problem(cfg["name"], "hinge", n, d, cfg["lam"], y.astype(np.float32),
                   _bounds(n, cfg["chunk_rows"]), X=np.ascontiguousarray(X))


def _dense_ridge(cfg) -> Problem:
    n, d = cfg["n"], cfg["d"]
    root = np.random.SeedSequence([cfg["seed"], 2])
    s_x, s_w, s_e = root.spawn(3)
    wstar = np.random.Generator(np.random.PCG64(s_w)).standard_normal(d)

    def blk(b, g):
        return g.standard_normal((b[1] - b[0], d)).astype(np.float32)

    X = np.concatenate(_run_blocks(blk, n, s_x), axis=0)
    eps = np.random.Generator(np.random.PCG64(s_e)).standard_normal(n) * cfg["noise"]
    y = X.astype(np.float64) @ wstar + eps
    return Problem(cfg["name"], "squared", n, d, cfg["lam"], y.astype(np.float32),
                   _bounds(n, cfg["chunk_rows"]), X=np.ascontiguousarray(X),
                   meta={"wstar": wstar})


# --------------------------------------------------------------------------- sparse

def _bounded_zipf(g: np.random.Generator, a: float, d: int, count: int) -> np.ndarray:
    """`count` ranks in [0, d) with P(rank j) proportional to (j+1)^-a (rejection of j >= d)."""
    out = np.empty(count, dtype=np.int64)
    filled = 0
    while filled < count:
        need = count - filled
        draw = g.zipf(a, size=int(need * 1.5) + 16)
        draw = draw[(draw >= 1) & (draw <= d)]
        take = min(need, draw.size)
        out[filled:filled + take] = draw[:take] - 1
        filled += take
    return out


def _distinct_zipf_rows(g, rows: int, k: int, a: float, d: int) -> np.ndarray:
    """[rows, k] ranks, distinct inside every row, ascending; duplicates are redrawn."""
    if k > d:
        raise ValueError("more entries per row than columns")
    r = _bounded_zipf(g, a, d, rows * k).reshape(rows, k)
    r.sort(axis=1)
    todo = np.arange(rows)
    while todo.size:
        sub = r[todo]
        dup = np.zeros(sub.shape, dtype=bool)
        dup[:, 1:] = sub[:, 1:] == sub[:, :-1]
        has = dup.any(axis=1)
        if not has.any():
            break
        todo = todo[has]
        sub = sub[has]
        dup = dup[has]
        sub[dup] = _bounded_zipf(g, a, d, int(dup.sum()))
        sub.sort(axis=1)
        r[todo] = sub
    return r


def _planted_labels(n, d, row_ptr, col, val, density, flip, s_w, s_f):
    """y = sign(x . w*) for a sparse planted w* (sign(0) = +1), then seeded label flips."""
    gw = np.random.Generator(np.random.PCG64(s_w))
    nz = max(1, int(round(d * density)))
    support = gw.choice(d, size=nz, replace=False)
    wstar = np.zeros(d, dtype=np.float64)
    wstar[support] = gw.standard_normal(nz)
    contrib = val.astype(np.float64) * wstar[col]
    z = np.add.reduceat(contrib, row_ptr[:-1]) if col.size else np.zeros(n)
    # reduceat misbehaves on empty rows; all generated rows have >= 1 entry
    y = np.where(z >= 0, 1.0, -1.0)
    flips = np.random.Generator(np.random.PCG64(s_f)).random(n) < flip
    y[flips] *= -1.0
    return y.astype(np.float32)


def _sparse_zipf(cfg) -> Problem:
    n, d, k, a = cfg["n"], cfg["d"], cfg["nnz_row"], cfg["zipf_a"]
    root = np.random.SeedSequence([cfg["seed"], 3])
    s_rows, s_perm, s_w, s_f = root.spawn(4)
    # popularity rank -> column id: hot columns are scattered over [0, d), as with hashed features
    rank_to_col = np.random.Generator(np.random.PCG64(s_perm)).permutation(d).astype(np.int32)

    def blk(b, g):
        rows = b[1] - b[0]
        ranks = _distinct_zipf_rows(g, rows, k, a, d)
        c = rank_to_col[ranks]
        c.sort(axis=1)
        v = g.random((rows, k))
        v /= np.sqrt((v * v).sum(axis=1))[:, None]
        return c.astype(np.int32), v.astype(np.float32)

    parts = _run_blocks(blk, n, s_rows)
    col = np.concatenate([p[0] for p in parts], axis=0).reshape(-1)
    val = np.concatenate([p[1] for p in parts], axis=0).reshape(-1)
    row_ptr = np.arange(n + 1, dtype=np.int64) * k
    y = _planted_labels(n, d, row_ptr, col, val, cfg["wstar_density"], cfg["flip"], s_w, s_f)
    return Problem(cfg["name"], "hinge", n, d, cfg["lam"], y, _bounds(n, cfg["chunk_rows"]),
                   row_ptr=row_ptr, col=col, val=val)


def _sparse_longrow(cfg) -> Problem:
    n, d = cfg["n"], cfg["d"]
    root = np.random.SeedSequence([cfg["seed"], 4])
    s_len, s_rows, s_w, s_f = root.spawn(4)
    gl = np.random.Generator(np.random.PCG64(s_len))
    lens = np.rint(gl.lognormal(np.log(cfg["median_len"]), cfg["sigma_len"], size=n))
    lens = np.clip(lens, 1, min(cfg["max_len"], d)).astype(np.int64)
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(lens, out=row_ptr[1:])

    def blk(b, g):
        ln = lens[b[0]:b[1]]
        total = int(ln.sum())
        rid = np.repeat(np.arange(ln.size, dtype=np.int64), ln)
        c = g.integers(0, d, size=total, dtype=np.int64)
        key = rid * d + c                      # sort by (row, column)
        key.sort()
        # redraw duplicate (row, column) pairs until none remain
        while True:
            dup = np.zeros(total, dtype=bool)
            dup[1:] = key[1:] == key[:-1]
            m = int(dup.sum())
            if m == 0:
                break
            rows_dup = key[dup] // d
            key[dup] = rows_dup * d + g.integers(0, d, size=m, dtype=np.int64)
            key.sort()
        c = (key % d).astype(np.int32)
        sign = np.where(g.random(total) < 0.5, -1.0, 1.0)
        v = sign / np.sqrt(np.repeat(ln, ln).astype(np.float64))
        return c, v.astype(np.float32)

    parts = _run_blocks(blk, n, s_rows, block=4096)
    col = np.concatenate([p[0] for p in parts])
    val = np.concatenate([p[1] for p in parts])
    y = _planted_labels(n, d, row_ptr, col, val, cfg["wstar_density"], cfg["flip"], s_w, s_f)
    return Problem(cfg["name"], "hinge", n, d, cfg["lam"], y, _bounds(n, cfg["chunk_rows"]),
                   row_ptr=row_ptr, col=col, val=val)


_KINDS = {
    "dense_hinge": _dense_hinge,
    "dense_ridge": _dense_ridge,
    "sparse_zipf": _sparse_zipf,
    "sparse_longrow": _sparse_longrow,
}


def make_problem(cfg: dict) -> Problem:
    """Generate the training set described by a dict from `workloads.configs.get_config`."""
    return _KINDS[cfg["kind"]](cfg)
