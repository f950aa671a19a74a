"""Python face of the CPU oracle (ctypes over `cocoa_oracle.c`, compiled with gcc).

TEST INFRASTRUCTURE ONLY: plain, single-threaded, double-precision.  The round follows the
paper's Section 2.2 ("CoCoA": K workers, local subproblems, combined into the shared model;
L = 1, H = all local samples) and Section 5.1 ("CoCoA": sigma = number of tasks); the
trainer/solver protocol is the one of Section 4.1-4.2 (solvers fetch the model, train on all
task-local chunks, post their update; the trainer merges).  Chunk ownership follows Section 3:
a solver's rows are the rows of the chunks assigned to it, chunks in ascending id, rows in
ascending order inside a chunk; the per-sample state (alpha) stays with its chunk.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cocoa_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

_LOSS = {"hinge": 0, "squared": 1, "logistic": 2}


def build_oracle(force: bool = False) -> str:
    """Compile the C oracle with gcc (about a second).  Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build_oracle()
        L = ctypes.CDLL(_LIB)
        c_i64, c_i32, c_d, c_vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_double, ctypes.c_void_p
        L.oracle_local_epoch_csr.argtypes = [ctypes.c_int, c_i64, c_vp, c_vp, c_vp, c_vp, c_vp,
                                             c_vp, c_vp, c_vp, c_d, c_i64, c_d]
        L.oracle_local_epoch_csr.restype = None
        L.oracle_local_epoch_dense.argtypes = [ctypes.c_int, c_i64, c_vp, c_vp, c_vp, c_i64, c_vp,
                                               c_vp, c_vp, c_d, c_i64, c_d]
        L.oracle_local_epoch_dense.restype = None
        L.oracle_gap.argtypes = [ctypes.c_int, c_i64, c_i64, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp,
                                 c_vp, c_d, c_d, c_vp]
        L.oracle_gap.restype = None
        L.oracle_soft_threshold.argtypes = [c_i64, c_vp, c_d, c_vp]
        L.oracle_soft_threshold.restype = None
        L.oracle_assign_greedy.argtypes = [c_vp, c_i32, c_i32, c_vp, c_vp, c_vp, c_vp]
        L.oracle_assign_greedy.restype = ctypes.c_int
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def assign_greedy(load: Sequence[int], K: int, speed: Optional[Sequence[int]] = None) -> np.ndarray:
    """Chunk -> solver table: longest-processing-time-first on integer loads and speeds."""
    L = _load()
    load = np.ascontiguousarray(load, dtype=np.int64)
    sp = None if speed is None else np.ascontiguousarray(speed, dtype=np.int32)
    if sp is not None and sp.size != K:
        raise ValueError("one speed per solver")
    out = np.empty(load.size, dtype=np.int32)
    order = np.empty(max(1, load.size), dtype=np.int32)
    acc = np.empty(max(1, K), dtype=np.int64)
    rc = L.oracle_assign_greedy(_p(load), load.size, K, _p(sp), _p(out), _p(order), _p(acc))
    if rc != 0:
        raise ValueError("bad assignment input")
    return out


def projected_round_time(K_tasks: Optional[int], nodes: int, base_nodes: int = 16,
                         slow_factor: Optional[float] = None, n_slow: int = 0) -> float:
    """Iteration time in the paper's normalised units (one task on 1/base_nodes of the data = 1).

    Section 5.3 methodology: K micro-tasks on N equal nodes need ceil(K/N) waves of length
    base/K each; uni-tasks redistribute the load so an iteration takes base/N.
    Section 5.4 methodology: with `n_slow` nodes slower by `slow_factor`, micro-tasks take
    min over splits of max(i*slow_factor, j) * base/K with i (j) tasks per slow (fast) node;
    uni-tasks give every node work proportional to its speed.
    `K_tasks=None` selects uni-tasks.
    """
    if slow_factor is None or n_slow == 0:
        if K_tasks is None:
            return base_nodes / nodes
        return base_nodes / K_tasks * (-(-K_tasks // nodes))
    n_fast = nodes - n_slow
    if K_tasks is None:
        capacity = n_fast * 1.0 + n_slow / slow_factor
        return base_nodes / capacity
    best = None
    for i in range(0, -(-K_tasks // max(n_slow, 1)) + 1):      # up to all tasks on the slow nodes
        rest = max(K_tasks - i * n_slow, 0)
        j = -(-rest // n_fast) if n_fast else (0 if rest == 0 else None)
        if j is None:
            continue
        t = max(i * slow_factor, j * 1.0) * base_nodes / K_tasks
        best = t if best is None or t < best else best
    return best


class OracleCoCoA:
    """State and steps of the round: alpha (per row), w, the chunk -> solver table.

    Data: dense `X` [n, d] fp32, or CSR (`row_ptr` int64 [n+1], `col` int32, `val` fp32);
    `y` fp32 [n]; `chunk_bounds` int64 row offsets of the chunks.
    """

    def __init__(self, loss: str, n: int, d: int, lam: float, y, chunk_bounds,
                 X=None, row_ptr=None, col=None, val=None, l1: float = 0.0):
        self.L = _load()
        self.loss = _LOSS[loss]
        self.n, self.d, self.lam = int(n), int(d), float(lam)
        self.y = np.ascontiguousarray(y, dtype=np.float32)
        self.chunk_bounds = np.ascontiguousarray(chunk_bounds, dtype=np.int64)
        self.X = None if X is None else np.ascontiguousarray(X, dtype=np.float32)
        self.row_ptr = None if row_ptr is None else np.ascontiguousarray(row_ptr, dtype=np.int64)
        self.col = None if col is None else np.ascontiguousarray(col, dtype=np.int32)
        self.val = None if val is None else np.ascontiguousarray(val, dtype=np.float32)
        self.alpha = np.zeros(self.n, dtype=np.float64)
        self.w = np.zeros(self.d, dtype=np.float64)
        # Elastic net (Section 2.2 speaks of generalised linear models in general): regulariser
        # lambda (|w|^2 / 2 + l1 |w|_1).  The solvers' updates add up in the dual image v; the shared
        # vector is its soft-thresholded image, w = S_l1(v).  A local pass is unchanged: it starts from
        # the shared w and its update is linear in the dual steps (the subproblem bounds the conjugate of
        # the regulariser, which is 1-smooth, by a quadratic around v).  l1 = 0: w = v.
        self.l1 = float(l1)
        self.v = np.zeros(self.d, dtype=np.float64)
        self.K = 0
        self.chunk_to_solver = None
        self.rows_of: List[np.ndarray] = []
        self._pending: Optional[np.ndarray] = None   # sum_k Delta w_k awaiting aggregation

    @classmethod
    def from_problem(cls, p, l1: float = 0.0):
        return cls(p.loss, p.n, p.d, p.lam, p.y, p.chunk_bounds, X=p.X, row_ptr=p.row_ptr,
                   col=p.col, val=p.val, l1=l1)

    # ---- scheduler side (between iterations) -------------------------------------------------
    def assign(self, K: int, chunk_to_solver) -> None:
        """Give every chunk to one of K solvers; sigma becomes K.  alpha is untouched."""
        if self._pending is not None:
            raise RuntimeError("assign between iterations only (aggregate first)")
        c2s = np.ascontiguousarray(chunk_to_solver, dtype=np.int32)
        if c2s.size != self.chunk_bounds.size - 1 or (c2s.size and (c2s.min() < 0 or c2s.max() >= K)):
            raise ValueError("bad chunk -> solver table")
        self.K = int(K)
        self.chunk_to_solver = c2s.copy()
        self.rows_of = []
        for k in range(K):
            parts = [np.arange(self.chunk_bounds[c], self.chunk_bounds[c + 1], dtype=np.int64)
                     for c in np.nonzero(c2s == k)[0]]
            self.rows_of.append(np.concatenate(parts) if parts else np.empty(0, dtype=np.int64))

    def rows_per_solver(self) -> List[int]:
        return [int(r.size) for r in self.rows_of]

    # ---- solver side (during an iteration) ---------------------------------------------------
    def solver_delta(self, k: int, perm) -> np.ndarray:
        """Run solver k's local pass from the current w; commits alpha; returns Delta w_k."""
        rows = self.rows_of[k]
        perm = np.ascontiguousarray(perm, dtype=np.int32)
        if perm.size != rows.size or (perm.size and not np.array_equal(np.sort(perm), np.arange(rows.size))):
            raise ValueError("perm must be a permutation of the solver's local rows")
        sigma = float(self.K)
        v = self.w.copy()
        if self.X is not None:
            self.L.oracle_local_epoch_dense(self.loss, rows.size, _p(rows), _p(perm), _p(self.X),
                                            self.d, _p(self.y), _p(self.alpha), _p(v),
                                            self.lam, self.n, sigma)
        else:
            self.L.oracle_local_epoch_csr(self.loss, rows.size, _p(rows), _p(perm), _p(self.row_ptr),
                                          _p(self.col), _p(self.val), _p(self.y), _p(self.alpha),
                                          _p(v), self.lam, self.n, sigma)
        return (v - self.w) / sigma

    def local_epoch(self, perms, keep_deltas: bool = True, on_delta=None):
        """All K local passes, one solver after the other, all from the same w.

        Returns the list of Delta w_k (or None when keep_deltas is False); `on_delta(k, dw)` is
        called for each solver when given.  The sum is held until `aggregate`.
        """
        if self._pending is not None:
            raise RuntimeError("aggregate before the next local epoch")
        total = np.zeros(self.d, dtype=np.float64)
        out = [] if keep_deltas else None
        for k in range(self.K):
            dw = self.solver_delta(k, perms[k])
            total += dw
            if on_delta is not None:
                on_delta(k, dw)
            if keep_deltas:
                out.append(dw)
        self._pending = total
        return out

    # ---- trainer side ------------------------------------------------------------------------
    def aggregate(self) -> np.ndarray:
        """v <- v + sum_k Delta w_k (adding, gamma = 1), w <- S_l1(v).  Returns the sum that was added."""
        if self._pending is None:
            raise RuntimeError("nothing to aggregate")
        s = self._pending
        self.v = self.v + s
        if self.l1 > 0.0:
            w = np.empty_like(self.v)
            self.L.oracle_soft_threshold(self.d, _p(self.v), self.l1, _p(w))
            self.w = w
        else:
            self.w = self.v.copy()
        self._pending = None
        return s

    def gap(self):
        """(P, D, P - D, Fenchel-Young form) at the current (w, alpha)."""
        out = np.zeros(4, dtype=np.float64)
        self.L.oracle_gap(self.loss, self.n, self.d, _p(self.X), _p(self.row_ptr), _p(self.col),
                          _p(self.val), _p(self.y), _p(self.alpha), _p(self.w), self.lam, self.l1, _p(out))
        return tuple(float(x) for x in out)
