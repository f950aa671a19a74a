"""ctypes binding of the C ABI in include/chicle_round.h: argument marshalling only.

The method names are the C entry points without the `chicle_` prefix.  Host arrays are numpy,
device arrays are torch CUDA tensors (PyTorch-ROCm supplies device memory and the stream).  If the
shared library is missing or a call fails this raises; there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libchicle_round.so")
_lib = None

OK, EINVAL, ENOMEM, ESTATE, EDEVICE = 0, -1, -2, -3, -4
LOSS = {"hinge": 0, "squared": 1, "logistic": 2}
SOLVER = {"auto": 0, "rowwise": 1, "batched": 2, "rowwise_one_cu": 3, "batched_one_cu": 4}
SEGMENT = {"local_epoch": 0, "aggregate": 1, "gap": 2, "epoch_gram": 3, "epoch_chain": 4}

EXPORTS = [
    "chicle_arena_bytes", "chicle_create", "chicle_load_chunk_csr", "chicle_load_chunk_dense",
    "chicle_balance", "chicle_assign", "chicle_solver_rows", "chicle_set_solver",
    "chicle_local_epoch", "chicle_local_epoch_ahead", "chicle_local_epoch_host_perm", "chicle_aggregate", "chicle_gap",
    "chicle_get_w", "chicle_set_w", "chicle_get_delta_w", "chicle_get_alpha", "chicle_set_alpha",
    "chicle_get_assignment", "chicle_debug_gram", "chicle_sync", "chicle_set_profiling",
    "chicle_last_kernel_ms", "chicle_last_error", "chicle_destroy",
    "chicle_solver_ms", "chicle_projected_iteration_time", "chicle_scale_out", "chicle_scale_in",
    "chicle_rebalance", "chicle_next_solver_count", "chicle_gap_noalloc", "chicle_set_l1",
]


class ChicleError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("chicle error %d: %s" % (code, msg))
        self.code = code


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """dlopen the built library; build it first (hipcc) only when no built library exists."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from .build import build_library
        build_library()
    # PyTorch-ROCm carries its own HIP runtime (same soname as the system one).  Import it first so
    # that this library binds to the runtime that owns the arena and the stream; two HIP runtimes in
    # one process do not see each other's allocations.
    import torch  # noqa: F401
    L = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double
    sz = ctypes.c_size_t
    sig = {
        "chicle_arena_bytes": (sz, [i64, i64, i32, i32, i32, i32]),
        "chicle_create": (ctypes.c_int, [ctypes.POINTER(vp), i32, i64, i32, dbl, i32, i32, i32, i64, vp, sz, vp]),
        "chicle_load_chunk_csr": (ctypes.c_int, [vp, i32, i32, vp, vp, vp, vp, vp]),
        "chicle_load_chunk_dense": (ctypes.c_int, [vp, i32, i32, vp, vp, vp]),
        "chicle_balance": (ctypes.c_int, [vp, i32, i32, vp, vp]),
        "chicle_assign": (ctypes.c_int, [vp, i32, vp]),
        "chicle_solver_rows": (ctypes.c_int, [vp, vp]),
        "chicle_set_solver": (ctypes.c_int, [vp, i32]),
        "chicle_set_l1": (ctypes.c_int, [vp, dbl]),
        "chicle_local_epoch": (ctypes.c_int, [vp, vp]),
        "chicle_local_epoch_ahead": (ctypes.c_int, [vp, vp, vp]),
        "chicle_local_epoch_host_perm": (ctypes.c_int, [vp, vp]),
        "chicle_aggregate": (ctypes.c_int, [vp]),
        "chicle_gap": (ctypes.c_int, [vp, ctypes.POINTER(dbl), ctypes.POINTER(dbl), ctypes.POINTER(dbl)]),
        "chicle_gap_noalloc": (ctypes.c_int, [vp, ctypes.POINTER(dbl), ctypes.POINTER(dbl), ctypes.POINTER(dbl)]),
        "chicle_get_w": (ctypes.c_int, [vp, vp]),
        "chicle_set_w": (ctypes.c_int, [vp, vp]),
        "chicle_get_delta_w": (ctypes.c_int, [vp, i32, vp]),
        "chicle_get_alpha": (ctypes.c_int, [vp, i32, vp]),
        "chicle_set_alpha": (ctypes.c_int, [vp, i32, vp]),
        "chicle_get_assignment": (ctypes.c_int, [vp, vp, ctypes.POINTER(i32)]),
        "chicle_debug_gram": (ctypes.c_int, [vp, vp, vp, i64, ctypes.POINTER(i32)]),
        "chicle_sync": (ctypes.c_int, [vp]),
        "chicle_set_profiling": (ctypes.c_int, [vp, i32]),
        "chicle_last_kernel_ms": (ctypes.c_int, [vp, i32, ctypes.POINTER(ctypes.c_float)]),
        "chicle_last_error": (ctypes.c_char_p, [vp]),
        "chicle_destroy": (None, [vp]),
        "chicle_solver_ms": (ctypes.c_int, [vp, vp]),
        "chicle_projected_iteration_time": (dbl, [i32, i32, i32, dbl, i32]),
        "chicle_scale_out": (ctypes.c_int, [vp, i32, i32, i32, vp, vp]),
        "chicle_scale_in": (ctypes.c_int, [vp, i32, i32, i32, vp]),
        "chicle_rebalance": (ctypes.c_int, [vp, i32, i32, vp, i32, i32, vp, ctypes.POINTER(i32)]),
        "chicle_next_solver_count": (i32, [vp, i32, i32, i32, ctypes.c_double, i32, i32]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    _lib = L
    return L


def _host(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def balance(chunk_load: Sequence[int], K: int, speed_q: Optional[Sequence[int]] = None) -> np.ndarray:
    """chicle_balance: greedy chunk -> solver table (host only)."""
    L = load_library()
    load = _host(chunk_load, np.int64)
    sp = None if speed_q is None else _host(speed_q, np.int32)
    if sp is not None and sp.size != K:
        raise ChicleError(EINVAL, "one speed per solver")
    out = np.empty(load.size, dtype=np.int32)
    rc = L.chicle_balance(_ptr(load), load.size, K, _ptr(sp), _ptr(out))
    if rc != OK:
        raise ChicleError(rc, "chicle_balance")
    return out


def projected_iteration_time(K_tasks: Optional[int], nodes: int, n_slow: int = 0, slow_factor: float = 1.0,
                             base_nodes: int = 16) -> float:
    """chicle_projected_iteration_time; K_tasks None (or 0) selects uni-tasks."""
    L = load_library()
    t = L.chicle_projected_iteration_time(int(K_tasks or 0), int(nodes), int(n_slow), float(slow_factor),
                                          int(base_nodes))
    if t < 0:
        raise ChicleError(EINVAL, "chicle_projected_iteration_time")
    return t


def scale_out(table, K_old: int, K_new: int, draw) -> np.ndarray:
    """chicle_scale_out: new solvers receive randomly picked chunks of every old solver (host only)."""
    L = load_library()
    t = _host(table, np.int32)
    dr = _host(draw, np.uint32)
    if dr.size != t.size:
        raise ChicleError(EINVAL, "one draw per chunk")
    out = np.empty_like(t)
    rc = L.chicle_scale_out(_ptr(t), t.size, K_old, K_new, _ptr(dr), _ptr(out))
    if rc != OK:
        raise ChicleError(rc, "chicle_scale_out")
    return out


def scale_in(table, K_old: int, K_new: int) -> np.ndarray:
    """chicle_scale_in: chunks of the freed solvers go round robin to the remaining ones (host only)."""
    L = load_library()
    t = _host(table, np.int32)
    out = np.empty_like(t)
    rc = L.chicle_scale_in(_ptr(t), t.size, K_old, K_new, _ptr(out))
    if rc != OK:
        raise ChicleError(rc, "chicle_scale_in")
    return out


def rebalance(chunk_load, K: int, unit_time, table, max_moves: int):
    """chicle_rebalance: returns (new table, chunks moved).  unit_time: iterations x K (host only)."""
    L = load_library()
    load = _host(chunk_load, np.int64)
    ut = _host(np.atleast_2d(unit_time), np.float64)
    t = _host(table, np.int32).copy()
    if ut.shape[1] != K or t.size != load.size:
        raise ChicleError(EINVAL, "unit_time is iterations x K, one table entry per chunk")
    moved = ctypes.c_int32(0)
    rc = L.chicle_rebalance(_ptr(load), load.size, K, _ptr(ut), ut.shape[0], int(max_moves), _ptr(t),
                            ctypes.byref(moved))
    if rc != OK:
        raise ChicleError(rc, "chicle_rebalance")
    return t, int(moved.value)


def next_solver_count(gaps, K: int, K_min: int, stall_ratio: float, patience: int, since_change: int) -> int:
    """chicle_next_solver_count: the number of solvers for the next round (host only)."""
    L = load_library()
    g = _host(gaps, np.float64)
    rc = L.chicle_next_solver_count(_ptr(g), g.size, int(K), int(K_min), float(stall_ratio), int(patience),
                                    int(since_change))
    if rc < 0:
        raise ChicleError(EINVAL, "chicle_next_solver_count")
    return int(rc)


class ChicleRound:
    """One context of the library.  Methods mirror the C entry points one to one."""

    def __init__(self, loss: str, n_total: int, d: int, lam: float, n_chunks: int, max_solvers: int,
                 dense: bool, total_entries: int, device: str = "cuda:0"):
        import torch
        self._L = load_library()
        if not torch.cuda.is_available():
            raise ChicleError(EDEVICE, "no GPU visible; this library has no CPU path")
        self._torch = torch
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        nbytes = self._L.chicle_arena_bytes(n_total, total_entries, d, n_chunks, max_solvers, int(dense))
        if nbytes == 0:
            raise ChicleError(EINVAL, "bad sizes")
        self.arena = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.stream = torch.cuda.current_stream(self.device)
        h = ctypes.c_void_p()
        rc = self._L.chicle_create(ctypes.byref(h), LOSS[loss], n_total, d, float(lam), n_chunks,
                                   max_solvers, int(dense), total_entries,
                                   ctypes.c_void_p(self.arena.data_ptr()), nbytes,
                                   ctypes.c_void_p(self.stream.cuda_stream))
        if rc != OK:
            raise ChicleError(rc, "chicle_create")
        self._h = h
        self.n_total, self.d, self.n_chunks, self.dense = n_total, d, n_chunks, dense
        self._chunk_rows = {}
        self.K = 0

    # -- helpers
    def _check(self, rc: int):
        if rc != OK:
            raise ChicleError(rc, self._L.chicle_last_error(self._h).decode())

    def close(self):
        if getattr(self, "_h", None) is not None:
            self._L.chicle_destroy(self._h)
            self._h = None
            self.arena = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- chunk store
    def load_chunk_csr(self, chunk_id, row_ptr, col, val, y, alpha0=None):
        rp, c, v, yy = _host(row_ptr, np.int32), _host(col, np.int32), _host(val, np.float32), _host(y, np.float32)
        a0 = None if alpha0 is None else _host(alpha0, np.float32)
        n_rows = rp.size - 1
        if c.size != v.size or (n_rows >= 0 and rp.size and c.size != int(rp[-1])) or yy.size != n_rows \
                or (a0 is not None and a0.size != n_rows):
            raise ChicleError(EINVAL, "array lengths disagree")
        self._check(self._L.chicle_load_chunk_csr(self._h, chunk_id, n_rows, _ptr(rp), _ptr(c), _ptr(v), _ptr(yy), _ptr(a0)))
        self._chunk_rows[chunk_id] = n_rows

    def load_chunk_dense(self, chunk_id, X, y, alpha0=None):
        Xc, yy = _host(X, np.float32), _host(y, np.float32)
        a0 = None if alpha0 is None else _host(alpha0, np.float32)
        if Xc.ndim != 2 or Xc.shape[1] != self.d or yy.size != Xc.shape[0] or (a0 is not None and a0.size != Xc.shape[0]):
            raise ChicleError(EINVAL, "array shapes disagree")
        self._check(self._L.chicle_load_chunk_dense(self._h, chunk_id, Xc.shape[0], _ptr(Xc), _ptr(yy), _ptr(a0)))
        self._chunk_rows[chunk_id] = Xc.shape[0]

    # -- scheduler
    def assign(self, K: int, chunk_to_solver):
        t = _host(chunk_to_solver, np.int32)
        if t.size != self.n_chunks:
            raise ChicleError(EINVAL, "table needs one entry per chunk")
        self._check(self._L.chicle_assign(self._h, K, _ptr(t)))
        self.K = K

    def solver_rows(self) -> np.ndarray:
        out = np.zeros(self.K, dtype=np.int64)
        self._check(self._L.chicle_solver_rows(self._h, _ptr(out)))
        return out

    def solver_ms(self) -> np.ndarray:
        out = np.empty(self.K, dtype=np.float32)
        self._check(self._L.chicle_solver_ms(self._h, _ptr(out)))
        return out

    def get_assignment(self):
        out = np.zeros(self.n_chunks, dtype=np.int32)
        k = ctypes.c_int32()
        self._check(self._L.chicle_get_assignment(self._h, _ptr(out), ctypes.byref(k)))
        return out, k.value

    def set_solver(self, kind: str):
        self._check(self._L.chicle_set_solver(self._h, SOLVER[kind]))

    def set_l1(self, l1: float):
        """Elastic net: regulariser lambda (|w|^2 / 2 + l1 |w|_1); 0 is the plain L2 round."""
        self._check(self._L.chicle_set_l1(self._h, float(l1)))

    # -- the round
    def upload_perm(self, perms):
        """Concatenate per-solver orders and put them in HBM (a torch int32 tensor)."""
        flat = np.concatenate([_host(p, np.int32) for p in perms]) if len(perms) else np.empty(0, np.int32)
        if flat.size != self.n_total:
            raise ChicleError(EINVAL, "orders must cover every row once")
        return self._torch.from_numpy(flat).to(self.device)

    def _perm_ptr(self, t):
        if t.dtype != self._torch.int32 or not t.is_cuda or not t.is_contiguous() or t.numel() != self.n_total:
            raise ChicleError(EINVAL, "perm must be a contiguous int32 device tensor of n_total entries")
        return ctypes.c_void_p(t.data_ptr())

    def local_epoch(self, perm_device):
        self._check(self._L.chicle_local_epoch(self._h, self._perm_ptr(perm_device)))

    def local_epoch_ahead(self, perm_device, perm_next_device=None):
        """perm_device None: run with the orders the previous call announced (the library kept a copy)."""
        cur = None if perm_device is None else self._perm_ptr(perm_device)
        nxt = None if perm_next_device is None else self._perm_ptr(perm_next_device)
        self._check(self._L.chicle_local_epoch_ahead(self._h, cur, nxt))

    def local_epoch_host_perm(self, perm_host):
        flat = _host(perm_host, np.int32)
        if flat.size != self.n_total:
            raise ChicleError(EINVAL, "orders must cover every row once")
        self._check(self._L.chicle_local_epoch_host_perm(self._h, _ptr(flat)))

    def aggregate(self):
        self._check(self._L.chicle_aggregate(self._h))

    def gap(self):
        p, dd, g = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
        self._check(self._L.chicle_gap(self._h, ctypes.byref(p), ctypes.byref(dd), ctypes.byref(g)))
        return p.value, dd.value, g.value

    def gap_noalloc(self):
        p, dd, g = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
        self._check(self._L.chicle_gap_noalloc(self._h, ctypes.byref(p), ctypes.byref(dd), ctypes.byref(g)))
        return p.value, dd.value, g.value

    # -- state access
    def get_w(self) -> np.ndarray:
        out = np.empty(self.d, dtype=np.float32)
        self._check(self._L.chicle_get_w(self._h, _ptr(out)))
        return out

    def set_w(self, w):
        a = _host(w, np.float32)
        if a.size != self.d:
            raise ChicleError(EINVAL, "w needs d entries")
        self._check(self._L.chicle_set_w(self._h, _ptr(a)))

    def get_delta_w(self, solver: int) -> np.ndarray:
        out = np.empty(self.d, dtype=np.float32)
        self._check(self._L.chicle_get_delta_w(self._h, solver, _ptr(out)))
        return out

    def get_alpha(self, chunk_id: int) -> np.ndarray:
        if chunk_id not in self._chunk_rows:
            raise ChicleError(EINVAL, "chunk not loaded")
        out = np.empty(self._chunk_rows[chunk_id], dtype=np.float32)
        self._check(self._L.chicle_get_alpha(self._h, chunk_id, _ptr(out)))
        return out

    def set_alpha(self, chunk_id: int, alpha):
        a = _host(alpha, np.float32)
        if chunk_id not in self._chunk_rows or a.size != self._chunk_rows[chunk_id]:
            raise ChicleError(EINVAL, "alpha needs one entry per row of the chunk")
        self._check(self._L.chicle_set_alpha(self._h, chunk_id, _ptr(a)))

    def debug_gram(self, perm_device) -> np.ndarray:
        """Tiles of the batched solver's Gram kernel, shape [n_tiles, 128, 64]."""
        n = ctypes.c_int32()
        ptr = ctypes.c_void_p(perm_device.data_ptr())
        self._check(self._L.chicle_debug_gram(self._h, ptr, None, 0, ctypes.byref(n)))
        out = np.empty((n.value, 128, 64), dtype=np.float32)
        self._check(self._L.chicle_debug_gram(self._h, ptr, _ptr(out), out.size, ctypes.byref(n)))
        return out

    def sync(self):
        self._check(self._L.chicle_sync(self._h))

    def set_profiling(self, on: bool):
        self._check(self._L.chicle_set_profiling(self._h, int(on)))

    def last_kernel_ms(self, segment: str) -> float:
        ms = ctypes.c_float()
        self._check(self._L.chicle_last_kernel_ms(self._h, SEGMENT[segment], ctypes.byref(ms)))
        return ms.value

    # -- convenience: marshal a whole generated problem through load_chunk_*
    def load_problem(self, p):
        for c in range(p.n_chunks):
            if p.dense:
                X, y = p.chunk_dense(c)
                self.load_chunk_dense(c, X, y)
            else:
                rp, col, val, y = p.chunk_csr(c)
                self.load_chunk_csr(c, rp, col, val, y)

    @classmethod
    def from_problem(cls, p, max_solvers: int, device: str = "cuda:0"):
        ctx = cls(p.loss, p.n, p.d, p.lam, p.n_chunks, max_solvers, p.dense, p.nnz, device=device)
        ctx.load_problem(p)
        return ctx
