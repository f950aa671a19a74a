"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, and its pure-host
entry points behave.  No compute call is made here."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_1909_04885_amd as m
    return m.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "chicle_round.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(chicle_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    from paper_1909_04885_amd.binding import EXPORTS
    names = declared_symbols()
    assert len(names) >= 20
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(EXPORTS) == names          # the binding covers the whole header


def test_balance_matches_oracle_bit_exact(lib, oracle_mod):
    import paper_1909_04885_amd as m
    g = np.random.default_rng(1)
    for trial in range(60):
        n = int(g.integers(1, 200))
        K = int(g.integers(1, 40))
        load = g.integers(0, 1000, size=n) if trial % 2 else g.integers(5, 8, size=n)
        speed = None if trial % 3 == 0 else [int(x) for x in g.integers(1, 5, size=K)]
        assert np.array_equal(m.balance(load, K, speed), oracle_mod.assign_greedy(load, K, speed))
    big = np.array([2**61, 2**61 - 1, 2**60, 7], dtype=np.int64)
    assert np.array_equal(m.balance(big, 3, [3, 2, 1]), oracle_mod.assign_greedy(big, 3, [3, 2, 1]))


def test_balance_on_workload_shapes(lib, oracle_mod):
    import paper_1909_04885_amd as m
    from workloads import get_config, make_problem
    from workloads.configs import speeds_for
    cfg = get_config("elastic", "mini")
    p = make_problem(cfg)
    for _, K in cfg["schedule"]:
        sp = speeds_for(cfg, K)
        t = m.balance(p.chunk_nnz(), K, sp)
        assert np.array_equal(t, oracle_mod.assign_greedy(p.chunk_nnz(), K, sp))
        loads = np.bincount(t, weights=p.chunk_nnz(), minlength=K)
        fast, slow = loads[0::2].mean(), loads[1::2].mean() if K > 1 else loads.mean()
        if K >= 4:
            assert 1.3 < fast / slow < 3.0    # fast solvers (weight 2) carry about twice the load


def test_balance_rejects_bad_input(lib):
    out = np.zeros(3, dtype=np.int32)
    load = np.array([1, 2, 3], dtype=np.int64)
    p = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    assert lib.chicle_balance(p(load), 3, 0, None, p(out)) == -1
    assert lib.chicle_balance(None, 3, 2, None, p(out)) == -1
    bad = np.array([1, 0], dtype=np.int32)
    assert lib.chicle_balance(p(load), 3, 2, p(bad), p(out)) == -1
    neg = np.array([1, -2, 3], dtype=np.int64)
    assert lib.chicle_balance(p(neg), 3, 2, None, p(out)) == -1


def test_arena_bytes_and_create_argument_checks(lib):
    assert lib.chicle_arena_bytes(0, 10, 4, 1, 1, 0) == 0
    assert lib.chicle_arena_bytes(10, 10, 0, 1, 1, 0) == 0
    small = lib.chicle_arena_bytes(1000, 40000, 500, 4, 2, 0)
    bigger = lib.chicle_arena_bytes(1000, 40000, 500, 4, 8, 0)
    assert 0 < small < bigger
    assert small >= 40000 * 8 + 1000 * 16 + 500 * 4 * 4
    h = ctypes.c_void_p()
    # null arena, bad loss, non-positive lambda: rejected before any device call
    assert lib.chicle_create(ctypes.byref(h), 0, 10, 4, 0.1, 1, 1, 0, 10, None, 1 << 20, None) == -1
    assert lib.chicle_create(ctypes.byref(h), 7, 10, 4, 0.1, 1, 1, 0, 10, ctypes.c_void_p(256), 1 << 20, None) == -1
    assert lib.chicle_create(ctypes.byref(h), 0, 10, 4, 0.0, 1, 1, 0, 10, ctypes.c_void_p(256), 1 << 20, None) == -1
    assert lib.chicle_create(ctypes.byref(h), 0, 10, 4, 0.1, 1, 1, 0, 10, ctypes.c_void_p(256), 16, None) == -2
    # the logistic loss is a valid loss id: with too small an arena it gets as far as the size check
    assert lib.chicle_create(ctypes.byref(h), 2, 10, 4, 0.1, 1, 1, 0, 10, ctypes.c_void_p(256), 16, None) == -2
    assert lib.chicle_create(ctypes.byref(h), 3, 10, 4, 0.1, 1, 1, 0, 10, ctypes.c_void_p(256), 16, None) == -1
    assert h.value is None
    assert lib.chicle_last_error(None) == b"null context"
    for fn in ("chicle_aggregate", "chicle_sync"):
        assert getattr(lib, fn)(None) == -1


def test_product_path_has_no_cpu_fallback():
    """Nothing in the package imports or mentions the oracle, and the binding refuses to run without a GPU."""
    pkg = os.path.join(ROOT, "paper_1909_04885_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower() or f == "binding.py" and False, f
    import torch
    if not torch.cuda.is_available():
        import paper_1909_04885_amd as m
        with pytest.raises(m.ChicleError):
            m.ChicleRound("hinge", 10, 4, 0.1, 1, 1, True, 40)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_stored_traffic_is_tied_to_the_kernel_sources(tmp_path, monkeypatch):
    from paper_1909_04885_amd import record_traffic as rt
    rec = {"workload": "w/full", "kernels": {"a": 2.0, "b": 3.0}, "local_pass_bytes": 5.0,
           "source_sha256": rt.source_hash()}
    f = tmp_path / "t.json"
    monkeypatch.setattr(rt, "TRAFFIC_FILE", str(f))
    assert rt.stored_traffic("w/full") is None                 # no record
    f.write_text(__import__("json").dumps(rec))
    assert rt.stored_traffic("w/full") == {"kernels": {"a": 2.0, "b": 3.0}, "local_pass_bytes": 5.0}
    assert rt.stored_traffic("other/full") is None
    rec["source_sha256"] = "0" * 64                             # measured on other sources
    f.write_text(__import__("json").dumps(rec))
    assert rt.stored_traffic("w/full") is None
