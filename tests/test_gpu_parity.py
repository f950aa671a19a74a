"""GPU parity: the HIP library against the CPU oracle, element by element, through the C ABI.

Mini sizes compare every solver's Delta w each round; full sizes (the sizes the benchmark times)
compare the summed update every round, every solver's update in the first, the middle and the last
round, and a sample of solvers in the others.  Integer work (the chunk -> solver table, rows per
solver) must be bit-exact."""
import sys

import numpy as np
import pytest

from harness import cached_problem, run_lockstep, TOL_DW, TOL_GAP
from workloads import get_config, make_problem, round_permutations

pytestmark = pytest.mark.gpu


def _log(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def mods(oracle_mod):
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_1909_04885_amd as binding
    return oracle_mod, binding


MINI_CASES = [("dense_hinge", "rowwise", False), ("dense_ridge", "rowwise", False),
              ("sparse_zipf", "rowwise", False), ("sparse_longrow", "rowwise", False),
              ("elastic", "rowwise", False), ("sparse_zipf", "batched", False),
              ("elastic", "batched", False), ("sparse_zipf", "batched", True), ("elastic", "batched", True),
              ("dense_ridge", "auto", True), ("dense_hinge", "auto", False), ("dense_hinge", "batched", False),
              # long rows with every solver kept on one compute unit ("rowwise" spreads it over several there)
              ("sparse_longrow", "rowwise_one_cu", False),
              # the batched solver with every solver kept on one compute unit
              ("sparse_zipf", "batched_one_cu", False), ("elastic", "batched_one_cu", True)]


@pytest.mark.parametrize("name,solver,ahead", MINI_CASES)
def test_mini_all_solvers_every_round(mods, name, solver, ahead):
    oracle_mod, binding = mods
    cfg, p = cached_problem(name, "mini")
    print("\ncase", name, "mini", solver, "ahead" if ahead else "", "n=%d d=%d" % (p.n, p.d), flush=True)
    run_lockstep(cfg, p, oracle_mod, binding, solver=solver, check_alpha_every=1, log=_log, ahead=ahead)


@pytest.mark.parametrize("name,size,solver,ahead", [
    ("dense_hinge", "mini", "auto", False), ("sparse_zipf", "mini", "rowwise", False),
    ("sparse_zipf", "mini", "batched", False), ("sparse_longrow", "mini", "auto", False),
    ("elastic", "mini", "rowwise", False), ("elastic", "mini", "batched", True),
    ("dense_hinge", "full", "auto", False)])
def test_logistic_loss_every_round(mods, name, size, solver, ahead):
    """The same data and schedules with the logistic loss (labels are +-1 already): the library's fp32
    root search, in the row-wise solvers and inside the blocked recurrences, against the oracle's
    bisection in fp64."""
    import dataclasses
    oracle_mod, binding = mods
    cfg, p = cached_problem(name, size)
    p = dataclasses.replace(p, loss="logistic")
    print("\ncase", name, size, solver, "logistic n=%d d=%d" % (p.n, p.d), flush=True)
    rec = run_lockstep(cfg, p, oracle_mod, binding, solver=solver, check_alpha_every=1, log=_log, ahead=ahead)
    assert abs(rec[0]["P_ref"] - rec[0]["P_gpu"]) < 1e-5 and rec[-1]["gap_ref"] < np.log(2.0)


def test_logistic_full_sparse_zipf(mods):
    """The benchmark's sizes with the logistic loss (blocked solver, tiles of the next pass prepared ahead)."""
    import dataclasses
    oracle_mod, binding = mods
    cfg, p = cached_problem("sparse_zipf", "full")
    p = dataclasses.replace(p, loss="logistic")
    print("\ncase sparse_zipf full logistic n=%d d=%d nnz=%d" % (p.n, p.d, p.nnz), flush=True)
    run_lockstep(cfg, p, oracle_mod, binding, rounds=5, sample_solvers=[0, 13, 31], log=_log, ahead=True)


@pytest.mark.parametrize("name", ["dense_hinge", "dense_ridge"])
def test_full_dense(mods, name):
    oracle_mod, binding = mods
    cfg, p = cached_problem(name, "full")
    print("\ncase", name, "full n=%d d=%d" % (p.n, p.d), flush=True)
    run_lockstep(cfg, p, oracle_mod, binding, check_alpha_every=10, log=_log)


@pytest.mark.parametrize("name", ["sparse_zipf", "elastic"])
def test_full_sparse_zipf(mods, name):
    oracle_mod, binding = mods
    cfg, p = cached_problem("sparse_zipf", "full")
    cfg = get_config(name, "full")
    print("\ncase", name, "full n=%d d=%d nnz=%d" % (p.n, p.d, p.nnz), flush=True)
    run_lockstep(cfg, p, oracle_mod, binding, sample_solvers=[0, 3, 7, 31], log=_log, ahead=True)


def test_full_sparse_zipf_elastic_net(mods):
    """The benchmark's sizes with the L1 term (over a third of the shared vector at exactly zero after five rounds):
    compact merge in solver slices, gap with the L1 term, tiles prepared ahead."""
    oracle_mod, binding = mods
    cfg, p = cached_problem("sparse_zipf", "full")
    print("\ncase sparse_zipf full l1=0.005 n=%d d=%d nnz=%d" % (p.n, p.d, p.nnz), flush=True)
    rec = run_lockstep(cfg, p, oracle_mod, binding, rounds=5, sample_solvers=[0, 13, 31], log=_log, ahead=True, l1=0.005)
    assert 0.05 < rec[-1]["w_zero"] < 0.95
    for r in rec:
        assert abs(r["P_gpu"] - r["P_ref"]) <= 1e-5 * abs(r["P_ref"]) + 1e-7


def test_full_sparse_longrow(mods):
    oracle_mod, binding = mods
    cfg, p = cached_problem("sparse_longrow", "full")
    print("\ncase sparse_longrow full n=%d d=%d nnz=%d" % (p.n, p.d, p.nnz), flush=True)
    run_lockstep(cfg, p, oracle_mod, binding, sample_solvers=[0, 17, 63], log=_log)


@pytest.mark.parametrize("name,loss,solver,ahead,l1", [
    ("dense_hinge", "hinge", "auto", False, 0.5), ("dense_ridge", "squared", "auto", True, 1.5),
    ("dense_hinge", "logistic", "auto", False, 0.5),
    ("sparse_zipf", "hinge", "rowwise", False, 0.1), ("sparse_zipf", "hinge", "batched", True, 0.1),
    ("sparse_zipf", "squared", "batched", False, 0.1), ("sparse_zipf", "logistic", "batched", True, 0.15),
    ("sparse_zipf", "squared", "batched_one_cu", False, 0.1),
    ("sparse_longrow", "hinge", "rowwise", False, 0.02), ("sparse_longrow", "logistic", "rowwise_one_cu", False, 0.02),
    ("elastic", "hinge", "batched", True, 0.1)])
def test_elastic_net_every_round(mods, name, loss, solver, ahead, l1):
    """Regulariser lambda (|w|^2 / 2 + l1 |w|_1): the merged updates live in the dual image, every solver starts
    from its soft-thresholded image, and primal and dual value carry the L1 term and the conjugate; every
    kernel family that reads or writes the shared vector, each loss, with l1 chosen so that a good part of
    the coordinates (and not all) sit at exactly zero."""
    import dataclasses
    oracle_mod, binding = mods
    cfg, p = cached_problem(name, "mini")
    p = dataclasses.replace(p, loss=loss)
    print("\ncase", name, "mini", loss, solver, "l1=%g n=%d d=%d" % (l1, p.n, p.d), flush=True)
    rec = run_lockstep(cfg, p, oracle_mod, binding, solver=solver, check_alpha_every=1, log=_log, ahead=ahead, l1=l1)
    assert 0.1 < rec[-1]["w_zero"] < 0.9
    for r in rec:
        assert abs(r["P_gpu"] - r["P_ref"]) <= 1e-5 * abs(r["P_ref"]) + 1e-7
        assert abs(r["D_gpu"] - r["D_ref"]) <= 1e-5 * abs(r["D_ref"]) + 1e-6


def test_elastic_net_setter_contract(mods):
    """l1 is refused when negative and between a local pass and its merge; with l1 > 0 the shared vector cannot
    be set from outside; changing l1 in READY re-thresholds the shared vector."""
    oracle_mod, binding = mods
    p = _tiny(binding, loss="squared")
    g = binding.ChicleRound.from_problem(p, max_solvers=3)
    with pytest.raises(binding.ChicleError):
        g.set_l1(-1.0)
    g.set_l1(0.05)                                              # legal before the first assignment too
    g.assign(3, np.array([0, 1, 2, 0, 1], dtype=np.int32))
    perms = round_permutations(3, 0, [int(x) for x in g.solver_rows()])
    g.local_epoch_host_perm(np.concatenate(perms))
    with pytest.raises(binding.ChicleError):
        g.set_l1(0.1)
    g.aggregate()
    w_a = g.get_w()
    with pytest.raises(binding.ChicleError):
        g.set_w(np.zeros(p.d, dtype=np.float32))
    g.set_l1(0.0)
    v = g.get_w().astype(np.float64)
    assert np.allclose(w_a, np.sign(v) * np.maximum(np.abs(v) - 0.05, 0.0), atol=1e-6)
    g.close()


def test_batched_solver_with_long_chunk_lists(mods):
    """One solver that owns 235 chunks, then three: the batched solver stages a solver's chunk descriptors in
    LDS, where they take the place of columns of the private vector; no list length sends the pass to the
    row-wise solver."""
    oracle_mod, binding = mods
    cfg = get_config("sparse_zipf", "mini")
    cfg.update(chunk_rows=128, K=1, schedule=[(0, 1), (2, 3)], rounds=4)
    p = make_problem(cfg)
    assert p.n_chunks > 200
    print("\ncase sparse_zipf mini, %d chunks, K = 1 then 3, batched" % p.n_chunks, flush=True)
    run_lockstep(cfg, p, oracle_mod, binding, solver="batched", check_alpha_every=1, log=_log)


def test_gram_tiles_match_their_definition(mods):
    """The batched solver's Gram kernel against x_i . x_j computed with numpy in double."""
    import scipy.sparse as sp
    oracle_mod, binding = mods
    cfg, p = cached_problem("sparse_zipf", "mini")
    K = 3
    g = binding.ChicleRound.from_problem(p, max_solvers=K)
    table = binding.balance(p.chunk_nnz(), K)
    g.assign(K, table)
    rows = g.solver_rows()
    perms = round_permutations(3, 0, rows)
    tiles = g.debug_gram(g.upload_perm(perms))
    X = sp.csr_matrix((p.val.astype(np.float64), p.col, p.row_ptr), shape=(p.n, p.d))
    q = np.asarray(X.multiply(X).sum(axis=1)).ravel()
    y = p.y.astype(np.float64)
    t = 0
    for k in range(K):
        own = np.concatenate([np.arange(*p.chunk_rows(c)) for c in np.nonzero(table == k)[0]])
        order = own[perms[k]]
        nb = (order.size + 63) // 64
        for b in range(nb):
            cur = order[b * 64:(b + 1) * 64]
            prev = order[(b - 1) * 64:b * 64] if b > 0 else np.empty(0, dtype=np.int64)
            want = np.zeros((128, 64))
            Xc = X[cur]
            if prev.size:
                G = (X[prev] @ Xc.T).toarray()                      # [prev j, cur i]
                want[:prev.size, :cur.size] = -G * y[prev][:, None] * y[cur][None, :] / q[cur][None, :]
            G = (Xc @ Xc.T).toarray()
            T = -G * y[cur][:, None] * y[cur][None, :] / q[cur][None, :]
            T = np.triu(T, k=1)                                     # keep [j, i] with j < i
            want[64:64 + cur.size, :cur.size] = T
            got = tiles[t]
            assert np.max(np.abs(got - want)) <= 2e-6 * max(1.0, np.max(np.abs(want))), (k, b)
            t += 1
    assert t == tiles.shape[0]
    g.close()


def test_thinly_occupied_private_vectors(mods):
    """Few rows over many columns: every solver touches a few of every hundred columns, the case in which the
    merge picks a solver's entries straight from its compact vector (here with the solvers divided over
    slices; the long-row benchmark size runs it unsliced)."""
    oracle_mod, binding = mods
    from workloads.generate import Problem
    g = np.random.default_rng(11)
    n, d, per_row, K = 600, 300000, 100, 4
    col = np.sort(np.stack([g.choice(d, per_row, replace=False) for _ in range(n)]), axis=1).astype(np.int32).ravel()
    val = (g.standard_normal(n * per_row) / np.sqrt(per_row)).astype(np.float32)
    y = np.where(g.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    bounds = np.array(list(range(0, n, 128)) + [n], dtype=np.int64)
    p = Problem("thin", "hinge", n, d, 1e-3, y, bounds, row_ptr=np.arange(n + 1, dtype=np.int64) * per_row, col=col, val=val)
    cfg = dict(seed=4, rounds=4, schedule=[(0, K)], K=K, speeds=None)
    print("\ncase thin n=%d d=%d K=%d" % (n, d, K), flush=True)
    run_lockstep(cfg, p, oracle_mod, binding, solver="auto", check_alpha_every=1, log=_log)


@pytest.mark.parametrize("loss,l1", [("hinge", 0.0), ("squared", 0.0), ("logistic", 0.0), ("squared", 0.002)])
def test_long_rows_over_a_shared_vector_of_many_slices(mods, loss, l1):
    """Rows of hundreds of entries over two million columns: the gap's row pass cuts the shared vector into
    slices (8 in float, 16 in double) and sums a row's dot product from its runs; rows of very different
    lengths, an empty row, a ragged last chunk."""
    oracle_mod, binding = mods
    from workloads.generate import Problem
    g = np.random.default_rng(17)
    n, d, K = 330, 2_000_000, 3
    lens = np.clip(np.round(g.lognormal(np.log(300), 0.7, n)), 1, 4000).astype(np.int64)
    lens[5] = 0
    rp = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(lens, out=rp[1:])
    col = np.concatenate([np.sort(g.choice(d, int(m), replace=False)) for m in lens]).astype(np.int32)
    val = np.concatenate([g.choice([-1.0, 1.0], int(m)) / np.sqrt(max(int(m), 1)) for m in lens]).astype(np.float32)
    y = np.where(g.random(n) < 0.5, 1.0, -1.0).astype(np.float32) if loss != "squared" else g.standard_normal(n).astype(np.float32)
    bounds = np.array(list(range(0, n, 100)) + [n], dtype=np.int64)
    p = Problem("slices", loss, n, d, 1e-3, y, bounds, row_ptr=rp, col=col, val=val)
    cfg = dict(seed=6, rounds=4, schedule=[(0, K)], K=K)
    print("\ncase slices %s l1=%g n=%d d=%d nnz=%d" % (loss, l1, n, d, rp[-1]), flush=True)
    run_lockstep(cfg, p, oracle_mod, binding, solver="auto", check_alpha_every=1, log=_log, l1=l1)


# ----------------------------------------------------------------------------- edges and contract
def _tiny(binding, loss="hinge", dense=False, n=300, d=50, chunk=64, K=3, seed=5):
    g = np.random.default_rng(seed)
    X = g.standard_normal((n, d)).astype(np.float32)
    X[g.random(X.shape) < 0.7] = 0
    X[3] = 0                       # an empty row
    y = np.where(g.random(n) < 0.5, 1.0, -1.0).astype(np.float32) if loss == "hinge" else g.standard_normal(n).astype(np.float32)
    bounds = np.array(list(range(0, n, chunk)) + [n], dtype=np.int64)
    from workloads.generate import Problem
    if dense:
        return Problem("tiny", loss, n, d, 0.01, y, bounds, X=X)
    mask = X != 0
    rp = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(mask.sum(1), out=rp[1:])
    return Problem("tiny", loss, n, d, 0.01, y, bounds, row_ptr=rp, col=np.nonzero(mask)[1].astype(np.int32), val=X[mask])


@pytest.mark.parametrize("loss", ["hinge", "squared"])
@pytest.mark.parametrize("dense", [False, True])
def test_tiny_ragged_with_empty_row_and_idle_solver(mods, loss, dense):
    oracle_mod, binding = mods
    p = _tiny(binding, loss, dense)
    o = oracle_mod.OracleCoCoA.from_problem(p)
    g = binding.ChicleRound.from_problem(p, max_solvers=6)
    table = np.array([0, 2, 2, 4, 0], dtype=np.int32)          # solvers 1, 3, 5 own nothing
    o.assign(6, table)
    g.assign(6, table)
    P, D, G = g.gap()
    Po, Do, Go, _ = o.gap()
    assert abs(G - Go) <= 1e-6 * abs(Go)
    for r in range(5):
        perms = round_permutations(9, r, o.rows_per_solver())
        dws = o.local_epoch(perms)
        g.local_epoch_host_perm(np.concatenate(perms))
        for k in range(6):
            got = g.get_delta_w(k)
            if o.rows_of[k].size == 0:
                assert not got.any()
            else:
                assert np.linalg.norm(got - dws[k]) <= TOL_DW * np.linalg.norm(dws[k])
        o.aggregate()
        g.aggregate()
        assert abs(g.gap()[2] - o.gap()[2]) <= TOL_GAP * abs(o.gap()[2])
    r0, r1 = p.chunk_rows(0)
    assert g.get_alpha(0)[3] == 0.0
    g.close()


@pytest.mark.parametrize("loss", ["hinge", "squared", "logistic"])
@pytest.mark.parametrize("d,dense,density", [(48, True, 1.0), (49, True, 1.0), (320, True, 1.0), (321, True, 1.0),
                                             (200, False, 0.2), (200, False, 0.3), (30, False, 0.9)])
def test_shapes_on_both_sides_of_every_solver_choice(mods, loss, d, dense, density):
    """Row widths at the borders between the solvers the library chooses from (dense rows stored with
    column ids up to 48 columns, the dense blocked solver up to 320, the sparse batched solver up to 48
    entries per row), each against the oracle for a few rounds with ragged chunks."""
    oracle_mod, binding = mods
    from workloads.generate import Problem
    g = np.random.default_rng(d + 7 * dense)
    n, chunk, K = 333, 70, 3
    X = g.standard_normal((n, d)).astype(np.float32)
    if density < 1.0:
        X[g.random(X.shape) >= density] = 0
    X[5] = 0
    y = g.standard_normal(n).astype(np.float32) if loss == "squared" else np.where(g.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    bounds = np.array(list(range(0, n, chunk)) + [n], dtype=np.int64)
    if dense:
        p = Problem("shape", loss, n, d, 0.02, y, bounds, X=X)
    else:
        mask = X != 0
        rp = np.zeros(n + 1, dtype=np.int64)
        np.cumsum(mask.sum(1), out=rp[1:])
        p = Problem("shape", loss, n, d, 0.02, y, bounds, row_ptr=rp, col=np.nonzero(mask)[1].astype(np.int32), val=X[mask])
    print("\ncase shape d=%d dense=%s density=%.1f %s max row %d" %
          (d, dense, density, loss, int((X != 0).sum(1).max())), flush=True)
    cfg = {"seed": 3, "rounds": 4, "schedule": [(0, K)], "K": K}
    table = (np.arange(p.n_chunks) % K).astype(np.int32)
    run_lockstep(cfg, p, oracle_mod, binding, rounds=4, check_alpha_every=1, log=_log,
                 tables=lambda r, Kp, tp: (K, table, table.copy()) if r == 0 else None, max_solvers=K)


def test_ownership_contract_and_errors(mods):
    oracle_mod, binding = mods
    p = _tiny(binding)
    g = binding.ChicleRound(p.loss, p.n, p.d, p.lam, p.n_chunks, 4, False, p.nnz)
    E = binding.ChicleError
    rp, col, val, y = p.chunk_csr(0)
    with pytest.raises(E) as e:
        g.assign(2, np.zeros(p.n_chunks, dtype=np.int32))       # chunks missing
    assert e.value.code == -1
    bad = col.copy(); bad[0] = p.d
    with pytest.raises(E):
        g.load_chunk_csr(0, rp, bad, val, y)
    rp_bad = rp.copy(); rp_bad[2] = rp_bad[1] - 1 if rp_bad[1] > 0 else 0; rp_bad[1] = rp_bad[2] + 1
    with pytest.raises(E):
        g.load_chunk_csr(0, rp_bad, col, val, y)
    with pytest.raises(E):
        g.load_chunk_csr(0, rp, col, val, y * 0.5)               # hinge label must be +-1
    g.load_problem(p)
    with pytest.raises(E):
        g.load_chunk_csr(0, rp, col, val, y)                      # already loaded
    with pytest.raises(E):
        g.assign(5, np.zeros(p.n_chunks, dtype=np.int32))        # K above max_solvers
    with pytest.raises(E):
        g.assign(2, np.full(p.n_chunks, 2, dtype=np.int32))      # solver id out of range
    with pytest.raises(E) as e:
        g.gap()                                                   # nothing assigned yet
    assert e.value.code == -3
    g.assign(2, np.arange(p.n_chunks, dtype=np.int32) % 2)
    rows = g.solver_rows()
    perms = round_permutations(0, 0, rows)
    g.local_epoch_host_perm(np.concatenate(perms))
    for call in (lambda: g.assign(2, np.zeros(p.n_chunks, dtype=np.int32)),
                 lambda: g.local_epoch_host_perm(np.concatenate(perms)),
                 lambda: g.gap(), lambda: g.set_alpha(0, np.zeros(p.chunk_rows(0)[1], dtype=np.float32)),
                 lambda: g.set_w(np.zeros(p.d, dtype=np.float32))):
        with pytest.raises(E) as e:
            call()
        assert e.value.code == -3
    g.aggregate()
    with pytest.raises(E) as e:
        g.get_delta_w(0)
    assert e.value.code == -3
    # an out-of-range visiting-order entry is skipped and reported, not dereferenced
    badperm = np.concatenate(perms).copy()
    badperm[1] = 10**6
    g.local_epoch_host_perm(badperm)
    with pytest.raises(E) as e:
        g.sync()
    assert e.value.code == -4
    g.sync()                                                      # flag cleared
    g.aggregate()
    assert g.gap()[2] >= 0
    g.close()


def test_set_state_resumes_a_run(mods):
    """Uploading the oracle's (alpha, w) and continuing gives the oracle's next round."""
    oracle_mod, binding = mods
    cfg, p = cached_problem("sparse_zipf", "mini")
    o = oracle_mod.OracleCoCoA.from_problem(p)
    K = cfg["K"]
    table = oracle_mod.assign_greedy(p.chunk_nnz(), K)
    o.assign(K, table)
    for r in range(3):
        o.local_epoch(round_permutations(1, r, o.rows_per_solver()), keep_deltas=False)
        o.aggregate()
    g = binding.ChicleRound.from_problem(p, max_solvers=K)
    g.assign(K, table)
    for c in range(p.n_chunks):
        r0, r1 = p.chunk_rows(c)
        g.set_alpha(c, o.alpha[r0:r1])
    g.set_w(o.w)
    assert abs(g.gap()[2] - o.gap()[2]) <= 1e-5 * abs(o.gap()[2])
    perms = round_permutations(1, 3, o.rows_per_solver())
    dws = o.local_epoch(perms)
    g.local_epoch(g.upload_perm(perms))
    for k in range(K):
        assert np.linalg.norm(g.get_delta_w(k) - dws[k]) <= TOL_DW * np.linalg.norm(dws[k])
    g.close()


@pytest.mark.parametrize("loss", ["hinge", "squared", "logistic"])
@pytest.mark.parametrize("shared", [0, 40])
def test_mixed_row_lengths(mods, loss, shared):
    """Rows from empty to 9000 entries in one visiting order (the row-wise solver keeps a fixed number of a
    row's entries in registers and streams the rest), columns spread over 300 000, and `shared` columns that
    every row of more than 20 entries carries as well."""
    oracle_mod, binding = mods
    from workloads.generate import Problem
    g = np.random.default_rng(17 + shared)
    n, d, K = 230, 300000, 2
    lens = g.choice([0, 3, 17, 60, 300, 1000, 1500, 2500], size=n, p=[.03, .1, .1, .17, .2, .2, .1, .1])
    lens[[20, 21]] = [5000, 9000]
    lens[7] = 4096
    common = g.choice(d, size=shared, replace=False)
    cols, vals = [], []
    for L in lens:
        c = g.choice(d, size=int(L), replace=False)
        if L > 20 and shared:
            c = np.unique(np.concatenate([c[:int(L) - shared], common]))
        c.sort()
        v = g.standard_normal(c.size)
        cols.append(c.astype(np.int32))
        vals.append((v / max(np.linalg.norm(v), 1e-30)).astype(np.float32))
    rp = np.zeros(n + 1, dtype=np.int64)
    np.cumsum([c.size for c in cols], out=rp[1:])
    y = g.standard_normal(n).astype(np.float32) if loss == "squared" else np.where(g.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    bounds = np.array([0, 50, 51, 120, 200, n], dtype=np.int64)
    p = Problem("mixed", loss, n, d, 0.02, y, bounds, row_ptr=rp, col=np.concatenate(cols), val=np.concatenate(vals))
    print("\ncase mixed row lengths %s shared=%d entries=%d" % (loss, shared, int(rp[-1])), flush=True)
    cfg = {"seed": 5, "rounds": 4, "schedule": [(0, K)], "K": K}
    table = (np.arange(p.n_chunks) % K).astype(np.int32)
    run_lockstep(cfg, p, oracle_mod, binding, rounds=4, check_alpha_every=1, log=_log,
                 tables=lambda r, Kp, tp: (K, table, table.copy()) if r == 0 else None, max_solvers=K)
