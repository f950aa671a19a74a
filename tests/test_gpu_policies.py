"""GPU parity of runs whose chunk tables come from the scheduling policies of Section 4.5: the
library's tables must equal the oracle's bit for bit at every step, and the rounds run under them
must stay within the tolerances of every other parity test."""
import numpy as np
import pytest

from harness import cached_problem, run_lockstep
from oracle import policies as opol
from workloads import chunk_draws, round_permutations

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mods(oracle_mod):
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_1909_04885_amd as binding
    return oracle_mod, binding


def _policy_schedule(cfg, p, binding):
    """4 solvers; grow to 9 before round 2 (random picks); shift load for three rounds from solvers
    that are given as twice as slow; shrink to 3 before round 6 (round robin)."""
    loads = p.chunk_nnz()
    n = p.n_chunks
    start = np.arange(n, dtype=np.int32) % 4

    def rates(K):
        return np.array([[1e-7 * (2.0 if k % 2 else 1.0) for k in range(K)]] * 3)

    def tables(r, K_prev, t_prev):
        if r == 0:
            return 4, start, start.copy()
        if r == 2:
            dr = chunk_draws(cfg["seed"], r, n)
            return 9, opol.scale_out(t_prev.tolist(), 4, 9, dr.tolist()), binding.scale_out(t_prev, 4, 9, dr)
        if r in (3, 4, 5):
            ref, m_ref = opol.rebalance(loads.tolist(), 9, rates(9).tolist(), t_prev.tolist(), 3)
            got, m_got = binding.rebalance(loads, 9, rates(9), t_prev, 3)
            assert m_ref == m_got
            return (9, ref, got) if m_ref else None
        if r == 6:
            return 3, opol.scale_in(t_prev.tolist(), 9, 3), binding.scale_in(t_prev, 9, 3)
        return None
    return tables


@pytest.mark.parametrize("solver,ahead", [("rowwise", False), ("batched", True)])
def test_policy_driven_elastic_run(mods, solver, ahead):
    oracle_mod, binding = mods
    cfg, p = cached_problem("elastic", "mini")
    print("\ncase elastic mini, policy tables,", solver, flush=True)
    rec = run_lockstep(cfg, p, oracle_mod, binding, rounds=8, solver=solver, ahead=ahead,
                       tables=_policy_schedule(cfg, p, binding), max_solvers=9,
                       log=lambda m: print(m, flush=True))
    assert [x["K"] for x in rec] == [4, 4, 9, 9, 9, 9, 3, 3]
    D = [x["D_gpu"] for x in rec]
    assert all(b >= a - 1e-6 for a, b in zip(D, D[1:])), "the dual objective never decreases"


def test_solver_runtimes_feed_the_rebalancing_policy(mods):
    """Per-solver runtimes come from device clock stamps; a solver with three times the rows must
    show clearly more time, an idle one none, and the rates learnt from them must give a valid table."""
    _, binding = mods
    cfg, p = cached_problem("sparse_zipf", "mini")
    print("\ncase sparse_zipf mini, solver runtimes", flush=True)
    K = 4
    g = binding.ChicleRound.from_problem(p, max_solvers=K)
    n = p.n_chunks
    table = np.array([0 if c < (3 * n) // 5 else 1 if c < (4 * n) // 5 else 2 for c in range(n)], dtype=np.int32)
    g.assign(K, table)                                   # solver 3 idle
    with pytest.raises(binding.ChicleError):
        g.solver_ms()                                    # no local epoch has run yet
    rows = g.solver_rows()
    g.set_profiling(True)
    hist = []
    for r in range(3):
        g.local_epoch(g.upload_perm(round_permutations(cfg["seed"], r, rows)))
        ms = g.solver_ms()
        total = g.last_kernel_ms("epoch_chain")
        g.aggregate()
        print("solver ms", ms, "kernel ms", total, flush=True)
        assert ms.shape == (K,) and np.all(ms >= 0) and ms[3] < 0.05 * ms[0]
        assert ms[0] > 2.0 * ms[1] and ms[0] > 2.0 * ms[2]
        assert ms.max() <= total * 1.05 + 0.05
        hist.append(ms)
    loads = p.chunk_nnz()
    per_solver = np.array([loads[table == k].sum() for k in range(K)], dtype=np.float64)
    live = per_solver > 0
    unit = np.array(hist, dtype=np.float64)
    unit[:, live] /= per_solver[live]
    unit[:, ~live] = np.median(unit[:, live])            # no history: the typical rate
    new, moved = binding.rebalance(loads, K, unit, table, 1000)
    assert moved > 0 and new.min() >= 0 and new.max() < K
    after = np.array([loads[new == k].sum() for k in range(K)])
    assert after.max() < per_solver.max()                # the longest solver got shorter
    g.close()


@pytest.mark.parametrize("K", [2, 6])
def test_microtask_emulation_run_matches_oracle(mods, K):
    """Constant-K runs (the emulation of K micro-tasks): the gap after every round and the number of
    rounds to the target agree with the oracle; the projection uses the printed model."""
    oracle_mod, binding = mods
    from paper_1909_04885_amd import sweep
    cfg, p = cached_problem("sparse_zipf", "mini")
    print("\ncase sparse_zipf mini, constant K =", K, flush=True)
    target, rounds = 0.1, 12
    res = sweep.run_to_gap(p, K, lambda r, rows: round_permutations(cfg["seed"], r, rows), target,
                           max_rounds=rounds, min_rounds=rounds)
    o = oracle_mod.OracleCoCoA.from_problem(p)
    o.assign(K, oracle_mod.assign_greedy(p.chunk_nnz(), K))
    ref = [o.gap()[2]]
    for r in range(rounds):
        o.local_epoch(round_permutations(cfg["seed"], r, o.rows_per_solver()))
        o.aggregate()
        ref.append(o.gap()[2])
    assert ref[0] == pytest.approx(1.0, abs=1e-12)          # hinge at alpha = 0, w = 0
    assert len(res["gaps"]) == rounds + 1
    for a, b in zip(res["gaps"], ref):
        assert abs(a - b) <= 1e-3 * abs(b)
    ref_reached = next((i for i, x in enumerate(ref) if i > 0 and x <= target * ref[0]), None)
    print("gaps", ["%.4f" % x for x in res["gaps"]], "reached", res["rounds_to_target"], ref_reached, flush=True)
    assert res["rounds_to_target"] == ref_reached
    rows = sweep.project([res], [K, 4])
    uni = [x for x in rows if x["mode"] == "uni-tasks"]
    assert len(uni) == 1 and uni[0]["iteration_time"] == pytest.approx(16.0 / K)


def test_scale_in_schedule_run_matches_oracle(mods):
    """Many solvers first, fewer after a few rounds (the schedule Section 2.2 cites): the driver's run,
    with its tables from the library's scale-in policy, against the oracle under the oracle's tables."""
    oracle_mod, binding = mods
    from paper_1909_04885_amd import sweep
    cfg, p = cached_problem("sparse_zipf", "mini")
    print("\ncase sparse_zipf mini, schedule 6 -> 3 -> 2", flush=True)
    sched, rounds = [(3, 3), (6, 2)], 9
    res = sweep.run_to_gap(p, 6, lambda r, rows: round_permutations(cfg["seed"], r, rows), 1e-9,
                           max_rounds=rounds, schedule=sched)
    assert res["K_per_round"] == [6, 6, 6, 3, 3, 3, 2, 2, 2]
    o = oracle_mod.OracleCoCoA.from_problem(p)
    K, table = 6, oracle_mod.assign_greedy(p.chunk_nnz(), 6).tolist()
    o.assign(K, np.asarray(table, dtype=np.int32))
    ref = [o.gap()[2]]
    for r in range(rounds):
        if r in dict(sched):
            K_new = dict(sched)[r]
            table = opol.scale_in(table, K, K_new)
            K = K_new
            o.assign(K, np.asarray(table, dtype=np.int32))
        o.local_epoch(round_permutations(cfg["seed"], r, o.rows_per_solver()))
        o.aggregate()
        ref.append(o.gap()[2])
    print("gaps", ["%.4f" % x for x in res["gaps"]], flush=True)
    for a, b in zip(res["gaps"], ref):
        assert abs(a - b) <= 1e-3 * abs(b)


def test_gap_driven_scale_in_run_matches_oracle(mods):
    """Solvers halved whenever a round leaves more than 0.8 of the gap: the driver's run, deciding through
    the library from the library's gaps, against the oracle deciding from its own.  The ratios at the
    decisions are far from the threshold (0.20, 0.90, 1.24), so both must take the same decisions."""
    oracle_mod, binding = mods
    from paper_1909_04885_amd import sweep
    cfg, p = cached_problem("sparse_zipf", "mini")
    print("\ncase sparse_zipf mini, gap-driven scale-in from 8 solvers", flush=True)
    rule, rounds = {"K_min": 2, "stall_ratio": 0.8, "patience": 1}, 8
    res = sweep.run_to_gap(p, 8, lambda r, rows: round_permutations(cfg["seed"], r, rows), 1e-9,
                           max_rounds=rounds, adaptive=rule)
    o = oracle_mod.OracleCoCoA.from_problem(p)
    K, table = 8, oracle_mod.assign_greedy(p.chunk_nnz(), 8).tolist()
    o.assign(K, np.asarray(table, dtype=np.int32))
    ref, ks, since = [o.gap()[2]], [], 0
    for r in range(rounds):
        o.local_epoch(round_permutations(cfg["seed"], r, o.rows_per_solver()))
        o.aggregate()
        ref.append(o.gap()[2])
        ks.append(K)
        since += 1
        K_new = opol.next_solver_count(ref, K, rule["K_min"], rule["stall_ratio"], rule["patience"], since)
        if K_new != K:
            table = opol.scale_in(table, K, K_new)
            K, since = K_new, 0
            o.assign(K, np.asarray(table, dtype=np.int32))
    print("solvers", res["K_per_round"], "gaps", ["%.4f" % x for x in res["gaps"]], flush=True)
    assert ks == [8, 8, 4, 2, 2, 2, 2, 2] and res["K_per_round"] == ks
    for a, b in zip(res["gaps"], ref):
        assert abs(a - b) <= 1e-3 * abs(b)


@pytest.mark.parametrize("K", [1, 17])
def test_odd_solver_counts_with_the_batched_solver(mods, K):
    """Solver counts that are not a multiple of the number of L2 partitions (the batched solver pairs every
    solver with a warming workgroup by index), including a single solver that owns every chunk."""
    oracle_mod, binding = mods
    cfg, p = cached_problem("sparse_zipf", "mini")
    print("\ncase sparse_zipf mini, K =", K, flush=True)
    table = (np.arange(p.n_chunks) % K).astype(np.int32)

    def tables(r, K_prev, t_prev):
        return (K, table, table.copy()) if r == 0 else None

    rec = run_lockstep(cfg, p, oracle_mod, binding, rounds=3, solver="batched", ahead=True, tables=tables,
                       max_solvers=K, log=lambda m: print(m, flush=True))
    assert [x["K"] for x in rec] == [K] * 3
