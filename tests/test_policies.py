"""Scheduling policies (Section 4.5) and the projection model (Sections 5.3, 5.4).

First the oracle's policies against what the paper and the arithmetic fix (hand-worked cases,
invariants, the heterogeneous example whose iteration time the paper prints), then the library's
host entry points against the oracle, table by table, bit for bit.  No GPU is needed: these entry
points never touch the device.
"""
import os

import numpy as np
import pytest

from oracle import policies as opol


# ------------------------------------------------------------------ oracle policies, pinned
def test_scale_out_hand_worked():
    # two solvers with four chunks each grow to four solvers: each gives floor(4*2/4) = 2 chunks,
    # those with the smallest draws; receivers 2, 3 are served in turn
    table = [0, 0, 0, 0, 1, 1, 1, 1]
    draw = [7, 6, 5, 4, 3, 2, 1, 0]
    assert opol.scale_out(table, 2, 4, draw) == [0, 0, 3, 2, 1, 1, 3, 2]


def test_scale_out_invariants():
    rng = np.random.default_rng(3)
    for _ in range(30):
        n, K_old = int(rng.integers(1, 80)), int(rng.integers(1, 9))
        K_new = K_old + int(rng.integers(1, 9))
        table = rng.integers(0, K_old, n).tolist()
        draw = rng.integers(0, 2 ** 32, n, dtype=np.uint64).tolist()
        new = opol.scale_out(table, K_old, K_new, draw)
        moved_total = 0
        for k in range(K_old):
            mine = [c for c in range(n) if table[c] == k]
            kept = [c for c in mine if new[c] == k]
            gone = [c for c in mine if new[c] != k]
            assert len(gone) == (len(mine) * (K_new - K_old)) // K_new
            assert all(new[c] >= K_old for c in gone)              # only to new solvers
            if kept and gone:                                      # the smallest draws left
                assert max((draw[c], c) for c in gone) < min((draw[c], c) for c in kept)
            moved_total += len(gone)
        counts = np.bincount(new, minlength=K_new)[K_old:]
        assert counts.sum() == moved_total and counts.max() - counts.min() <= 1


def test_scale_in_hand_worked_and_invariants():
    assert opol.scale_in([0, 1, 2, 3, 0, 1, 2, 3], 4, 2) == [0, 1, 0, 0, 0, 1, 1, 1]
    rng = np.random.default_rng(4)
    for _ in range(30):
        n, K_new = int(rng.integers(1, 80)), int(rng.integers(1, 8))
        K_old = K_new + int(rng.integers(1, 8))
        table = rng.integers(0, K_old, n).tolist()
        new = opol.scale_in(table, K_old, K_new)
        assert all(0 <= s < K_new for s in new)
        assert all(new[c] == table[c] for c in range(n) if table[c] < K_new)   # survivors keep theirs
        got = np.bincount([new[c] for c in range(n) if table[c] >= K_new], minlength=K_new)
        assert got.max() - got.min() <= 1                                      # round robin


def test_rebalance_hand_worked():
    # solver 1 is twice as slow: times 40 vs 80; one chunk (10 units -> 10 on the receiver) moves,
    # then 50 vs 60 differ by no more than one chunk's time
    table = [0, 0, 0, 0, 1, 1, 1, 1]
    new, moved = opol.rebalance([10] * 8, 2, [[1.0, 2.0]], table, 10)
    assert moved == 1 and new == [0, 0, 0, 0, 1, 1, 1, 0]


def test_rebalance_reaches_the_printed_heterogeneous_time():
    # Section 5.4: 8 fast nodes and 8 that take 1.5x as long; uni-tasks end at 1.2 time units with the
    # fast nodes holding 1.5x the samples.  960 equal chunks start evenly spread (60 each).
    K, n = 16, 960
    table = [c % K for c in range(n)]
    rate = [1.0 if k < 8 else 1.5 for k in range(K)]
    load = [1000] * n
    steps = 0
    while True:
        table, moved = opol.rebalance(load, K, [rate], table, 4)     # gradual: 4 chunks per iteration
        steps += 1
        if moved == 0:
            break
        assert steps < 1000
    counts = np.bincount(table, minlength=K)
    unit = n / 16.0
    times = [counts[k] / unit * rate[k] for k in range(K)]
    assert max(times) == pytest.approx(1.2, abs=1.5 / unit)          # within one chunk on a slow node
    assert round(max(times), 1) == 1.2
    assert abs(counts[:8].mean() / counts[8:].mean() - 1.5) < 0.05
    assert steps > 10                                                # it did take several iterations


def test_rebalance_never_lengthens_the_iteration_and_uses_the_median():
    rng = np.random.default_rng(5)
    for _ in range(20):
        n, K = int(rng.integers(2, 60)), int(rng.integers(2, 7))
        load = rng.integers(1, 1000, n).tolist()
        table = rng.integers(0, K, n).tolist()
        rate = rng.uniform(0.5, 2.0, K)

        def span(t):
            return max(rate[k] * sum(load[c] for c in range(n) if t[c] == k) for k in range(K))

        cur = table
        for _ in range(200):
            new, moved = opol.rebalance(load, K, [rate.tolist()], cur, 1)
            assert span(new) <= span(cur) + 1e-9
            if moved == 0:
                break
            cur = new
        else:
            raise AssertionError("did not settle")
        # one wild iteration out of three does not change the decision
        wild = (rate * rng.uniform(5, 50, K)).tolist()
        a, _ = opol.rebalance(load, K, [rate.tolist()], table, 3)
        b, _ = opol.rebalance(load, K, [rate.tolist(), wild, rate.tolist()], table, 3)
        assert a == b


# ------------------------------------------------------------------ library against the oracle
@pytest.fixture(scope="module")
def chicle():
    import paper_1909_04885_amd as m
    m.load_library()
    return m


def test_library_projection_model_on_the_printed_examples(chicle):
    path = os.path.join(os.path.dirname(__file__), "golden", "projection_examples.txt")
    seen = 0
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, K, nodes, n_slow, sf, want, digits = line.split()
        got = chicle.projected_iteration_time(None if K == "uni" else int(K), int(nodes), int(n_slow),
                                              1.0 if sf == "-" else float(sf))
        assert round(got, int(digits)) == float(want), name
        seen += 1
    assert seen == 4


def test_library_projection_model_matches_oracle(chicle, oracle_mod):
    for K in [None, 1, 7, 16, 24, 32, 64, 100]:
        for nodes in range(1, 20):
            a = chicle.projected_iteration_time(K, nodes)
            b = oracle_mod.projected_round_time(K, nodes)
            assert a == pytest.approx(b, rel=1e-15)
            for n_slow in range(0, nodes + 1, 3):
                a = chicle.projected_iteration_time(K, nodes, n_slow, 1.5)
                b = oracle_mod.projected_round_time(K, nodes, slow_factor=1.5, n_slow=n_slow)
                assert a == pytest.approx(b, rel=1e-15)
    with pytest.raises(chicle.ChicleError):
        chicle.projected_iteration_time(4, 0)
    with pytest.raises(chicle.ChicleError):
        chicle.projected_iteration_time(4, 4, 5, 1.5)


def test_library_scaling_tables_bit_exact(chicle):
    rng = np.random.default_rng(11)
    for _ in range(60):
        n, K_old = int(rng.integers(1, 600)), int(rng.integers(1, 40))
        K_new = K_old + int(rng.integers(1, 40))
        table = rng.integers(0, K_old, n).astype(np.int32)
        draw = rng.integers(0, 8, n).astype(np.uint32) if rng.random() < 0.3 else \
            rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32)      # some with many ties
        assert chicle.scale_out(table, K_old, K_new, draw).tolist() == \
            opol.scale_out(table.tolist(), K_old, K_new, draw.tolist())
        big = rng.integers(0, K_new, n).astype(np.int32)
        assert chicle.scale_in(big, K_new, K_old).tolist() == opol.scale_in(big.tolist(), K_new, K_old)
    with pytest.raises(chicle.ChicleError):
        chicle.scale_out([0, 1], 2, 2, [1, 2])
    with pytest.raises(chicle.ChicleError):
        chicle.scale_out([0, 2], 2, 3, [1, 2])
    with pytest.raises(chicle.ChicleError):
        chicle.scale_in([0, 1], 2, 2)


def test_library_rebalance_bit_exact(chicle):
    rng = np.random.default_rng(12)
    for _ in range(60):
        n, K, I = int(rng.integers(1, 300)), int(rng.integers(1, 20)), int(rng.integers(1, 6))
        load = rng.integers(0, 5000, n).astype(np.int64)
        if rng.random() < 0.3:
            load[:] = 4096 * 40                                   # equal chunks: every tie rule matters
        table = rng.integers(0, K, n).astype(np.int32)
        ut = rng.uniform(1e-7, 3e-7, (I, K))
        moves = int(rng.integers(0, 12))
        got, m_got = chicle.rebalance(load, K, ut, table, moves)
        ref, m_ref = opol.rebalance(load.tolist(), K, ut.tolist(), table.tolist(), moves)
        assert got.tolist() == ref and m_got == m_ref
    with pytest.raises(chicle.ChicleError):
        chicle.rebalance([1, 2], 2, [[1.0, 0.0]], [0, 1], 1)
    with pytest.raises(chicle.ChicleError):
        chicle.rebalance([1, 2], 2, [[1.0, 1.0]], [0, 2], 1)


def test_projection_special_cases(oracle_mod):
    """Mixed-node model against the equal-node one: no slow node, or only slow nodes (then every task
    takes slow_factor times as long), or slow_factor 1, all reduce to base/K * ceil(K/N)."""
    for K in [1, 5, 16, 32, 33, 64]:
        for N in [1, 3, 14, 16]:
            eq = 16.0 / K * -(-K // N)
            assert oracle_mod.projected_round_time(K, N) == pytest.approx(eq)
            assert oracle_mod.projected_round_time(K, N, slow_factor=1.5, n_slow=N) == pytest.approx(1.5 * eq)
            assert oracle_mod.projected_round_time(K, N, slow_factor=1.0, n_slow=N // 2) == pytest.approx(eq)
            assert oracle_mod.projected_round_time(None, N, slow_factor=2.0, n_slow=N) == pytest.approx(2.0 * 16 / N)


def test_scale_in_trigger_hand_worked():
    """Gaps 1, .5, .45, .43: rounds 2 and 3 each left more than 0.8 of their gap.  With patience 2 the
    change comes after round 3, not earlier, and only if both rounds ran with the current K."""
    g = [1.0, 0.5, 0.45, 0.43]
    assert opol.next_solver_count(g[:2], 64, 8, 0.8, 1, 1) == 64          # 0.5 of the gap left: progress
    assert opol.next_solver_count(g[:3], 64, 8, 0.8, 1, 2) == 32          # 0.9 left: stalled
    assert opol.next_solver_count(g[:3], 64, 8, 0.8, 2, 2) == 64          # only one of the last two stalled
    assert opol.next_solver_count(g, 64, 8, 0.8, 2, 3) == 32
    assert opol.next_solver_count(g, 64, 8, 0.8, 2, 1) == 64              # K changed one round ago
    assert opol.next_solver_count(g, 9, 8, 0.8, 1, 3) == 8                # never below the floor
    assert opol.next_solver_count(g, 8, 8, 0.8, 1, 3) == 8
    assert opol.next_solver_count(g, 5, 1, 0.8, 1, 3) == 3                # halves round up
    assert opol.next_solver_count([1.0], 64, 8, 0.8, 1, 0) == 64          # no round yet
    assert opol.next_solver_count([1.0, 1.5], 64, 8, 0.8, 1, 1) == 32     # a gap that grew has stalled


def test_library_scale_in_trigger_matches_oracle(chicle):
    rng = np.random.default_rng(13)
    for _ in range(300):
        n = int(rng.integers(1, 12))
        g = np.cumprod(np.concatenate([[1.0], rng.choice([0.3, 0.7, 0.79, 0.81, 0.95, 1.1], n - 1)])) if n > 1 else np.array([1.0])
        K, K_min = int(rng.integers(1, 70)), int(rng.integers(1, 20))
        ratio = float(rng.choice([0.5, 0.8, 1.0]))
        patience, since = int(rng.integers(1, 4)), int(rng.integers(0, 6))
        assert chicle.next_solver_count(g, K, K_min, ratio, patience, since) == \
            opol.next_solver_count(g.tolist(), K, K_min, ratio, patience, since)
    for bad in [dict(K=0), dict(K_min=0), dict(stall_ratio=0.0), dict(stall_ratio=1.5), dict(patience=0),
                dict(since_change=-1)]:
        args = dict(gaps=[1.0, 0.9], K=4, K_min=2, stall_ratio=0.8, patience=1, since_change=1)
        args.update(bad)
        with pytest.raises(chicle.ChicleError):
            chicle.next_solver_count(**args)
