"""Lock-step driver used by the GPU parity tests: the HIP library and the CPU oracle run the same
rounds on the same seeded inputs and the same visiting orders, compared after every step."""
from __future__ import annotations

import functools

import numpy as np

from workloads import get_config, make_problem, round_permutations
from workloads.configs import k_for_round, speeds_for

# Tolerances of the target: per-round relative L2 error of every Delta w, relative error of the final
# duality gap.  fp32 kernels against the fp64 oracle, free-running (no resynchronisation).
TOL_DW = 1e-4
TOL_GAP = 1e-3
# Both sides keep alpha and the shared vector's mirror in fp32 on the device.  Once a run has converged so far
# that an update is smaller than the fp32 resolution of the vector it is added to, an error relative to the
# update measures rounding of the state, not the update: the error of every Delta w is therefore taken
# relative to max(|Delta w_ref|, DW_FLOOR_ULPS * 2^-23 * |w| / TOL_DW), i.e. it passes when it is within
# 1e-4 of the update or within DW_FLOOR_ULPS units in the last place of |w|, whichever is larger.
# Applied to every loss and every case.
EPS32 = 2.0 ** -23
DW_FLOOR_ULPS = 1.0


def gap_tolerance(gap_ref: float, primal_ref: float) -> float:
    """The final gap must be within 1e-3 of the oracle's, or within one unit in the last place (fp32, the
    precision of the state) of the primal value it is the difference of, whichever is larger: a gap far
    below 2^-23 |P| is below what fp32 alpha and w can express."""
    return max(TOL_GAP * abs(gap_ref), EPS32 * abs(primal_ref))


def dw_floor(wnorm: float) -> float:
    return max(DW_FLOOR_ULPS * EPS32 * wnorm / TOL_DW, 1e-12 * max(wnorm, 1.0))


@functools.lru_cache(maxsize=2)
def cached_problem(name: str, size: str):
    cfg = get_config(name, size)
    return cfg, make_problem(cfg)


def rel_l2(got: np.ndarray, ref: np.ndarray, floor: float) -> float:
    den = max(float(np.linalg.norm(ref)), floor)
    return float(np.linalg.norm(got.astype(np.float64) - ref)) / den


def greedy_tables(cfg, p, oracle_mod, binding_mod):
    """The configured schedule: a greedy balanced table from each side whenever K changes."""
    loads = p.chunk_nnz()

    def tables(r, K_prev, t_prev):
        Kr = k_for_round(cfg, r)
        if Kr == K_prev:
            return None
        sp = speeds_for(cfg, Kr)
        return Kr, oracle_mod.assign_greedy(loads, Kr, sp), binding_mod.balance(loads, Kr, sp)
    return tables


def run_lockstep(cfg, p, oracle_mod, binding_mod, rounds=None, solver="auto", sample_solvers=None,
                 check_alpha_every=0, log=None, ahead=False, tables=None, max_solvers=None, l1=0.0):
    """`sample_solvers`: None compares every solver's Delta w in every round; a list compares every solver
    in the first, the middle and the last round and those of the list in the others (the summed update is
    compared in every round either way).  Returns a list of per-round records; raises AssertionError on the
    first violation.

    `tables(r, K_prev, table_prev)` returns None (no change before round r) or (K, table from the
    oracle side, table from the library side); default: the configured greedy schedule.
    `l1` > 0: the elastic-net regulariser lambda (|w|^2 / 2 + l1 |w|_1) on both sides."""
    o = oracle_mod.OracleCoCoA.from_problem(p, l1=l1)
    maxK = max_solvers or max(k for _, k in cfg["schedule"])
    tables = tables or greedy_tables(cfg, p, oracle_mod, binding_mod)
    table = None
    g = binding_mod.ChicleRound.from_problem(p, max_solvers=maxK)
    g.set_solver(solver)
    if l1:
        g.set_l1(l1)
    rounds = cfg["rounds"] if rounds is None else rounds
    K = None
    rec = []
    loads = p.chunk_nnz()
    announced = False    # the previous round announced this round's visiting orders
    for r in range(rounds):
        change = tables(r, K, table)
        if change is not None:
            K, t_ref, t_gpu = change
            t_ref = np.asarray(t_ref, dtype=np.int32)
            assert np.array_equal(t_ref, t_gpu), "chunk -> solver table differs at round %d" % r
            table = t_ref
            alpha_before = [g.get_alpha(c) for c in range(min(p.n_chunks, 4))] if r > 0 else None
            o.assign(K, t_ref)
            g.assign(K, t_gpu)
            back, kb = g.get_assignment()
            assert kb == K and np.array_equal(back, t_ref)
            assert list(g.solver_rows()) == o.rows_per_solver()
            if alpha_before is not None:      # state stays with its chunk across a reassignment
                for c, a in enumerate(alpha_before):
                    assert np.array_equal(a, g.get_alpha(c))
        perms = round_permutations(cfg["seed"], r, o.rows_per_solver())
        if not ahead:
            g.local_epoch(g.upload_perm(perms))
        else:
            # announce the next round's orders unless the schedule reassigns chunks before it; a round whose
            # orders were announced runs with the library's copy of them (the tensor is gone by then)
            cur_dev = None if announced else g.upload_perm(perms)
            next_dev = None
            if r + 1 < rounds and tables(r + 1, K, table) is None:
                next_dev = g.upload_perm(round_permutations(cfg["seed"], r + 1, o.rows_per_solver()))
            g.local_epoch_ahead(cur_dev, next_dev)
            announced = next_dev is not None
            del cur_dev, next_dev
        wnorm = float(np.linalg.norm(o.w))
        worst = [0.0]
        every = sample_solvers is None or r in (0, rounds // 2, rounds - 1)
        which = set(range(K)) if every else {s % K for s in sample_solvers}
        floor = dw_floor(wnorm)

        def on_delta(k, dw):
            if k in which:
                e = rel_l2(g.get_delta_w(k), dw, floor)
                worst[0] = max(worst[0], e)
                assert e <= TOL_DW, "round %d solver %d: Delta w rel L2 error %.3e" % (r, k, e)

        o.local_epoch(perms, keep_deltas=False, on_delta=on_delta)
        tot = o._pending
        e_sum = rel_l2(g.get_delta_w(-1), tot, floor)
        assert e_sum <= TOL_DW, "round %d: summed Delta w rel L2 error %.3e" % (r, e_sum)
        o.aggregate()
        g.aggregate()
        Pg, Dg, Gg = g.gap()
        Po, Do, Go, _ = o.gap()
        e_w = rel_l2(g.get_w(), o.w, 1e-30)
        rec.append(dict(round=r, K=K, dw_err=worst[0], dw_sum_err=e_sum, w_err=e_w, w_zero=float(np.mean(o.w == 0.0)),
                        gap_gpu=Gg, gap_ref=Go, P_gpu=Pg, P_ref=Po, D_gpu=Dg, D_ref=Do))
        if log:
            log("r=%d K=%d dw_err=%.2e sum_err=%.2e w_err=%.2e gap gpu=%.6e ref=%.6e" %
                (r, K, worst[0], e_sum, e_w, Gg, Go))
        assert Gg >= -1e-6, "weak duality violated on the GPU side"
        if check_alpha_every and (r % check_alpha_every == 0 or r == rounds - 1):
            for c in range(p.n_chunks):
                r0, r1 = p.chunk_rows(c)
                a = g.get_alpha(c)
                assert np.max(np.abs(a.astype(np.float64) - o.alpha[r0:r1])) <= 5e-4, "alpha drift in chunk %d" % c
    last = rec[-1]
    assert abs(last["gap_gpu"] - last["gap_ref"]) <= gap_tolerance(last["gap_ref"], last["P_ref"]), \
        "final gap %.9e vs %.9e" % (last["gap_gpu"], last["gap_ref"])
    g.close()
    return rec
