"""Micro-task emulation on the GPU library (Section 5.1 "Micro-tasks", Section 5.3 "Methodology").

With micro-tasks the convergence per epoch depends only on the number of tasks K, so a run with a
constant K measures it; convergence over time is then projected with the iteration-time model:
K tasks on N nodes need ceil(K/N) waves of 16/K time units each, while uni-tasks (one task per
node, K = N) need 16/N.  This module runs the rounds through `ChicleRound` (every step in the HIP
library) and does the projection through `chicle_projected_iteration_time`.

    python -m paper_1909_04885_amd.sweep --workload sparse_zipf --size full --tasks 16 24 32 64 --nodes 16 14 8
"""
from __future__ import annotations

import argparse
import json
import sys
import time
from typing import Callable, Dict, List, Optional, Sequence

import numpy as np

from .binding import ChicleRound, balance, next_solver_count, projected_iteration_time, scale_in, scale_out


def run_to_gap(problem, K: int, permutations: Callable[[int, Sequence[int]], list], target_rel: float,
               max_rounds: int, min_rounds: int = 0, table: Optional[np.ndarray] = None,
               device: str = "cuda:0", schedule: Optional[Sequence] = None,
               draws: Optional[Callable[[int, int], np.ndarray]] = None,
               adaptive: Optional[Dict] = None) -> Dict:
    """Rounds with a constant number of solvers K from alpha = 0, w = 0 until the duality gap has
    fallen to `target_rel` times its initial value (or `max_rounds`).

    permutations(round, rows_per_solver) supplies the visiting orders (they are inputs of the method).
    Returns the gap after every round (entry 0: before the first), the first round count at which the
    target was met (None if never), and the wall-clock time of the rounds up to that point (visiting
    orders are uploaded before the clock starts).

    schedule: optional [(round, K), ...] changes of the number of solvers before the given rounds
    (Section 2.2 cites that starting with many partitions and reducing them after a few iterations
    speeds up convergence): fewer solvers through the scale-in policy, more through the scale-out policy
    with draws(round, n_chunks) as its random words.  K is then the first entry's solver count.

    adaptive: {"K_min", "stall_ratio", "patience"}: after every round `chicle_next_solver_count` decides
    from the gaps so far whether to halve the number of solvers (scale-in policy) before the next one."""
    import torch
    changes = dict(schedule or [])
    g = ChicleRound.from_problem(problem, max_solvers=max([K] + list(changes.values())), device=device)
    try:
        if table is None:
            table = balance(problem.chunk_nnz(), K)
        g.assign(K, table)
        rows = g.solver_rows()
        ks = [K]
        g0 = g.gap()[2]
        gaps = [g0]
        reached, t_reached = None, None
        block = 16                                  # orders are generated and uploaded in blocks
        elapsed = 0.0
        r = 0
        since_change = 0
        while r < max_rounds and (reached is None or r < min_rounds):
            if r in changes and changes[r] != K:
                K_new = changes[r]
                table = scale_in(table, K, K_new) if K_new < K else \
                    scale_out(table, K, K_new, draws(r, len(table)))
                K = K_new
                g.assign(K, table)
                rows = g.solver_rows()
                since_change = 0
            nxt = min([c for c in changes if c > r] or [max_rounds])
            n_blk = min(block, max_rounds - r, nxt - r)
            dev = [g.upload_perm(permutations(r + i, rows)) for i in range(n_blk)]
            torch.cuda.synchronize()
            for i in range(n_blk):
                t0 = time.perf_counter()
                # the first round of a block brings its orders, the others run with the orders announced before
                g.local_epoch_ahead(dev[i] if i == 0 else None, dev[i + 1] if i + 1 < n_blk else None)
                g.aggregate()
                gap = g.gap()[2]                    # the scalars come back: the round has ended
                elapsed += time.perf_counter() - t0
                gaps.append(gap)
                ks.append(K)
                r += 1
                since_change += 1
                if reached is None and gap <= target_rel * g0:
                    reached, t_reached = r, elapsed
                if reached is not None and r >= min_rounds:
                    break
                if adaptive:
                    K_new = next_solver_count(gaps, K, adaptive["K_min"], adaptive["stall_ratio"],
                                              adaptive["patience"], since_change)
                    if K_new != K:                  # orders uploaded for later rounds no longer fit
                        changes[r] = K_new
                        break
        return {"K": ks[0], "K_per_round": ks[1:], "gaps": gaps, "rounds_to_target": reached, "seconds_to_target": t_reached,
                "seconds": elapsed, "rounds": r}
    finally:
        g.close()


def project(results: List[Dict], nodes: Sequence[int]) -> List[Dict]:
    """Projected time to the target (normalised units) of every run on every node count: rounds to
    the target times the iteration time of K micro-tasks on N nodes; a run with K = N also is the
    uni-task run for N nodes."""
    rows = []
    for res in results:
        R = res["rounds_to_target"]
        for N in nodes:
            it = projected_iteration_time(res["K"], N)
            rows.append({"K": res["K"], "nodes": N, "mode": "micro-tasks", "iteration_time": it,
                         "time_to_target": None if R is None else R * it})
            if res["K"] == N:
                it = projected_iteration_time(None, N)
                rows.append({"K": res["K"], "nodes": N, "mode": "uni-tasks", "iteration_time": it,
                             "time_to_target": None if R is None else R * it})
    return rows


def main(argv=None) -> int:
    from workloads import get_config, make_problem, round_permutations
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--workload", default="sparse_zipf")
    ap.add_argument("--size", default="full")
    ap.add_argument("--tasks", type=int, nargs="+", default=[16, 24, 32, 64])
    ap.add_argument("--nodes", type=int, nargs="+", default=[16, 14, 8])
    ap.add_argument("--target", type=float, default=1e-3, help="gap relative to the initial gap")
    ap.add_argument("--max-rounds", type=int, default=200)
    ap.add_argument("--adaptive", nargs=4, default=None, metavar=("K0", "K_MIN", "STALL_RATIO", "PATIENCE"),
                    help="one more run that starts with K0 solvers and halves them whenever PATIENCE rounds in a row "
                         "left more than STALL_RATIO of the gap, e.g. 64 8 0.75 1")
    ap.add_argument("--schedule", nargs="*", default=[], metavar="ROUND:K",
                    help="one more run that changes the number of solvers before the given rounds, e.g. 0:64 3:32 6:16")
    args = ap.parse_args(argv)
    cfg = get_config(args.workload, args.size)
    p = make_problem(cfg)
    results = []
    for K in sorted(set(args.tasks) | set(args.nodes)):
        res = run_to_gap(p, K, lambda r, rows: round_permutations(cfg["seed"], r, rows), args.target,
                         args.max_rounds)
        print("K=%3d  rounds to gap <= %g x initial: %s  (%.1f ms per round, final gap %.3e)" %
              (K, args.target, res["rounds_to_target"], 1e3 * res["seconds"] / max(res["rounds"], 1),
               res["gaps"][-1]), file=sys.stderr, flush=True)
        results.append(res)
    scheduled = None
    if args.schedule:
        from workloads import chunk_draws
        sched = sorted(tuple(int(x) for x in item.split(":")) for item in args.schedule)
        scheduled = run_to_gap(p, sched[0][1], lambda r, rows: round_permutations(cfg["seed"], r, rows), args.target,
                               args.max_rounds, schedule=sched[1:],
                               draws=lambda r, n: chunk_draws(cfg["seed"], r, n))
        print("schedule %s: rounds to target %s, %.1f ms to target" %
              (sched, scheduled["rounds_to_target"], 1e3 * (scheduled["seconds_to_target"] or float("nan"))),
              file=sys.stderr, flush=True)
    adaptive = None
    if args.adaptive:
        K0, K_min, ratio, patience = int(args.adaptive[0]), int(args.adaptive[1]), float(args.adaptive[2]), int(args.adaptive[3])
        adaptive = run_to_gap(p, K0, lambda r, rows: round_permutations(cfg["seed"], r, rows), args.target,
                              args.max_rounds, adaptive={"K_min": K_min, "stall_ratio": ratio, "patience": patience})
        print("adaptive from K=%d (floor %d, stall ratio %g, patience %d): solvers per round %s, rounds to target %s, "
              "%.1f ms to target" % (K0, K_min, ratio, patience, adaptive["K_per_round"], adaptive["rounds_to_target"],
                                     1e3 * (adaptive["seconds_to_target"] or float("nan"))), file=sys.stderr, flush=True)
    out = {"workload": "%s/%s" % (args.workload, args.size), "target_rel": args.target,
           "adaptive": None if adaptive is None else {k: v for k, v in adaptive.items() if k != "gaps"},
           "scheduled": None if scheduled is None else {k: v for k, v in scheduled.items() if k != "gaps"},
           "runs": [{k: v for k, v in r.items() if k != "gaps"} for r in results],
           "gaps": {str(r["K"]): r["gaps"] for r in results},
           "projection": project(results, args.nodes)}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
