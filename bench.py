#!/usr/bin/env python3
"""Benchmark of the CoCoA round on one MI355X.

A step is one whole round: the local SDCA pass of all K solvers, the aggregation of their updates
and the duality-gap evaluation, on a synthetic workload already resident in HBM (visiting orders
included).  Prints one JSON line: whole-round throughput in stored matrix entries per second, the
HBM roofline position of the dominant kernel (the local pass), and the CPU oracle timed on a bounded
sample of the same workload on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes(p, K, touched):
    """Bytes the local pass must move per launch: the matrix once, the per-row state once, and each
    solver's touched part of its private vector in and out once (cache traffic is not counted).
    CSR: 8 B per entry + 24 B per row (row offset, order entry, label, norm, alpha read and write)
    + 8 B per distinct column a solver touches (`touched`: their number over all solvers).  Dense:
    4 B per entry + 20 B per row + 8 B per column per solver."""
    if p.dense:
        return 4 * p.nnz + 20 * p.n + 8 * p.d * K
    return 8 * p.nnz + 24 * p.n + 8 * touched


def aggregate_bytes(p, table, K, touched):
    """Bytes the merge must move: every solver's update once in and (cleared) once out, w in and out in
    double plus its float mirror out.  Where a private vector is mostly untouched (long-row workload)
    only the touched columns count: 8 B per distinct column a solver touches + the shared vector."""
    dense = 4 * p.d * (2 * K) + 20 * p.d
    if touched is None:
        return dense
    return min(dense, 8 * touched + 20 * p.d)


def touched_columns(p, table, K):
    """Distinct (solver, column) pairs of the assignment (sparse workloads)."""
    touched = 0
    for k in range(K):
        seen = np.zeros(p.d, dtype=bool)
        for c in np.nonzero(table == k)[0]:
            r0, r1 = p.chunk_rows(c)
            seen[p.col[p.row_ptr[r0]:p.row_ptr[r1]]] = True
        touched += int(seen.sum())
    return touched


def stream_copy_gbs(torch, n_bytes=1 << 30, reps=5):
    """What a plain device-to-device copy reaches on this GPU (bytes read + bytes written per second): the
    practical ceiling to set beside the datasheet's 8 TB/s."""
    src = torch.empty(n_bytes // 4, dtype=torch.float32, device="cuda:0").fill_(1.0)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    best = 0.0
    for _ in range(reps):
        e0.record()
        dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        best = max(best, 2.0 * n_bytes / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    del src, dst
    return best


def host_cpu():
    model, total = "unknown", os.cpu_count()
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    return model, total


def cpu_baseline(p, cfg, table, K, budget_s=15.0):
    """The oracle as it stands, single-threaded, on whole rounds of the same workload until about
    budget_s seconds of CPU work have been spent (at least one round)."""
    import oracle
    o = oracle.OracleCoCoA.from_problem(p)
    o.assign(K, table)
    from workloads import round_permutations
    rounds, spent = 0, 0.0
    while rounds < 1 or (spent < budget_s and rounds < cfg["rounds"]):
        perms = round_permutations(cfg["seed"], rounds, o.rows_per_solver())
        t0 = time.perf_counter()
        o.local_epoch(perms, keep_deltas=False)
        o.aggregate()
        o.gap()
        spent += time.perf_counter() - t0
        rounds += 1
    model, total = host_cpu()
    return {"value": p.nnz * rounds / spent, "unit": "nnz/s", "cores": 1, "kind": "oracle",
            "cpu_model": model, "host_cores_total": total,
            "sample": "%d whole rounds of the same workload (local pass + aggregate + gap), %.1f s" % (rounds, spent)}


def elastic_schedule(chicle, p, cfg, round_permutations):
    """The configured (round, K) schedule with unequal solver speeds (Section 5.4: uni-tasks on nodes of
    different speed get data in proportion to their speed): per phase the measured time of a round, the time
    of the reassignment, and the projected iteration time of the greedy assignment, max_k load_k / speed_k,
    against a perfect split (total load / total speed).  The GPU runs every solver at full speed: the speeds
    only weight the assignment, so the measured time is that of the unbalanced table."""
    import torch
    from workloads.configs import k_for_round, speeds_for
    loads = p.chunk_nnz()
    g = chicle.ChicleRound.from_problem(p, max_solvers=max(k for _, k in cfg["schedule"]))
    phases, K, rows = [], None, None
    for r in range(cfg["rounds"]):
        Kr = k_for_round(cfg, r)
        if Kr != K:
            K = Kr
            sp = speeds_for(cfg, K)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            table = chicle.balance(loads, K, sp)
            g.assign(K, table)
            g.sync()
            assign_ms = (time.perf_counter() - t0) * 1e3
            rows = g.solver_rows()
            speed = np.array([1.0] * K if sp is None else [q / max(sp) for q in sp])
            per_solver = np.bincount(table, weights=loads, minlength=K)
            phases.append({"first_round": r, "K": K, "assign_ms": assign_ms, "round_ms": [],
                           "projected_iteration_load": float(np.max(per_solver / speed)),
                           "perfect_split_load": float(loads.sum() / speed.sum())})
        perm = g.upload_perm(round_permutations(cfg["seed"], r, rows))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        g.local_epoch(perm); g.aggregate(); gap = g.gap()[2]
        phases[-1]["round_ms"].append((time.perf_counter() - t0) * 1e3)
        phases[-1]["gap_after"] = gap
    g.close()
    for ph in phases:
        ph["rounds"] = len(ph["round_ms"])
        ph["round_ms_median"] = float(np.median(ph.pop("round_ms")))
        ph["imbalance"] = ph["projected_iteration_load"] / ph["perfect_split_load"]
    return phases


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="sparse_zipf")
    ap.add_argument("--size", default="full")
    ap.add_argument("--solver", default="auto")
    ap.add_argument("--loss", default=None, choices=["hinge", "squared", "logistic"],
                    help="train this loss on the workload's data instead of its own (labels must fit)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-time-to-gap", action="store_true")
    ap.add_argument("--gap-round-cap", type=int, default=100)
    ap.add_argument("--scale-in-from", type=int, default=0, metavar="K0",
                    help="also time the run to the gap target that starts with K0 solvers and scales in as rounds stall")
    ap.add_argument("--repeats", type=int, default=3,
                    help="timed runs of --steps rounds each; `value` is the first, the others are reported beside it")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (untimed), as a reference for HBM byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the K local solvers run concurrently on a single MI355X and "
              "nothing here uses a second device; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_1909_04885_amd as chicle
    from paper_1909_04885_amd.record_traffic import stored_traffic
    from workloads import get_config, make_problem, round_permutations

    cfg = get_config(args.workload, args.size)
    t0 = time.time()
    p = make_problem(cfg)
    K = cfg["K"]
    if args.loss and args.loss != p.loss:
        import dataclasses
        p = dataclasses.replace(p, loss=args.loss)
    table = chicle.balance(p.chunk_nnz(), K)
    print("generated %s/%s: n=%d d=%d entries=%d chunks=%d K=%d in %.1fs" %
          (args.workload, args.size, p.n, p.d, p.nnz, p.n_chunks, K, time.time() - t0), file=sys.stderr, flush=True)

    g = chicle.ChicleRound.from_problem(p, max_solvers=K)
    g.set_solver(args.solver)
    g.assign(K, table)
    rows = g.solver_rows()
    total = args.warmup + args.steps * max(args.repeats, 1)
    perms = [g.upload_perm(round_permutations(cfg["seed"], r, rows)) for r in range(total)]
    g.set_profiling(True)
    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").fill_(1.0)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                     # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    torch.cuda.synchronize()

    def nxt(r):
        return perms[r + 1] if r + 1 < total else None

    def cur(r):                            # every round but the first runs with the orders announced before it
        return perms[r] if r == 0 else None

    for r in range(args.warmup):
        g.local_epoch_ahead(cur(r), nxt(r)); g.aggregate(); g.gap()
    torch.cuda.synchronize()
    copy_gbs = stream_copy_gbs(torch)
    seg_ms = {"local_epoch": [], "aggregate": [], "gap": [], "epoch_gram": [], "epoch_chain": []}
    gaps = []
    run_ms = []
    r = args.warmup
    for run in range(max(args.repeats, 1)):
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        for _ in range(args.steps):
            g.local_epoch_ahead(cur(r), nxt(r))       # announces the next round's orders (all are in HBM)
            g.aggregate()
            gaps.append(g.gap()[2])          # synchronises: the three scalars come back to the host
            for s in seg_ms:                  # events of this round have completed
                try:
                    seg_ms[s].append(g.last_kernel_ms(s))
                except chicle.ChicleError:
                    pass                      # segment not part of this solver kind
            r += 1
        torch.cuda.synchronize()
        run_ms.append((time.perf_counter() - t_start) * 1e3 / args.steps)
    ms_per_step = run_ms[0]                   # the K timed steps of the contract: the first run

    def med(name):
        return float(np.median(seg_ms[name])) if seg_ms[name] else None

    epoch_ms, agg_ms, gap_ms = med("local_epoch"), med("aggregate"), med("gap")
    touched = None if p.dense else touched_columns(p, table, K)
    abytes = algorithmic_bytes(p, K, touched)
    achieved = abytes / (epoch_ms * 1e-3) / 1e9
    agg_bytes = aggregate_bytes(p, table, K, touched)
    gap_bytes = (8 if not p.dense else 4) * p.nnz + 12 * p.n + 4 * p.d
    traffic = stored_traffic("%s/%s" % (args.workload, args.size)) if args.solver == "auto" and not args.loss else None
    out = {
        "metric": "nnz_per_s_per_cocoa_round",
        "value": p.nnz / (ms_per_step * 1e-3),
        "unit": "nnz/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s/%s" % (args.workload, args.size), "n": p.n, "d": p.d, "entries": p.nnz,
                   "K": K, "chunk_rows": cfg["chunk_rows"], "lambda": cfg["lam"], "loss": p.loss,
                   "solver": args.solver},
        # every timed run of `steps` rounds; segment times below are medians over the rounds of all runs
        "runs_ms_per_step": run_ms, "ms_per_step_median_of_runs": float(np.median(run_ms)),
        # The local pass as the round sees it: everything chicle_local_epoch enqueues on the context's stream,
        # the wait for the Gram tiles included.  chain_ms: the kernel that takes the coordinate steps;
        # gram_ms: the Gram-tile kernel of the next pass, which runs beside it on the other compute units.
        "local_epoch": {"ms": epoch_ms, "nnz_per_s": p.nnz / (epoch_ms * 1e-3),
                        "coord_updates_per_s": p.n / (epoch_ms * 1e-3),
                        "gram_ms": med("epoch_gram"), "chain_ms": med("epoch_chain"),
                        # the dependency chain: a solver's coordinate steps come one after the other
                        "max_rows_per_solver": int(max(rows)),
                        "ns_per_step_of_longest_solver": epoch_ms * 1e6 / max(int(max(rows)), 1)},
        "aggregate": {"ms": agg_ms, "algorithmic_bytes": agg_bytes, "GB_per_s": agg_bytes / (agg_ms * 1e-3) / 1e9,
                      "frac_hbm_peak": agg_bytes / (agg_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "gap": {"ms": gap_ms, "algorithmic_bytes": gap_bytes, "GB_per_s": gap_bytes / (gap_ms * 1e-3) / 1e9,
                "frac_hbm_peak": gap_bytes / (gap_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "first": gaps[0], "last": gaps[-1]},
        "roofline": {"kernel": "local_epoch", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     # what a plain device copy reaches on this GPU, and the fraction of that
                     "stream_copy_GBps": copy_gbs, "frac_of_stream_copy": achieved / copy_gbs,
                     # Bytes that left L2 per round for the local pass (chain kernel + Gram kernel), from
                     # FETCH_SIZE / WRITE_SIZE counter runs scaled by a plain copy of known size; null unless
                     # taken on exactly these kernel sources.  Infinity-Cache hits are included: the counters
                     # sit between L2 and the fabric, not at the HBM pins.
                     "traffic": None if traffic is None else traffic["local_pass_bytes"],
                     "traffic_by_kernel": None if traffic is None else traffic["kernels"],
                     "traffic_unit": "bytes between L2 and the fabric per round",
                     "algorithmic_bytes": abytes},
    }
    g.close()
    if not args.no_time_to_gap:
        # from alpha = 0, w = 0 to a duality gap of 1e-3 of its initial value: wall clock over local
        # epoch + aggregate + gap of every round, visiting orders already in HBM
        from paper_1909_04885_amd.sweep import run_to_gap
        res = run_to_gap(p, K, lambda r, rws: round_permutations(cfg["seed"], r, rws), 1e-3,
                         max_rounds=args.gap_round_cap, table=table)
        out["time_to_gap"] = {"target": "gap <= 1e-3 x gap(alpha=0, w=0)", "rounds": res["rounds_to_target"],
                              "ms": None if res["seconds_to_target"] is None else 1e3 * res["seconds_to_target"],
                              "round_cap": args.gap_round_cap, "final_gap": res["gaps"][-1],
                              "initial_gap": res["gaps"][0]}
        if args.scale_in_from and args.scale_in_from > K:
            # the same target with the number of solvers chosen as the run goes: start with more solvers
            # and halve them whenever a round leaves more than 3/4 of the gap (never below K / 4)
            rule = {"K_min": max(K // 4, 1), "stall_ratio": 0.75, "patience": 1}
            res = run_to_gap(p, args.scale_in_from, lambda r, rws: round_permutations(cfg["seed"], r, rws), 1e-3,
                             max_rounds=args.gap_round_cap, adaptive=rule)
            out["time_to_gap_scale_in"] = {
                "rule": dict(rule, K_start=args.scale_in_from), "rounds": res["rounds_to_target"],
                "ms": None if res["seconds_to_target"] is None else 1e3 * res["seconds_to_target"],
                "solvers_per_round": res["K_per_round"][:res["rounds_to_target"] or None]}
    if len(cfg["schedule"]) > 1:
        out["elastic_schedule"] = elastic_schedule(chicle, p, cfg, round_permutations)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(p, cfg, table, K)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
