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


def algorithmic_bytes(p, table, K):
    """Bytes the local pass must move per launch: the matrix once, the per-row state once, and each
    solver's touched part of its private vector in and out once (cache traffic is not counted).
    CSR: 8 B per entry + 24 B per row (row offset, order entry, label, norm, alpha read and write)
    + 8 B per distinct column a solver touches.  Dense: 4 B per entry + 20 B per row + 8 B per column
    per solver."""
    if p.dense:
        return 4 * p.nnz + 20 * p.n + 8 * p.d * K
    touched = 0
    for k in range(K):
        seen = np.zeros(p.d, dtype=bool)
        for c in np.nonzero(table == k)[0]:
            r0, r1 = p.chunk_rows(c)
            seen[p.col[p.row_ptr[r0]:p.row_ptr[r1]]] = True
        touched += int(seen.sum())
    return 8 * p.nnz + 24 * p.n + 8 * touched


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
    return {"value": p.nnz * rounds / spent, "unit": "nnz/s", "cores": 1, "kind": "oracle",
            "sample": "%d whole rounds of the same workload (local pass + aggregate + gap), %.1f s" % (rounds, spent)}


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
    total = args.warmup + args.steps
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
    seg_ms = {"local_epoch": [], "aggregate": [], "gap": [], "epoch_gram": [], "epoch_chain": []}
    gaps = []
    t_start = time.perf_counter()
    for r in range(args.warmup, total):
        g.local_epoch_ahead(cur(r), nxt(r))       # announces the next round's orders (all are in HBM)
        g.aggregate()
        gaps.append(g.gap()[2])          # synchronises: the three scalars come back to the host
        for s in seg_ms:                  # events of this round have completed
            try:
                seg_ms[s].append(g.last_kernel_ms(s))
            except chicle.ChicleError:
                pass                      # segment not part of this solver kind
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start

    ms_per_step = elapsed * 1e3 / args.steps
    epoch_ms = float(np.mean(seg_ms["local_epoch"]))
    agg_ms = float(np.mean(seg_ms["aggregate"]))
    gap_ms = float(np.mean(seg_ms["gap"]))
    abytes = algorithmic_bytes(p, table, K)
    achieved = abytes / (epoch_ms * 1e-3) / 1e9
    agg_bytes = 4 * p.d * (2 * K + 2)
    gap_bytes = (8 if not p.dense else 4) * p.nnz + 12 * p.n + 4 * p.d
    out = {
        "metric": "nnz_per_s_per_cocoa_round",
        "value": p.nnz * args.steps / elapsed,
        "unit": "nnz/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s/%s" % (args.workload, args.size), "n": p.n, "d": p.d, "entries": p.nnz,
                   "K": K, "chunk_rows": cfg["chunk_rows"], "lambda": cfg["lam"], "loss": p.loss,
                   "solver": args.solver},
        "local_epoch": {"ms": epoch_ms, "nnz_per_s": p.nnz / (epoch_ms * 1e-3),
                        "coord_updates_per_s": p.n / (epoch_ms * 1e-3),
                        "gram_ms": float(np.mean(seg_ms["epoch_gram"])) if seg_ms["epoch_gram"] else None,
                        "chain_ms": float(np.mean(seg_ms["epoch_chain"])) if seg_ms["epoch_chain"] else None,
                        # the dependency chain: a solver's coordinate steps come one after the other
                        "max_rows_per_solver": int(max(rows)),
                        "ns_per_step_of_longest_solver": epoch_ms * 1e6 / max(int(max(rows)), 1)},
        "aggregate": {"ms": agg_ms, "GB_per_s": agg_bytes / (agg_ms * 1e-3) / 1e9,
                      "frac_hbm_peak": agg_bytes / (agg_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "gap": {"ms": gap_ms, "GB_per_s": gap_bytes / (gap_ms * 1e-3) / 1e9,
                "frac_hbm_peak": gap_bytes / (gap_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "first": gaps[0], "last": gaps[-1]},
        "roofline": {"kernel": "local_epoch", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     # measured HBM bytes per launch of the chain kernel; null unless they were taken on
                     # exactly these kernel sources (paper_1909_04885_amd/record_traffic.py)
                     "traffic": stored_traffic("%s/%s" % (args.workload, args.size)) if args.solver == "auto" else None,
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
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(p, cfg, table, K)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
