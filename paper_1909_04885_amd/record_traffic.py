"""Store the measured HBM traffic of the local pass's chain kernel next to the sources it was measured on.

    python -m paper_1909_04885_amd.record_traffic FETCH_DB WRITE_DB [--workload sparse_zipf/full]

FETCH_DB / WRITE_DB are the result databases of two counter runs of bench.py with --calibrate-copy,
    rocprofv3 --pmc FETCH_SIZE -d DIR -o f -- python3 bench.py --steps 3 --warmup 1 --no-cpu-baseline --no-time-to-gap --calibrate-copy
    rocprofv3 --pmc WRITE_SIZE -d DIR -o w -- python3 bench.py --steps 3 --warmup 1 --no-cpu-baseline --no-time-to-gap --calibrate-copy
Each counter (KiB per dispatch) is scaled by what it shows for the known 1 GiB device copy of
--calibrate-copy.  The result goes to hbm_traffic.json together with a hash of the kernel sources;
bench.py reports it as roofline.traffic only while that hash still matches.
"""
from __future__ import annotations

import argparse
import glob
import hashlib
import json
import os
import sqlite3

_HERE = os.path.dirname(os.path.abspath(__file__))
TRAFFIC_FILE = os.path.join(_HERE, "hbm_traffic.json")
CHAIN_KERNEL = "sdca_batched_csr"
GIB_KIB = 1048576.0


def source_hash() -> str:
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(_HERE, "csrc", "*"))):
        h.update(os.path.basename(path).encode())
        h.update(open(path, "rb").read())
    return h.hexdigest()


def _counter(db: str, name: str):
    c = sqlite3.connect(db)
    cols = [r[1] for r in c.execute("pragma table_info(counters_collection)")]
    kn = "kernel_name" if "kernel_name" in cols else "name"
    rows = list(c.execute("select %s, value from counters_collection where counter_name = ?" % kn, (name,)))
    chain = [v for k, v in rows if CHAIN_KERNEL in k]
    copies = [v for k, v in rows if "copyBuffer" in k]
    if not chain or not copies:
        raise SystemExit("%s: no %s dispatches or no calibration copy in %s" % (name, CHAIN_KERNEL, db))
    return sum(chain) / len(chain), max(copies)


def stored_traffic(workload: str):
    """HBM bytes per launch of the chain kernel if measured on exactly these sources, else None."""
    try:
        rec = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        return None
    if rec.get("workload") != workload or rec.get("source_sha256") != source_hash():
        return None
    return rec.get("hbm_bytes_per_launch")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("fetch_db")
    ap.add_argument("write_db")
    ap.add_argument("--workload", default="sparse_zipf/full")
    a = ap.parse_args()
    fetch, fetch_copy = _counter(a.fetch_db, "FETCH_SIZE")
    write, write_copy = _counter(a.write_db, "WRITE_SIZE")
    fs, ws = GIB_KIB / fetch_copy, GIB_KIB / write_copy
    rec = {"workload": a.workload, "kernel": CHAIN_KERNEL, "fetch_kib": fetch, "write_kib": write,
           "fetch_scale": fs, "write_scale": ws,
           "hbm_bytes_per_launch": 1024.0 * (fetch * fs + write * ws), "source_sha256": source_hash()}
    json.dump(rec, open(TRAFFIC_FILE, "w"), indent=1)
    print(json.dumps(rec))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
