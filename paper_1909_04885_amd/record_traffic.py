"""Measured memory traffic of the local pass, stored next to the kernel sources it was measured on.

`hbm_traffic.json` holds, per kernel of the local pass (the kernel that takes the coordinate steps and,
for the blocked solver, the Gram-tile kernel), the bytes that crossed between L2 and the fabric per
launch: rocprofv3's FETCH_SIZE and WRITE_SIZE counters, each scaled by what the same counter shows for
a plain device copy of known size, together with a hash of `csrc/`.  bench.py reports the figures as
`roofline.traffic` only while that hash still matches the sources in the tree.
"""
from __future__ import annotations

import glob
import hashlib
import json
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
TRAFFIC_FILE = os.path.join(_HERE, "hbm_traffic.json")


def source_hash() -> str:
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(_HERE, "csrc", "*"))):
        h.update(os.path.basename(path).encode())
        h.update(open(path, "rb").read())
    return h.hexdigest()


def stored_traffic(workload: str):
    """{"kernels": {name: bytes per launch}, "local_pass_bytes": their sum} if measured on exactly these
    sources for this workload, else None."""
    try:
        rec = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        return None
    if rec.get("workload") != workload or rec.get("source_sha256") != source_hash() or "kernels" not in rec:
        return None
    return {"kernels": rec["kernels"], "local_pass_bytes": rec["local_pass_bytes"]}
