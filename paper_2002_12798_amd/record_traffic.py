"""Turn four rocprofv3 --pmc counter runs into profiles/traffic_<workload>.json.

Usage:  python -m paper_2002_12798_amd.record_traffic <dir> [workload]

<dir> must hold the csv output of (see profiles/*_hbm_traffic.md for the commands)
    fused-only_FETCH_SIZE, copy-only_FETCH_SIZE, fused-only_WRITE_SIZE, copy-only_WRITE_SIZE
i.e. `bench.py --fused-only` and `bench.py --copy-only` each under `--pmc FETCH_SIZE` and
`--pmc WRITE_SIZE`.  The copy run moves a known number of bytes and scales the counters.
"""
from __future__ import annotations

import csv
import hashlib
import json
import os
import statistics
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCES = ["paper_2002_12798_amd/csrc/amap_kernels.hip", "paper_2002_12798_amd/csrc/amap_index.hpp", "paper_2002_12798_amd/csrc/amap_compose.cpp",
           "paper_2002_12798_amd/csrc/amap_plan.cpp", "paper_2002_12798_amd/csrc/amap_device.hpp"]
COPY_BYTES = 106496000  # read and written per launch of `bench.py --copy-only`


def mean_kib(d, tag, counter):
    rows = csv.DictReader(open(os.path.join(d, f"{tag}_{counter}_counter_collection.csv")))
    v = [float(r["Counter_Value"]) for r in rows if "amap_pieces" in r["Kernel_Name"] and r["Counter_Name"] == counter]
    return statistics.mean(v), len(v)


def main():
    d = sys.argv[1]
    workload = sys.argv[2] if len(sys.argv) > 2 else "cfg1"
    ff, nf = mean_kib(d, "fused-only", "FETCH_SIZE")
    fc, _ = mean_kib(d, "copy-only", "FETCH_SIZE")
    wf, _ = mean_kib(d, "fused-only", "WRITE_SIZE")
    wc, _ = mean_kib(d, "copy-only", "WRITE_SIZE")
    fetch_factor, write_factor = COPY_BYTES / (fc * 1024), COPY_BYTES / (wc * 1024)
    h = hashlib.sha256()
    for f in SOURCES:
        h.update(open(os.path.join(ROOT, f), "rb").read())
    rec = {
        "workload": workload, "dispatches": nf, "sources": SOURCES, "sources_sha256": h.hexdigest(),
        "fetch_kib_fused": ff, "fetch_kib_copy": fc, "write_kib_fused": wf, "write_kib_copy": wc,
        "fetch_factor": fetch_factor, "write_factor": write_factor,
        "read_bytes_per_launch": ff * 1024 * fetch_factor, "write_bytes_per_launch": wf * 1024 * write_factor,
    }
    rec["traffic_bytes_per_launch"] = rec["read_bytes_per_launch"] + rec["write_bytes_per_launch"]
    out = os.path.join(ROOT, "profiles", f"traffic_{workload}.json")
    json.dump(rec, open(out, "w"), indent=1)
    print(json.dumps(rec, indent=1))


if __name__ == "__main__":
    main()
