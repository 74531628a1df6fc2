"""Turns two rocprofv3 --pmc runs of bench.py (FETCH_SIZE, WRITE_SIZE; both with
--calibrate-copy) into per-kernel HBM bytes per launch.

The counters are scaled by what they read for the plain 1 GiB device copy that
bench.py --calibrate-copy issues (reads 1 GiB, writes 1 GiB).  Usage:

  python -m paper_2408_10284_amd.pmc_summary FETCH_DIR WRITE_DIR OUT.json

where each DIR holds bench_counter_collection.csv.  bench.py reports the figure
of its dominant kernel as roofline.traffic when OUT.json is profiles/pmc_traffic.json.
"""
from __future__ import annotations

import collections
import csv
import json
import os
import sys

COPY_BYTES = 1 << 30


def _load(path, counter):
    rows = list(csv.DictReader(open(os.path.join(path, "bench_counter_collection.csv"))))
    per = collections.defaultdict(list)
    for r in rows:
        if r["Counter_Name"] == counter:
            per[r["Kernel_Name"]].append(float(r["Counter_Value"]))
    return per


def _copy_reference(per):
    # the calibration copy is the largest dispatch of a copy kernel
    best = None
    for name, vals in per.items():
        if "copy" in name.lower():
            m = max(vals)
            if best is None or m > best:
                best = m
    if not best:
        raise SystemExit("no copy kernel found: run bench.py with --calibrate-copy")
    return best


def summarise(fetch_dir, write_dir):
    fetch, write = _load(fetch_dir, "FETCH_SIZE"), _load(write_dir, "WRITE_SIZE")
    f_factor = COPY_BYTES / _copy_reference(fetch)     # bytes per counter unit
    w_factor = COPY_BYTES / _copy_reference(write)
    out = {"calibration": {"copy_bytes_each_way": COPY_BYTES, "fetch_bytes_per_unit": f_factor, "write_bytes_per_unit": w_factor},
           "kernels": {}}
    for name in fetch:
        if "adapmoe::" not in name:
            continue
        fv, wv = fetch[name], write.get(name, [0.0])
        out["kernels"][name] = {
            "launches": len(fv),
            "fetch_bytes_per_launch": sum(fv) / len(fv) * f_factor,
            "write_bytes_per_launch": sum(wv) / len(wv) * w_factor,
            "fetch_bytes_max": max(fv) * f_factor,
        }
    return out


if __name__ == "__main__":
    if len(sys.argv) != 4:
        raise SystemExit(__doc__)
    res = summarise(sys.argv[1], sys.argv[2])
    with open(sys.argv[3], "w") as f:
        json.dump(res, f, indent=1)
    for k, v in res["kernels"].items():
        print(f"{k[:70]:70s} fetch {v['fetch_bytes_per_launch'] / 1e6:9.2f} MB  write {v['write_bytes_per_launch'] / 1e6:7.3f} MB  ({v['launches']} launches)")
