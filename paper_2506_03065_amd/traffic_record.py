"""Writes profiles/traffic.json, the record bench.py reads roofline.traffic from.

Hardware counters cannot be read from inside the benchmark process.  The HBM
traffic of the dominant kernel therefore comes from two rocprofv3 runs of the
benchmark command (one with --pmc FETCH_SIZE, one with --pmc WRITE_SIZE, each
with --copy-calibration so that the run also holds one dispatch of the library's
streaming copy: 1 GiB read, 1 GiB written), and this module turns their CSV
output into the record:

    python -m paper_2506_03065_amd.traffic_record --bench-json RUN.json \\
        --fetch-csv FETCH/..._counter_collection.csv --write-csv WRITE/..._counter_collection.csv

RUN.json is the JSON line bench.py printed in one of the two runs; its
roofline.dispatches names the kernels of the dominant launch (name part and grid
size in work-items).  Both counters read KiB per dispatch; each is scaled by what
it reads for the copy (2^20 KiB moved each way), averaged over the matching
dispatches and summed over the kernels.  The record carries the hash of the
kernel sources it was measured on; bench.py ignores a record whose hash differs.
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COPY_KIB = float(1 << 20)


def read_counter(path, counter):
    """{(kernel name, grid size): [values]} of one counter."""
    out = collections.defaultdict(list)
    with open(path, newline="") as f:
        for row in csv.DictReader(f):
            if row["Counter_Name"] == counter:
                out[(row["Kernel_Name"], int(row["Grid_Size"]))].append(float(row["Counter_Value"]))
    return out


def average(values_by_kernel, name_part, grid_size=None):
    vals = [v for (name, grid), vs in values_by_kernel.items() if name_part in name and (grid_size is None or grid == grid_size)
            for v in vs]
    if not vals:
        raise SystemExit(f"no dispatch of '{name_part}' (grid {grid_size}) in the counter output")
    return sum(vals) / len(vals), len(vals)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--bench-json", required=True)
    ap.add_argument("--fetch-csv", required=True)
    ap.add_argument("--write-csv", required=True)
    ap.add_argument("--out", default=os.path.join(ROOT, "profiles", "traffic.json"))
    args = ap.parse_args()
    sys.path.insert(0, ROOT)
    import bench

    with open(args.bench_json) as f:
        run = json.loads([line for line in f.read().splitlines() if line.startswith("{")][-1])
    roofline = run["roofline"]
    fetch, write = read_counter(args.fetch_csv, "FETCH_SIZE"), read_counter(args.write_csv, "WRITE_SIZE")
    copy_fetch, _ = average(fetch, "copy_probe_kernel")
    copy_write, _ = average(write, "copy_probe_kernel")
    scale_fetch, scale_write = COPY_KIB / copy_fetch, COPY_KIB / copy_write
    kernels, total = [], 0.0
    for d in roofline["dispatches"]:
        f_kib, n = average(fetch, d["kernel"], d.get("grid_size"))
        w_kib, _ = average(write, d["kernel"], d.get("grid_size"))
        nbytes = (f_kib * scale_fetch + w_kib * scale_write) * 1024.0
        total += nbytes
        kernels.append({"kernel": d["kernel"], "grid_size": d.get("grid_size"), "dispatches_averaged": n,
                        "FETCH_SIZE_KiB": round(f_kib), "WRITE_SIZE_KiB": round(w_kib), "bytes": round(nbytes)})
    try:
        with open(args.out) as f:
            record = json.load(f)
    except (OSError, ValueError):
        record = {"note": "HBM bytes per launch of the dominant kernel(s) of a workload, from rocprofv3 --pmc FETCH_SIZE "
                          "and --pmc WRITE_SIZE runs of bench.py, written by paper_2506_03065_amd/traffic_record.py",
                  "records": {}}
    cfg = run["config"]
    entry = {"bytes": round(total), "kernels": kernels,
             "scale": {"FETCH_SIZE": round(scale_fetch, 4), "WRITE_SIZE": round(scale_write, 4),
                       "copy_FETCH_SIZE_KiB": round(copy_fetch), "copy_WRITE_SIZE_KiB": round(copy_write)},
             "kernel_source_stamp": bench.kernel_source_stamp(),
             "source": f"rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of bench.py --workload {cfg['workload']} "
                       f"--precision {cfg['precision']}, recorded {time.strftime('%Y-%m-%d')}"}
    record["records"].setdefault(cfg["precision"], {}).setdefault(cfg["workload"], {})[roofline["traffic_key"]] = entry
    with open(args.out, "w") as f:
        json.dump(record, f, indent=1, sort_keys=True)
        f.write("\n")
    print(f"{cfg['workload']} {cfg['precision']} {roofline['traffic_key']}: {total / 1e6:.1f} MB per launch "
          f"(scales {scale_fetch:.3f} / {scale_write:.3f})")


if __name__ == "__main__":
    main()
