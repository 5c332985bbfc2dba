"""Turns two rocprofv3 --pmc runs of bench.py (FETCH_SIZE, then WRITE_SIZE) into the HBM traffic
summary bench.py quotes in its roofline object.

    python -m paper_2510_11062_amd.traffic_from_pmc FETCH.csv WRITE.csv WORKLOAD OUT.json

Both runs must use `bench.py --calibration-copy`: the torch copy of 1 GiB (1 GiB read, 1 GiB
written) that ends the run gives the factor between a counter's reading and bytes, which is applied
to the head kernels' readings.  Per kernel, launches whose duration shows they had no rows are
dropped and the rest averaged.  The summary records a digest of the HIP sources; bench.py reports
the traffic only while the sources still match it.
"""
from __future__ import annotations

import csv
import json
import os
import sys
from collections import defaultdict

GIB = float(1 << 30)
HEAD_KERNELS = ("k_head_fwd", "k_head_dz", "k_head_dh", "k_head_dw", "k_head_dw_km")


def read_counter(path, counter):
    """{dispatch id: (kernel name, counter value summed over the rows of that dispatch, duration ns)}"""
    out = {}
    acc = defaultdict(float)
    meta = {}
    for row in csv.DictReader(open(path)):
        if row["Counter_Name"] != counter:
            continue
        d = row["Dispatch_Id"]
        acc[d] += float(row["Counter_Value"])
        meta[d] = (row["Kernel_Name"], float(row["End_Timestamp"]) - float(row["Start_Timestamp"]))
    for d, v in acc.items():
        out[d] = (meta[d][0], v, meta[d][1])
    return out


def summarise(path, counter):
    disp = read_counter(path, counter)
    # calibration: the largest copy kernel of the run is the 1 GiB one (1 GiB read, 1 GiB written)
    copies = [v for (name, v, _) in disp.values() if "copy" in name.lower() and v > 0]
    if not copies:
        raise SystemExit(f"no copy kernel found in {path}")
    cal_reading = max(copies)
    scale = GIB / cal_reading                      # bytes per counter unit
    per_kernel = {}
    for sym in HEAD_KERNELS:
        rows = [(v, dur) for (name, v, dur) in disp.values() if sym + "<" in name or sym + "(" in name]
        if not rows:
            continue
        longest = max(dur for _, dur in rows)
        working = [v for v, dur in rows if dur > 0.02 * longest]
        per_kernel[sym] = {"launches": len(working), "bytes_per_launch": scale * sum(working) / len(working)}
    return scale, cal_reading, per_kernel


def main():
    fetch_csv, write_csv, workload, out_path = sys.argv[1:5]
    f_scale, f_cal, f_k = summarise(fetch_csv, "FETCH_SIZE")
    w_scale, w_cal, w_k = summarise(write_csv, "WRITE_SIZE")
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import bench
    kernels = {}
    for sym in f_k:
        if sym not in w_k:
            continue
        kernels[sym if sym != "k_head_dw_km" else "k_head_dw"] = {
            "launches_with_rows": f_k[sym]["launches"],
            "fetch_bytes_per_launch": f_k[sym]["bytes_per_launch"],
            "write_bytes_per_launch": w_k[sym]["bytes_per_launch"],
            "hbm_bytes_per_launch": f_k[sym]["bytes_per_launch"] + w_k[sym]["bytes_per_launch"],
        }
    commands = [
        "cd /tmp && export TMPDIR=/tmp",
        f"rocprofv3 --pmc FETCH_SIZE -d <out>/pmc_fetch -o f --output-format csv -- python3 bench.py --config {workload} "
        "--steps 1 --warmup 0 --cpu-sample 0 --calibration-copy",
        f"rocprofv3 --pmc WRITE_SIZE -d <out>/pmc_write -o w --output-format csv -- python3 bench.py --config {workload} "
        "--steps 1 --warmup 0 --cpu-sample 0 --calibration-copy",
        f"python3 -m paper_2510_11062_amd.traffic_from_pmc <out>/pmc_fetch/f_counter_collection.csv "
        f"<out>/pmc_write/w_counter_collection.csv {workload} profiles/hbm_traffic_{workload}.txt",
    ]
    rec = {"what": "bytes between L2 and the memory fabric per launch of each head kernel (launches with rows "
                   "only), from rocprofv3 counters scaled by a 1 GiB copy in the same run",
           "commands": commands,
           "workload": workload, "source_digest": bench.kernel_source_digest(),
           "calibration": {"copy_bytes_each_way": GIB, "FETCH_SIZE_reading": f_cal, "bytes_per_FETCH_SIZE_unit": f_scale,
                           "WRITE_SIZE_reading": w_cal, "bytes_per_WRITE_SIZE_unit": w_scale},
           "kernels": kernels}
    json.dump(rec, open(out_path, "w"), indent=1)
    print(json.dumps(rec, indent=1))


if __name__ == "__main__":
    main()
