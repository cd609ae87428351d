"""Writes profiles/traffic.json: HBM bytes per launch of each workload's worker pass, from
rocprofv3 byte counters.

Recipe (one counter per run; see any file under profiles/ for the full commands):

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d OUT_F -o NAME -- \\
        python3 bench.py --workload NAME --others "" --no-cpu-baseline --no-modes --steps 3 --warmup 1 --calib-copy
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d OUT_W -o NAME -- (the same command)
    python -m paper_1905_05957_amd.traffic --workload NAME --fetch OUT_F/NAME_counter_collection.csv \\
        --write OUT_W/NAME_counter_collection.csv --kernel SUBSTRING [--kernel ...] --commit $(git rev-parse --short HEAD)

Both counters are in KiB per dispatch and are scaled by what the same counter reads for the
1 GiB device copy that `--calib-copy` adds to the run (1,048,576 KiB read and written).  Per
--kernel substring the largest dispatch of the run's last step counts (a kernel that serves the
worker and the server call does more for the workers); the worker pass is their sum.
bench.py reports that figure as roofline.traffic.
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COPY_KIB = 1048576.0


def _per_kernel(path: str):
    rows = sorted(csv.DictReader(open(path)), key=lambda r: int(r["Dispatch_Id"]))
    agg = collections.defaultdict(list)
    for r in rows:
        agg[r["Kernel_Name"]].append(float(r["Counter_Value"]))
    return agg


def _calibration(agg) -> float:
    copies = [max(v) for k, v in agg.items() if "copyBuffer" in k]
    if not copies:
        raise SystemExit("no calibration copy in the counter file: run bench.py with --calib-copy")
    return COPY_KIB / max(copies)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", required=True)
    ap.add_argument("--fetch", required=True)
    ap.add_argument("--write", required=True)
    ap.add_argument("--kernel", action="append", required=True, help="substring of a kernel name of the worker call")
    ap.add_argument("--commit", default="")
    ap.add_argument("--steps-in-run", type=int, default=4, help="steps the profiled run made (warm-up included)")
    a = ap.parse_args()
    f, w = _per_kernel(a.fetch), _per_kernel(a.write)
    sf, sw = _calibration(f), _calibration(w)
    kernels, total = {}, 0.0
    for pat in a.kernel:
        def last_step_max(agg):
            vals = [v[-max(1, len(v) // a.steps_in_run):] for k, v in agg.items() if pat in k]
            return max(max(v) for v in vals) if vals else 0.0
        rd, wr = last_step_max(f) * sf * 1024.0, last_step_max(w) * sw * 1024.0
        kernels[pat] = {"read_bytes": round(rd), "written_bytes": round(wr)}
        total += rd + wr
    path = os.path.join(ROOT, "profiles", "traffic.json")
    table = {}
    if os.path.exists(path):
        with open(path) as fh:
            table = json.load(fh)
    table[a.workload] = {"worker_call_bytes": round(total), "kernels": kernels, "fetch_scale": round(sf, 4),
                         "write_scale": round(sw, 4), "commit": a.commit}
    with open(path, "w") as fh:
        json.dump(table, fh, indent=1, sort_keys=True)
        fh.write("\n")
    print(json.dumps(table[a.workload]))


if __name__ == "__main__":
    main()
