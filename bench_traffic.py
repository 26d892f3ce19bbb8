#!/usr/bin/env python3
"""HBM traffic per launch of the library's kernels from two rocprofv3 counter runs.

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d DIR1 -o t -- python3 bench.py --pmc-calib ...
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d DIR2 -o t -- python3 bench.py --pmc-calib ...
    python3 bench_traffic.py --workload NAME DIR1/t_counter_collection.csv DIR2/t_counter_collection.csv

Both counters are in KiB per dispatch.  They are scaled by what the same counter reads for the
plain elementwise copy (dst = src + 1 over 256 MiB of int32) that `bench.py --pmc-calib` runs
first: it reads 256 MiB and writes 256 MiB.  Writes profiles/traffic.json (bytes per call of owq_linear, summed over the kernels
of one call and averaged over the layers of the workload) and prints a short table.
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import os

ROOT = os.path.dirname(os.path.abspath(__file__))
CALIB_BYTES = 256 << 20


def read(path, counter):
    per_kernel = collections.OrderedDict()
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        per_kernel.setdefault(r["Kernel_Name"], []).append((int(r["Grid_Size"]), float(r["Counter_Value"])))
    return per_kernel


def summarize(path, counter):
    k = read(path, counter)
    # the calibration copies: the only elementwise kernels of the run that move this much
    copies = [v for name, vals in k.items() if "elementwise" in name.lower()
              for g, v in vals if v >= CALIB_BYTES / 1024.0 / 8]
    if not copies:
        raise SystemExit(f"{path}: no calibration copy found (run bench.py with --pmc-calib)")
    copy_kib = sorted(copies)[len(copies) // 2]
    factor = CALIB_BYTES / 1024.0 / copy_kib
    ours = {name: [v for _, v in vals] for name, vals in k.items() if "owq" in name}
    return factor, copy_kib, ours


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("fetch_csv")
    ap.add_argument("write_csv")
    ap.add_argument("--workload", required=True)
    ap.add_argument("--calls", type=int, required=True, help="owq_linear calls the profiled run made (steps+warmup) x layers")
    ap.add_argument("--algorithmic-bytes", type=int, default=0, help="algorithmic bytes per call, for the table")
    args = ap.parse_args()
    total = 0.0
    lines = []
    for path, counter in ((args.fetch_csv, "FETCH_SIZE"), (args.write_csv, "WRITE_SIZE")):
        factor, copy_kib, ours = summarize(path, counter)
        lines.append(f"{counter}: 256 MiB copy reads as {copy_kib:.0f} KiB -> scale factor {factor:.4f}")
        for name, vals in ours.items():
            per_call = sum(vals) * 1024.0 * factor / args.calls
            total += per_call
            short = name.replace("(anonymous namespace)::", "").split("(")[0]
            lines.append(f"  {short[:60]:60s} {len(vals):5d} dispatches, {sum(vals) / len(vals):10.1f} KiB each (raw)"
                         f" -> {per_call / 1e6:8.3f} MB per call of owq_linear")
    lines.append(f"HBM traffic per call of owq_linear: {total / 1e6:.3f} MB"
                 + (f" (algorithmic {args.algorithmic_bytes / 1e6:.3f} MB, ratio {total / args.algorithmic_bytes:.3f})"
                    if args.algorithmic_bytes else ""))
    print("\n".join(lines))
    path = os.path.join(ROOT, "profiles", "traffic.json")
    data = json.load(open(path)) if os.path.exists(path) else {}
    data[args.workload] = int(round(total))
    json.dump(data, open(path, "w"), indent=1, sort_keys=True)


if __name__ == "__main__":
    main()
