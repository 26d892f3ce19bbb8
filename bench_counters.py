#!/usr/bin/env python3
"""Per-kernel means of the hardware counters of one or more rocprofv3 --pmc runs.

    rocprofv3 --pmc SQ_WAVES SQ_INSTS_VALU ... --output-format csv -d DIR -o t -- python3 bench.py ...
    python3 bench_counters.py DIR/t_counter_collection.csv [more.csv ...] [--match owq]

Prints, for every kernel whose name contains --match, the number of dispatches and the mean of
each counter per dispatch (a counter rocprofv3 reports per shader engine or per die is summed
over them first, as its csv has one row per dispatch and counter)."""
from __future__ import annotations

import argparse
import collections
import csv


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("csv", nargs="+")
    ap.add_argument("--match", default="owq")
    args = ap.parse_args()
    for path in args.csv:
        acc = collections.OrderedDict()                     # kernel -> counter -> {dispatch id: value}
        for r in csv.DictReader(open(path)):
            if args.match not in r["Kernel_Name"]:
                continue
            per = acc.setdefault(r["Kernel_Name"], collections.OrderedDict()).setdefault(r["Counter_Name"], {})
            per[r["Dispatch_Id"]] = per.get(r["Dispatch_Id"], 0.0) + float(r["Counter_Value"])
        print(path)
        for name, counters in acc.items():
            short = name.split("(")[0].replace("void ", "")
            n = len(next(iter(counters.values())))
            print(f"  {short}: {n} dispatches")
            for c, vals in counters.items():
                v = sorted(vals.values())
                print(f"    {c:44s} mean {sum(v) / len(v):16.1f}   median {v[len(v) // 2]:16.1f}")


if __name__ == "__main__":
    main()
