"""Turn two rocprofv3 --pmc runs of bench.py (FETCH_SIZE, then WRITE_SIZE) into HBM bytes
per launch of the expert kernels and store them in measured_traffic.json, which bench.py
reports as roofline.traffic.

Usage (after the two profiling runs, each made with `--calibrate-copy`):
  python -m paper_2505_19645_amd.traffic_from_pmc <fetch_counter.csv> <write_counter.csv> <key>
key = "<preset>/B<B>/g<gamma>/skew<skew>" as bench.py builds it.

Both counters tick in units whose size is taken from a plain 1 GiB device copy in the same
run (1 GiB read, 1 GiB written): factor = 2^30 / counter value of one copy dispatch.  bench.py
makes that copy before anything else, so it is the first device-to-device copy of the run.
"""
from __future__ import annotations

import csv
import json
import os
import sys
from collections import defaultdict

HERE = os.path.dirname(os.path.abspath(__file__))
OUT = os.path.join(HERE, "measured_traffic.json")


def per_kernel(path, counter):
    """-> {kernel name: [counter values in dispatch order]}"""
    rows = []
    with open(path) as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] == counter:
                rows.append((int(r["Dispatch_Id"]), r["Kernel_Name"], float(r["Counter_Value"])))
    vals = defaultdict(list)
    for _, name, v in sorted(rows):
        vals[name].append(v)
    return vals


def pick(vals, needle):
    hits = [v for k, v in vals.items() if needle in k]
    if not hits:
        raise SystemExit(f"no kernel matching {needle!r}")
    return [x for v in hits for x in v]


def main():
    fetch_csv, write_csv, key = sys.argv[1:4]
    fetch = per_kernel(fetch_csv, "FETCH_SIZE")
    write = per_kernel(write_csv, "WRITE_SIZE")
    # the calibration copy: the first device-to-device copy of the run is bench.py's 1 GiB tensor
    # copy (torch issues it through the runtime's copy kernel); it is repeated three times
    f_copy = sorted(pick(fetch, "copyBuffer")[:3])[1]
    w_copy = sorted(pick(write, "copyBuffer")[:3])[1]
    f_unit, w_unit = 2.0 ** 30 / f_copy, 2.0 ** 30 / w_copy
    out = {"fetch_unit_bytes": f_unit, "write_unit_bytes": w_unit}
    for name, needle in (("gate_up", "expert_stream_kernel<0,"), ("down", "expert_stream_kernel<1,")):
        fv, wv = pick(fetch, needle), pick(write, needle)
        out[name] = {"fetch_bytes": sum(fv) / len(fv) * f_unit, "write_bytes": sum(wv) / len(wv) * w_unit,
                     "launches": len(fv)}
    data = {}
    if os.path.exists(OUT):
        with open(OUT) as f:
            data = json.load(f)
    data[key] = out
    with open(OUT, "w") as f:
        json.dump(data, f, indent=1, sort_keys=True)
    print(json.dumps(out, indent=1))


if __name__ == "__main__":
    main()
