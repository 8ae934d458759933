"""Turn two rocprofv3 counter runs of bench.py into measured_traffic.json.

Usage (after the two runs described below, from the repository root):
    python -m paper_2003_08646_amd.traffic_from_pmc FETCH.csv WRITE.csv cfg2_n128_c64_k64_32

The runs (one counter each, the program directly after `--`):
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d OUT1 -o pmc -- \
        python3 bench.py --steps 3 --warmup 1 --no-cpu-baseline --copy-calibration
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d OUT2 -o pmc -- \
        python3 bench.py --steps 3 --warmup 1 --no-cpu-baseline --copy-calibration
FETCH.csv / WRITE.csv are their pmc_counter_collection.csv files.

Both counters report KiB per dispatch.  Their scale is taken from the 256 MiB device copy that
`--copy-calibration` runs (the largest-grid elementwise kernel in the trace): factor = known KiB /
reading, applied to the readings of the library's kernels.  bench.py reports fetch + write of its
dominant kernel as `roofline.traffic`.
"""
from __future__ import annotations

import collections
import csv
import json
import os
import sys

COPY_KIB = 256 * 1024  # bytes read (and written) by the calibration copy, in KiB

# kernel symbol fragment -> bench.py's kernel label
LABELS = {"input_range_kernel": "range_pass", "range_finalize_kernel": "range_reduce",
          "input_kernel": "quantize_pass", "gemm_fused": "gemm_epilogue",
          "conv_fused_c64_kernel": "quantize_gemm_epilogue"}


def read(path, counter):
    per = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] == counter:
            per[r["Kernel_Name"]].append(float(r["Counter_Value"]))
    return per


def copy_reading(per):
    cands = [(max(v), k) for k, v in per.items() if "elementwise" in k or "copy" in k.lower()]
    if not cands:
        raise SystemExit("no calibration copy kernel in the trace (run with --copy-calibration)")
    return max(cands)[0]


def main(argv):
    fetch_csv, write_csv, workload = argv[1:4]
    fetch, write = read(fetch_csv, "FETCH_SIZE"), read(write_csv, "WRITE_SIZE")
    ff, wf = COPY_KIB / copy_reading(fetch), COPY_KIB / copy_reading(write)
    out = {}
    for frag, label in LABELS.items():
        fk = [k for k in fetch if frag in k and "lance" in k]
        if not fk:
            continue
        k = fk[0]
        fv = sum(fetch[k]) / len(fetch[k])
        wv = sum(write[k]) / len(write[k]) if k in write else 0.0
        out[label] = {"kernel": k.replace("(anonymous namespace)::", "").split("(")[0], "fetch_bytes": round(fv * ff * 1024),
                      "write_bytes": round(wv * wf * 1024),
                      "fetch_kib_raw": fv, "write_kib_raw": wv}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "measured_traffic.json")
    try:
        rec = json.load(open(path))
    except (OSError, ValueError):
        rec = {}
    rec[workload] = out
    rec.setdefault("_calibration", {})[workload] = {"fetch_factor": ff, "write_factor": wf,
                                                    "copy_kib": COPY_KIB}
    json.dump(rec, open(path, "w"), indent=1, sort_keys=True)
    print(json.dumps(rec[workload], indent=1))


if __name__ == "__main__":
    main(sys.argv)
