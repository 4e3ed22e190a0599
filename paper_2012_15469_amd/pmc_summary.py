"""Turns two rocprofv3 counter runs of bench.py into the HBM traffic of the single-pass kernel.

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d DIR_F -- python3 bench.py --steps 3 --warmup 1 \\
        --no-cpu-baseline --others '' --plain-launch --pmc-calibration
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d DIR_W -- python3 bench.py --steps 3 --warmup 1 \\
        --no-cpu-baseline --others '' --plain-launch --pmc-calibration
    python -m paper_2012_15469_amd.pmc_summary DIR_F DIR_W cfg3_logreg_p65536_cada2 > profiles/..._traffic.json

FETCH_SIZE / WRITE_SIZE count in KiB per dispatch.  Each is scaled by what the same counter reads
for the calibration kernel of the same run (an elementwise pass that reads 1 GiB and writes
1 GiB), so that a counter that under- or over-reports by a constant factor cancels.
"""
from __future__ import annotations

import csv
import glob
import hashlib
import json
import os
import sys

GIB = float(1 << 30)


def _rows(d):
    for path in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
        with open(path, newline="") as f:
            yield from csv.DictReader(f)


def _mean_counter(d, counter, match, largest_only=False):
    vals = [float(r["Counter_Value"]) for r in _rows(d)
            if r["Counter_Name"] == counter and match(r["Kernel_Name"])]
    if not vals:
        raise SystemExit("no %s rows for the requested kernel under %s" % (counter, d))
    if largest_only:      # the calibration pass is by far the largest elementwise kernel of the run
        vals = [v for v in vals if v > 0.5 * max(vals)]
    return sum(vals) / len(vals), len(vals)


def main(argv):
    dir_f, dir_w, workload = argv[1:4]
    is_fused = lambda n: "k_fused<" in n          # (not k_fused_tail, the small kernel that adds up a split last round)
    is_cal = lambda n: "elementwise_kernel" in n
    out = {"workload": workload}
    total = 0.0
    for d, counter, key in ((dir_f, "FETCH_SIZE", "fetch"), (dir_w, "WRITE_SIZE", "write")):
        k, nk = _mean_counter(d, counter, is_fused)
        c, nc = _mean_counter(d, counter, is_cal, largest_only=True)
        factor = GIB / (c * 1024.0)            # true bytes per counted byte
        out[key] = {"counter_kib_per_launch": k, "launches": nk, "calibration_kib": c, "calibration_launches": nc,
                    "scale_factor": factor, "bytes_per_launch": k * 1024.0 * factor}
        total += k * 1024.0 * factor
    out["hbm_bytes_per_launch"] = total
    here = os.path.dirname(os.path.abspath(__file__))
    src = os.path.join(here, "csrc", "cada_logreg_fused.hip")
    # the kernel is everything above the host-side planning code of that file
    text = open(src).read().split("// Chooses the cluster geometry")[0]
    out["kernel_source_sha256"] = hashlib.sha256(text.encode()).hexdigest()
    json.dump(out, sys.stdout, indent=1)
    print()


if __name__ == "__main__":
    main(sys.argv)
