#!/usr/bin/env python3
"""Turn two rocprofv3 counter runs of bench.py into measured HBM traffic per kernel launch.

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <dir_f> -- python3 bench.py ... --calibration-copy
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <dir_w> -- python3 bench.py ... --calibration-copy
    python3 paper_2510_00932_amd/record_traffic.py <dir_f> <dir_w> <workload name>

Each counter is scaled by what it reads for the calibration copy of that same run: a
plain device-to-device copy of exactly 1 GiB (1 GiB fetched, 1 GiB written).  The result,
with a digest of the kernel sources it belongs to, goes to measured_traffic.json next to
this file; bench.py reports it as roofline.traffic only while the digest still matches.
A text summary is printed on stdout.
"""
import csv
import glob
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
CAL_BYTES = 1 << 30
CAL_KERNEL = "__amd_rocclr_copyBuffer"
# kernel names as rocprofv3 prints them; the elementwise and the dot first-pass kernels exist in an
# index-ordered / tiled and a paced form, of which a run uses one per workload
KERNEL_KEYS = (("copy", "stream_kernel", "(opal::Op)0"), ("scale", "stream_kernel", "(opal::Op)1"),
               ("add", "stream_kernel", "(opal::Op)2"), ("triad", "stream_kernel", "(opal::Op)3"),
               ("dot", "dot_", "_kernel"), ("dot_final", "dot_final_kernel", ""))


def source_digest():
    from paper_2510_00932_amd.build import kernel_source_digest
    return kernel_source_digest()


def per_kernel(dirname, counter):
    files = glob.glob(os.path.join(dirname, "**", "*counter_collection.csv"), recursive=True)
    if len(files) != 1:
        raise SystemExit("expected one counter_collection.csv under %s, found %d" % (dirname, len(files)))
    vals = {}
    with open(files[0]) as f:
        for row in csv.DictReader(f):
            if row["Counter_Name"] == counter:
                vals.setdefault(row["Kernel_Name"], []).append(float(row["Counter_Value"]))
    return vals


def pick(vals, *needles):
    hits = [v for k, v in vals.items() if all(x in k for x in needles)
            and not (needles[0] == "dot_" and "dot_final" in k)]
    if len(hits) != 1:
        raise SystemExit("kernel %r: expected one match, found %d" % (needles, len(hits)))
    return sum(hits[0]) / len(hits[0]), len(hits[0])


def main():
    if len(sys.argv) != 4:
        raise SystemExit(__doc__)
    fetch, write = per_kernel(sys.argv[1], "FETCH_SIZE"), per_kernel(sys.argv[2], "WRITE_SIZE")
    workload = sys.argv[3]
    cal_f, _ = pick(fetch, CAL_KERNEL)
    cal_w, _ = pick(write, CAL_KERNEL)
    bytes_per_fetch_unit = CAL_BYTES / cal_f
    bytes_per_write_unit = CAL_BYTES / cal_w
    print("calibration copy of %d bytes: FETCH_SIZE reads %.1f, WRITE_SIZE reads %.1f" % (CAL_BYTES, cal_f, cal_w))
    print("=> one FETCH_SIZE unit = %.2f bytes, one WRITE_SIZE unit = %.2f bytes" % (bytes_per_fetch_unit, bytes_per_write_unit))
    print("%-10s %14s %14s %16s %16s %16s %9s" % ("kernel", "FETCH_SIZE", "WRITE_SIZE", "fetched bytes", "written bytes",
                                                   "HBM bytes", "launches"))
    out = {}
    for name, *needles in KERNEL_KEYS:
        f_avg, nf = pick(fetch, *needles)
        w_avg, _ = pick(write, *needles)
        fb, wb = f_avg * bytes_per_fetch_unit, w_avg * bytes_per_write_unit
        out[name] = int(round(fb + wb))
        print("%-10s %14.1f %14.1f %16.0f %16.0f %16.0f %9d" % (name, f_avg, w_avg, fb, wb, fb + wb, nf))
    out["dot"] += out.pop("dot_final")
    path = os.path.join(HERE, "measured_traffic.json")
    rec = {"source_digest": source_digest(), "workloads": {}}
    if os.path.exists(path):
        with open(path) as f:
            old = json.load(f)
        if old.get("source_digest") == rec["source_digest"]:
            rec = old
    rec["workloads"][workload] = out
    rec["note"] = ("HBM bytes per launch: rocprofv3 FETCH_SIZE and WRITE_SIZE per dispatch, each scaled by its reading "
                   "for a 1 GiB device-to-device copy in the same run; dot = first pass + second pass")
    with open(path, "w") as f:
        json.dump(rec, f, indent=1, sort_keys=True)
        f.write("\n")
    print("wrote %s (source digest %s)" % (os.path.relpath(path, ROOT), rec["source_digest"]))


if __name__ == "__main__":
    main()
