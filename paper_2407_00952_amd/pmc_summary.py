"""Turn two rocprofv3 counter runs (FETCH_SIZE, WRITE_SIZE) of bench.py into the HBM-traffic summary.

Usage:
    python -m paper_2407_00952_amd.pmc_summary FETCH_counter_collection.csv WRITE_counter_collection.csv > summary.md

Both runs must have been made with `bench.py --copy-calibration`: the plain copy of known size at the end
(FedAvg with one client: 256 MiB read, 256 MiB written per launch) gives the factor that converts the
counter's unit into bytes.  The GEMM figure is the average over every launch of the bf16 GEMM kernel.
"""
from __future__ import annotations

import csv
import hashlib
import os
import sys

CAL_BYTES = 64 * 1024 * 1024 * 4


def per_kernel(path, counter):
    vals = {}
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        vals.setdefault(r["Kernel_Name"], []).append(float(r["Counter_Value"]))
    return vals


def main(fetch_csv, write_csv):
    out = {}
    for name, path in (("FETCH_SIZE", fetch_csv), ("WRITE_SIZE", write_csv)):
        v = per_kernel(path, name)
        cal = [x for k, xs in v.items() if "fedavg_kernel" in k for x in xs if x > 0]
        # the last three fedavg launches are the calibration copies (the per-step FedAvg is tiny)
        cal = sorted(cal)[-3:]
        gemm = [x for k, xs in v.items() if "gemm_kernel" in k for x in xs]
        factor = CAL_BYTES / (sum(cal) / len(cal))
        out[name] = dict(cal=sum(cal) / len(cal), factor=factor, n=len(gemm), raw=sum(gemm) / len(gemm),
                         bytes=sum(gemm) / len(gemm) * factor)
    here = os.path.dirname(os.path.abspath(__file__))
    h = hashlib.sha256()
    for name in ("gemm.hip", "gemm_epilogue.h"):          # the GEMM kernel's source (bench.py checks the same digest)
        h.update(open(os.path.join(here, "csrc", name), "rb").read())
    sha = h.hexdigest()
    total = out["FETCH_SIZE"]["bytes"] + out["WRITE_SIZE"]["bytes"]
    print("# HBM traffic of the bf16 GEMM kernel, workload 3 (rocprofv3 counters)\n")
    print("Commands (from /tmp with TMPDIR=/tmp, one counter per run):\n")
    for counter, path in (("FETCH_SIZE", fetch_csv), ("WRITE_SIZE", write_csv)):
        outdir = os.path.dirname(path) or "."
        prefix = os.path.basename(path).replace("_counter_collection.csv", "")
        print("    rocprofv3 --pmc %s --kernel-trace --output-format csv -d %s -o %s -- "
              "python3 bench.py --steps 2 --warmup 1 --no-cpu-baseline --no-legs --copy-calibration"
              % (counter, outdir, prefix))
    print("    python -m paper_2407_00952_amd.pmc_summary <f_counter_collection.csv> <w_counter_collection.csv>\n")
    print("| counter | copy kernel reads (256 MiB moved) | bytes per count | GEMM launches | GEMM average count | GEMM bytes per launch |")
    print("|---|---|---|---|---|---|")
    for name in ("FETCH_SIZE", "WRITE_SIZE"):
        o = out[name]
        print("| %s | %.1f | %.1f | %d | %.1f | %.4e |" % (name, o["cal"], o["factor"], o["n"], o["raw"], o["bytes"]))
    print("\ntraffic_bytes_per_launch: %.6e" % total)
    print("gemm_source_sha256: %s" % sha)


if __name__ == "__main__":
    main(sys.argv[1], sys.argv[2])
