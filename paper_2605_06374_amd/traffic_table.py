"""Turns two rocprofv3 counter runs of bench.py (FETCH_SIZE, WRITE_SIZE) into the table of
measured HBM bytes per launch that bench.py reports under roofline.traffic.

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d prof/pmc_fetch -o pmc -- \\
        python3 bench.py --steps 8 --warmup 2 --no-cpu-baseline --no-kernel-timing --calibrate-copy
    (the same with WRITE_SIZE into prof/pmc_write)
    python -m paper_2605_06374_amd.traffic_table <workload> prof/pmc_fetch prof/pmc_write

Every counter is scaled by what it reads for bench_copy_kernel, a plain copy of known size run
by --calibrate-copy under the same command.  The table is keyed by a digest of the kernel
sources, so that bench.py reports null once the kernels have changed.  File handling only."""
from __future__ import annotations

import collections
import csv
import glob
import json
import os
import re
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
KERNELS = ("plan_kernel", "fwd_combine_kernel", "fwd_kernel", "bwd_dkv_kernel", "bwd_dq_kernel",
           "bwd_combine_kernel", "bench_copy_kernel")


def counter_means(directory: str, counter: str) -> dict:
    files = glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise SystemExit(f"no *counter_collection.csv under {directory}")
    acc = collections.defaultdict(list)
    for f in files:
        for r in csv.DictReader(open(f)):
            if r["Counter_Name"] != counter:
                continue
            m = re.search("|".join(KERNELS), r["Kernel_Name"])
            if m:
                acc[m.group(0)].append(float(r["Counter_Value"]))
    return {k: sum(v) / len(v) for k, v in acc.items()}


def main(argv) -> int:
    if len(argv) != 4:
        print(__doc__)
        return 2
    workload, fetch_dir, write_dir = argv[1:]
    sys.path.insert(0, ROOT)
    import bench
    fetch, write = counter_means(fetch_dir, "FETCH_SIZE"), counter_means(write_dir, "WRITE_SIZE")
    if "bench_copy_kernel" not in fetch or "bench_copy_kernel" not in write:
        raise SystemExit("the runs hold no bench_copy_kernel: pass --calibrate-copy to bench.py")
    f_scale = bench.CALIBRATION_COPY_BYTES / fetch["bench_copy_kernel"]
    w_scale = bench.CALIBRATION_COPY_BYTES / write["bench_copy_kernel"]
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    digest = bench.csrc_digest()
    try:
        table = json.load(open(path))
    except (OSError, ValueError):
        table = {}
    if table.get("csrc_sha256") != digest:
        table = {"csrc_sha256": digest, "entries": {}}
    table["bytes_per_count"] = {"FETCH_SIZE": round(f_scale, 2), "WRITE_SIZE": round(w_scale, 2)}
    table["entries"][workload] = {
        k: {"fetch_bytes": round(fetch[k] * f_scale), "write_bytes": round(write.get(k, 0.0) * w_scale)}
        for k in sorted(fetch) if k != "bench_copy_kernel"}
    json.dump(table, open(path, "w"), indent=1, sort_keys=True)
    print(json.dumps(table["entries"][workload], indent=1))
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
