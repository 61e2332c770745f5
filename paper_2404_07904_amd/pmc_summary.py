"""Turn two `rocprofv3 --pmc` runs of bench.py (FETCH_SIZE in one, WRITE_SIZE in the other, both
with --calibrate-copy) into the HBM bytes every kernel moves per launch.

Each counter is scaled by what it reads for the library's own copy probe of known size (bench.py
--calibrate-copy copies 1 GiB with hgrn2_probe_copy), so that a counter which sees only part of the
traffic on this machine is corrected by the same factor for every kernel.  The result is written as
JSON (default: profiles/measured_traffic.json); bench.py reports these figures as `roofline.traffic`.

    python -m paper_2404_07904_amd.pmc_summary <dir of the FETCH_SIZE run> <dir of the WRITE_SIZE run> [out.json]
"""
from __future__ import annotations

import csv
import glob
import json
import os
import subprocess
import sys

COPY_KERNEL = "probe_copy_kernel"
COPY_BYTES = 1 << 30          # what bench.py --calibrate-copy copies per launch
KIB = 1024.0

# kernels of interest: short name -> substring of the profiler's kernel name
KERNELS = {
    "bwd_fused_kernel": "bwd_fused_kernel",
    "fwd_fused_kernel": "fwd_fused_kernel",
    "bwd_grad_kernel": "bwd_grad_kernel",
    "sweep_kernel_mode1": "sweep_kernelIDF16bLi128ELi128ELi64ELi1E",
    "step_kernel": "step_kernel",
    "hgrn1_fwd_kernel": "hgrn1_fwd_kernel",
    "hgrn1_bwd_kernel": "hgrn1_bwd_kernel<true, false, false>",
    "hgrn1_bwd_saved_kernel": "hgrn1_bwd_kernel<true, false, true>",
    "proj_fwd_gemm": "gemm_dl_kernel<0,",
    "proj_dx_gemm": "gemm_dl_kernel<1,",
    "proj_dw_gemm": "gemm_kernel<true, true, 2",
    "proj_dact_kernel": "proj_dact_kernel",
}


def per_kernel(directory: str, counter: str):
    files = glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise SystemExit("no *counter_collection.csv under %s" % directory)
    sums, counts = {}, {}
    for path in files:
        with open(path, newline="") as fh:
            for row in csv.DictReader(fh):
                if row["Counter_Name"] != counter:
                    continue
                name = row["Kernel_Name"]
                sums[name] = sums.get(name, 0.0) + float(row["Counter_Value"])
                counts[name] = counts.get(name, 0) + 1
    return {k: (sums[k] / counts[k], counts[k]) for k in sums}


def pick(table, needle):
    hits = [(v, k) for k, v in table.items() if needle in k]
    if not hits:
        return None
    # several template instances may match: take the one launched most often
    return max(hits, key=lambda h: h[0][1])[0]


def main(argv):
    if len(argv) < 3:
        raise SystemExit(__doc__)
    fetch_dir, write_dir = argv[1], argv[2]
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = argv[3] if len(argv) > 3 else os.path.join(root, "profiles", "measured_traffic.json")
    fetch, write = per_kernel(fetch_dir, "FETCH_SIZE"), per_kernel(write_dir, "WRITE_SIZE")
    cf, cw = pick(fetch, COPY_KERNEL), pick(write, COPY_KERNEL)
    if cf is None or cw is None:
        raise SystemExit("the copy probe is missing from the runs: pass --calibrate-copy to bench.py")
    scale_r = COPY_BYTES / (cf[0] * KIB)
    scale_w = COPY_BYTES / (cw[0] * KIB)
    try:
        commit = subprocess.run(["git", "-C", root, "rev-parse", "--short", "HEAD"], capture_output=True, text=True).stdout.strip()
    except OSError:
        commit = ""
    result = {"unit": "bytes per launch", "source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch), each scaled by "
              "the factor that makes the 1 GiB copy probe read 1 GiB", "commit": commit,
              "calibration": {"copy_bytes": COPY_BYTES, "FETCH_SIZE_KiB": round(cf[0], 1), "WRITE_SIZE_KiB": round(cw[0], 1),
                              "fetch_scale": round(scale_r, 4), "write_scale": round(scale_w, 4)},
              "kernels": {}}
    for short, needle in KERNELS.items():
        r, w = pick(fetch, needle), pick(write, needle)
        if r is None or w is None:
            continue
        rb, wb = r[0] * KIB * scale_r, w[0] * KIB * scale_w
        result["kernels"][short] = {"read_bytes": round(rb), "write_bytes": round(wb), "bytes": round(rb + wb),
                                    "launches_seen": [r[1], w[1]]}
    with open(out, "w") as fh:
        json.dump(result, fh, indent=1, sort_keys=True)
        fh.write("\n")
    print(json.dumps(result, indent=1, sort_keys=True))


if __name__ == "__main__":
    main(sys.argv)
