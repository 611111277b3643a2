"""Turns two rocprofv3 counter runs of bench.py (FETCH_SIZE, then WRITE_SIZE) into the HBM-traffic
summary that bench.py reports as roofline.traffic.

    python -m paper_1909_09577_amd.traffic_summary FETCH.csv WRITE.csv OUT.md "<command line of the runs>"

FETCH.csv / WRITE.csv are the `*_counter_collection.csv` files of

    rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d DIR -o NAME -- \\
        python3 bench.py --steps 10 --warmup 2 --no-cpu-baseline --calibration-copies 5

(and the same with WRITE_SIZE).  Both counters are in KiB per dispatch; they are scaled by what the
same counter reads for the plain 256 MiB copy kernels (dst = src + 1 on int32) that `--calibration-copies` runs first
(256 MiB fetched and 256 MiB written per copy).  The summary records a hash of the kernel sources:
bench.py reports the traffic only while the sources still match.
"""
from __future__ import annotations

import csv
import hashlib
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COPY_BYTES = 256 << 20


def sources_sha256() -> str:
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_1909_09577_amd", "csrc")
    for f in sorted(os.listdir(csrc)):
        if f.endswith((".hip", ".h")):
            h.update(open(os.path.join(csrc, f), "rb").read())
    return h.hexdigest()


def per_kernel(path: str, counter: str):
    """{key: [KiB per dispatch]} with the two conv launches told apart by the kernel before them."""
    rows = [r for r in csv.DictReader(open(path)) if r["Counter_Name"] == counter]
    rows.sort(key=lambda r: int(r["Dispatch_Id"]))
    out, prev = {}, ""
    for r in rows:
        name = r["Kernel_Name"]
        key = None
        if "conv_gemm_kernel" in name:
            key = "dgrad" if "_prepare_kernel" in prev else "fwd"  # the input gradient follows a preparation kernel
        elif "wgrad_shared_kernel" in name or "wgrad_fast_kernel" in name or "wgrad_kernel" in name:
            key = "wgrad"
        elif "prepack_kernel" in name:
            key = "weight packing (fwd)"
        elif "dgrad_prepare" in name:
            key = "weight packing + dz/dres pass (dgrad)"
        elif "bwd_prepare" in name:
            key = "weight packing + dz pass for both gradients (nm_conv1d_bwd)"
        elif "dz_pack" in name:
            key = "dz pass (wgrad)"
        elif "wgrad_reduce" in name:
            key = "dw reduction"
        elif "vectorized_elementwise_kernel" in name and "_add<" in name and int(r["Grid_Size"]) >= (1 << 20):
            key = "calibration copy"  # the 64 Mi-element dst = src + 1 kernels of --calibration-copies
        if key:
            out.setdefault(key, []).append(float(r["Counter_Value"]))
        prev = name
    return out


def main():
    fetch_csv, write_csv, out_md, command = sys.argv[1:5]
    fetch, write = per_kernel(fetch_csv, "FETCH_SIZE"), per_kernel(write_csv, "WRITE_SIZE")
    avg = lambda v: sum(v) / len(v)
    f_scale = COPY_BYTES / (avg(fetch["calibration copy"]) * 1024.0)  # true bytes per counted byte
    w_scale = COPY_BYTES / (avg(write["calibration copy"]) * 1024.0)
    lines = [
        "# HBM traffic per launch, headline workload (B=32, C=512, K=17, T=800)", "",
        "Commands (MI355X, one GPU; one counter per run):", "",
        "    " + command.replace("COUNTER", "FETCH_SIZE"),
        "    " + command.replace("COUNTER", "WRITE_SIZE"),
        "    python -m paper_1909_09577_amd.traffic_summary <FETCH csv> <WRITE csv> <this file> '<command>'", "",
        "FETCH_SIZE / WRITE_SIZE are KiB per dispatch.  Scale factors from the plain 256 MiB device copies run",
        f"first in the same process: fetch x{f_scale:.4f}, write x{w_scale:.4f} (true bytes per counted byte).", "",
        f"sources_sha256: {sources_sha256()}", "",
        "| kernel | launches | fetched MB | written MB | total MB |", "|---|---|---|---|---|",
    ]
    for key in ("fwd", "dgrad", "wgrad", "weight packing (fwd)", "weight packing + dz/dres pass (dgrad)",
                "weight packing + dz pass for both gradients (nm_conv1d_bwd)", "dz pass (wgrad)", "dw reduction",
                "calibration copy"):
        if key in fetch and key in write:
            fb = avg(fetch[key]) * 1024.0 * f_scale / 1e6
            wb = avg(write[key]) * 1024.0 * w_scale / 1e6
            lines.append(f"| {key} | {len(fetch[key])} | {fb:.1f} | {wb:.1f} | {fb + wb:.1f} MB |")
    lines += ["", "Algorithmic bytes per launch for comparison: fwd 87.6 MB, dgrad 87.6 MB (+26.2 MB dres), wgrad 70.2 MB",
              "(x + dz + dw; the dz pass and the reduction have their own rows).", ""]
    open(out_md, "w").write("\n".join(lines))
    print("\n".join(lines))


if __name__ == "__main__":
    main()
