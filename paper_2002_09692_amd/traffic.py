"""Turns two rocprofv3 counter runs of bench.py into the measured HBM traffic per launch of a kernel.

  cd /tmp && export TMPDIR=/tmp
  rocprofv3 --pmc FETCH_SIZE --output-format csv -d <dirF> -o pmc -- python3 bench.py --no-cpu --no-others --workload cfg3 --steps 5 --warmup 1
  rocprofv3 --pmc WRITE_SIZE --output-format csv -d <dirW> -o pmc -- python3 bench.py --no-cpu --no-others --workload cfg3 --steps 5 --warmup 1
  python3 -m paper_2002_09692_amd.traffic --workload cfg3 --kernel fused_pair_kernel \
          --fetch <dirF>/.../pmc_counter_collection.csv --write <dirW>/.../pmc_counter_collection.csv

Both counters are KiB per dispatch in the unit of the TCC request size; the scale to bytes is taken from the
copy yardstick of the same run (stream_copy_kernel reads and writes 4 * n * ld bytes, known exactly).  The
result goes into profiles/hbm_traffic.json under the workload's name, stamped with a hash of the kernel sources
so that bench.py can tell when the stored figure no longer belongs to the kernels in the tree.  Reads files only.
"""
from __future__ import annotations

import argparse
import csv
import hashlib
import json
import os
import sys
from collections import defaultdict

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
KERNEL_SOURCES = ("paper_2002_09692_amd/csrc/saps_device.hpp", "paper_2002_09692_amd/csrc/saps_api.hip")


def kernel_source_sha16() -> str:
    """Hash of the kernel sources without comments and white space (a reworded comment changes no kernel)."""
    import re
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "r") as f:
            text = f.read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        text = re.sub(r"//[^\n]*", "", text)
        h.update("".join(text.split()).encode())
    return h.hexdigest()[:16]


def per_kernel_mean(path: str, counter: str) -> dict:
    """Mean counter value per dispatch, by kernel name (template arguments kept, parameter list cut)."""
    acc = defaultdict(list)
    with open(path, newline="") as f:
        for row in csv.DictReader(f):
            if row["Counter_Name"] != counter:
                continue
            name = row["Kernel_Name"].split("(")[0].replace("void ", "").replace("saps::", "").strip()
            acc[name].append(float(row["Counter_Value"]))
    return {k: (sum(v) / len(v), len(v)) for k, v in acc.items()}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True)
    ap.add_argument("--kernel", required=True, help="prefix of the kernel's name, e.g. fused_round_kernel")
    ap.add_argument("--fetch", required=True)
    ap.add_argument("--write", required=True)
    ap.add_argument("--out", default=os.path.join(ROOT, "profiles", "hbm_traffic.json"))
    args = ap.parse_args()

    sys.path.insert(0, ROOT)
    from paper_2002_09692_amd import synth
    wl = synth.workload(args.workload)
    copy_bytes = 4.0 * wl.n * wl.ld()

    F = per_kernel_mean(args.fetch, "FETCH_SIZE")
    W = per_kernel_mean(args.write, "WRITE_SIZE")
    copy_f = next(v for k, v in F.items() if k.startswith("stream_copy_kernel"))[0]
    copy_w = next(v for k, v in W.items() if k.startswith("stream_copy_kernel"))[0]
    fetch_scale = copy_bytes / (copy_f * 1024.0)
    write_scale = copy_bytes / (copy_w * 1024.0)
    kf = max(((k, v) for k, v in F.items() if k.startswith(args.kernel)), key=lambda kv: kv[1][0])
    kw = max(((k, v) for k, v in W.items() if k.startswith(args.kernel)), key=lambda kv: kv[1][0])
    fetch_bytes = kf[1][0] * 1024.0 * fetch_scale
    write_bytes = kw[1][0] * 1024.0 * write_scale

    stored = {}
    if os.path.exists(args.out):
        with open(args.out) as f:
            stored = json.load(f)
    stored[args.workload] = {
        "kernel": kf[0], "fetch_bytes": fetch_bytes, "write_bytes": write_bytes, "total_bytes": fetch_bytes + write_bytes,
        "fetch_scale": fetch_scale, "write_scale": write_scale, "dispatches": [kf[1][1], kw[1][1]],
        "kernel_source_sha16": kernel_source_sha16(),
    }
    with open(args.out, "w") as f:
        json.dump(stored, f, indent=1)
    print(f"{args.workload}: {kf[0]}: read {fetch_bytes / 1e9:.4f} GB + written {write_bytes / 1e9:.4f} GB per launch "
          f"(scales x{fetch_scale:.4f}, x{write_scale:.4f}); all kernels:")
    for k in sorted(set(F) | set(W)):
        print(f"  {k:60s} FETCH_SIZE {F.get(k, (0, 0))[0]:14.1f}  WRITE_SIZE {W.get(k, (0, 0))[0]:14.1f}  KiB/dispatch")
    return 0


if __name__ == "__main__":
    sys.exit(main())
