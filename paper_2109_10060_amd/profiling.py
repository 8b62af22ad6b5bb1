"""Turns rocprofv3 CSV output into the short text / JSON summaries kept under profiles/.

  python -m paper_2109_10060_amd.profiling stats  <kernel_stats.csv> <out.txt> "<title>" "<command>"
  python -m paper_2109_10060_amd.profiling traffic <fetch.csv> <write.csv> <copy_fetch.csv> <copy_write.csv> \
         <copy_bytes> <out.json> "<commands>"

`traffic` reads two counter-collection runs of the benchmark (FETCH_SIZE, then WRITE_SIZE, KiB per
dispatch), scales each by what the same counter reads for a plain device copy of known size, and
stores the HBM bytes per launch of the grouped GEMM kernel together with a hash of the kernel
source, so that bench.py reports the figure only while the kernel is unchanged.
"""
from __future__ import annotations

import csv
import hashlib
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
KERNEL_SOURCES = ["csrc/gemm.hip", "csrc/conv3.hip", "csrc/thin.hip", "csrc/common.h"]
# the grouped GEMM is three kernels: gemm_kernel (linear, 1x1, strided and KxK layers), conv3_kernel (3x3 stride-1
# layers) and thin_kernel (1x1 layers with at most 64 / 128 input channels); the summaries treat them as one kernel
# class, as bench.py does
GEMM_KERNELS = ("gemm_kernel", "conv3_kernel", "thin_kernel")


def kernel_source_hash() -> str:
    h = hashlib.sha256()
    for f in KERNEL_SOURCES:
        h.update(open(os.path.join(HERE, f), "rb").read())
    return h.hexdigest()[:16]


def _short(name: str) -> str:
    name = name.replace("(anonymous namespace)::", "")
    for k in GEMM_KERNELS:
        if k in name:
            return k
    name = name.split("(")[0]
    return name[-60:]


def stats(csv_path, out_path, title, command, top=14):
    agg = {}
    for r in csv.DictReader(open(csv_path)):
        k = _short(r["Name"])
        e = agg.setdefault(k, [0, 0.0])
        e[0] += int(r["Calls"])
        e[1] += float(r["TotalDurationNs"])
    total = sum(v[1] for v in agg.values())
    lines = [f"# {title}", f"# command: {command}", "kernel | calls | total_ns | avg_ns | percent"]
    for k, (n, t) in sorted(agg.items(), key=lambda kv: -kv[1][1])[:top]:
        lines.append(f"{k} | {n} | {t:.0f} | {t / n:.0f} | {100 * t / total:.2f}")
    open(out_path, "w").write("\n".join(lines) + "\n")


def _per_launch(csv_path, counter, match):
    match = (match,) if isinstance(match, str) else match
    vals = [float(r["Counter_Value"]) for r in csv.DictReader(open(csv_path))
            if r["Counter_Name"] == counter and any(m in r["Kernel_Name"] for m in match)]
    return sum(vals) / len(vals), len(vals)


def traffic(fetch_csv, write_csv, copy_fetch_csv, copy_write_csv, copy_bytes, out_json, commands):
    copy_kib = int(copy_bytes) / 1024.0
    cf, _ = _per_launch(copy_fetch_csv, "FETCH_SIZE", "copyBuffer")
    cw, _ = _per_launch(copy_write_csv, "WRITE_SIZE", "copyBuffer")
    ff, fw = copy_kib / cf, copy_kib / cw
    gf, n = _per_launch(fetch_csv, "FETCH_SIZE", GEMM_KERNELS)
    gw, _ = _per_launch(write_csv, "WRITE_SIZE", GEMM_KERNELS)
    out = {"kernel": "gemm_kernel+conv3_kernel+thin_kernel", "source_hash": kernel_source_hash(), "launches_sampled": n,
           "fetch_kib_per_launch": gf, "write_kib_per_launch": gw, "fetch_factor": ff, "write_factor": fw,
           "hbm_bytes_per_launch": (gf * ff + gw * fw) * 1024.0, "commands": commands}
    json.dump(out, open(out_json, "w"), indent=1)
    print(json.dumps(out))


if __name__ == "__main__":
    if sys.argv[1] == "stats":
        stats(*sys.argv[2:6])
    elif sys.argv[1] == "traffic":
        traffic(*sys.argv[2:9])
    else:
        raise SystemExit(__doc__)
