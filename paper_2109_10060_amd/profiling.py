"""Turns rocprofv3 CSV output into the short text / JSON summaries kept under profiles/.

  python -m paper_2109_10060_amd.profiling stats  <kernel_stats.csv> <out.txt> "<title>" "<command>"
  python -m paper_2109_10060_amd.profiling traffic <fetch.csv> <write.csv> <copy_fetch.csv> <copy_write.csv> \
         <copy_bytes> <out.json> "<commands>"
  python -m paper_2109_10060_amd.profiling layers <kernel_trace.csv> <layers.json> <out.txt> "<title>" "<command>"

  python -m paper_2109_10060_amd.profiling counters <counter_collection.csv> [more.csv ...] <out.txt> "<title>" "<command>"

`counters` averages the hardware counters of one or more rocprofv3 --pmc runs per kernel (over that kernel's dispatches)
and derives, where the raw counters are present: the share of time the matrix pipes were busy (SQ_VALU_MFMA_BUSY_CYCLES
over GRBM_GUI_ACTIVE x 1024 SIMDs), the LDS busy and bank-conflict shares, the L2 hit rate and the bytes the L2 served.

`layers` joins a rocprofv3 kernel trace of the benchmark with the per-launch work list the benchmark writes
(`bench.py --layers-json`): one row per kernel launch of a forward pass with its algorithmic flops and bytes, its
duration averaged over the traced passes, the rates these give, the roof its arithmetic intensity selects
(bf16 matrix peak above the ridge of 2500 TFLOP/s / 8 TB/s = 312 flop per byte, HBM below) and the fraction reached.

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


# kernel-name fragments -> class of the per-launch work list (cost.py)
CLASS_OF = (("attention_kernel", "attention"), ("layernorm", "layernorm"), ("dwconv", "dwconv"), ("dwpw_kernel", "dwconv"),
            ("stem_", "stem"), ("maxpool_kernel", "maxpool"))
PEAK_TFLOPS, PEAK_GBS = 2500.0, 8000.0


def layers(trace_csv, layers_json, out_path, title, command):
    work = json.load(open(layers_json))
    rows = sorted(csv.DictReader(open(trace_csv)), key=lambda r: int(r["Start_Timestamp"]))   # launch order
    per_class = {}
    for r in rows:
        name = r["Kernel_Name"]
        cls = None
        if any(k in name for k in GEMM_KERNELS):
            cls = "gemm*"
        else:
            for frag, c in CLASS_OF:
                if frag in name:
                    cls = c
                    break
        if cls is None:
            continue
        per_class.setdefault(cls, []).append((_short(name), (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) * 1e-3))
    want = {}
    for i, w in enumerate(work):
        cls = "gemm*" if w["kind"] in ("gemm", "gemm_taps") else w["kind"]
        want.setdefault(cls, []).append(i)
    lines = [f"# {title}", f"# command: {command}",
             "# us = mean duration of that launch over the traced passes; roof = the one the launch's flop per byte selects",
             "layer | kernel | shape | GFLOP | MB | flop/B | us | TFLOP/s | GB/s | roof | fraction"]
    out_rows = {}
    for cls, idx in want.items():
        got = per_class.get(cls, [])
        n = len(idx)
        if not got or len(got) < n or cls in ("gate", "head", "index"):
            continue
        passes = min(len(got) // n, 8)           # the last passes of the run: warm, and aligned to the end of the trace
        tail = got[len(got) - passes * n:]
        for k, i in enumerate(idx):
            durs = [tail[p * n + k][1] for p in range(passes)]
            out_rows[i] = (tail[(passes - 1) * n + k][0], sum(durs) / len(durs), passes)
    tot = {"mfma": [0.0, 0.0], "hbm": [0.0, 0.0]}
    for i, w in enumerate(work):
        if i not in out_rows:
            continue
        kern, us, _ = out_rows[i]
        ai = w["flops"] / max(w["bytes"], 1.0)
        tf, gbs = w["flops"] / (us * 1e-6) / 1e12, w["bytes"] / (us * 1e-6) / 1e9
        roof = "mfma" if ai >= PEAK_TFLOPS * 1e12 / (PEAK_GBS * 1e9) else "hbm"
        frac = tf / PEAK_TFLOPS if roof == "mfma" else gbs / PEAK_GBS
        tot[roof][0] += us
        tot[roof][1] += frac * us
        lines.append(f"{w['name']} | {kern} | {w['shape']} | {w['flops'] / 1e9:.2f} | {w['bytes'] / 1e6:.1f} | {ai:.0f} | "
                     f"{us:.1f} | {tf:.0f} | {gbs:.0f} | {roof} | {frac:.3f}")
    for roof, (us, acc) in tot.items():
        if us:
            lines.append(f"# launches under the {roof} roof: {us:.0f} us per pass, time-weighted fraction {acc / us:.3f}")
    open(out_path, "w").write("\n".join(lines) + "\n")


def counters(csv_paths, out_path, title, command, top=12):
    agg = {}     # kernel -> counter -> [sum, dispatches]
    for path in csv_paths:
        per_dispatch = {}
        for r in csv.DictReader(open(path)):
            key = (r["Dispatch_Id"], _short(r["Kernel_Name"]))
            c, v = r["Counter_Name"], float(r["Counter_Value"])
            d = per_dispatch.setdefault(key, {})
            d[c] = d.get(c, 0.0) + v
        for (_, k), vals in per_dispatch.items():
            for c, v in vals.items():
                e = agg.setdefault(k, {}).setdefault(c, [0.0, 0])
                e[0] += v
                e[1] += 1
    mean = {k: {c: v[0] / v[1] for c, v in cs.items()} for k, cs in agg.items()}
    order = sorted(mean, key=lambda k: -mean[k].get("GRBM_GUI_ACTIVE", 0.0) * max(v[1] for v in agg[k].values()))[:top]
    names = sorted({c for k in order for c in mean[k]})
    lines = [f"# {title}", f"# command: {command}",
             "# per kernel: mean over its dispatches; derived figures first (clocks = GRBM_GUI_ACTIVE / 8 XCDs; mfma_busy: SQ_VALU_MFMA_BUSY_CYCLES / (clocks x 1024 SIMDs);",
             "# lds_busy: SQ_LDS_IDX_ACTIVE / (clocks x 256 compute units); wave_wait: SQ_WAIT_ANY / SQ_WAVE_CYCLES, the share of resident wave cycles spent waiting)",
             "kernel | dispatches | " + " | ".join(["mfma_busy_pct", "lds_busy_pct", "lds_conflict_pct_of_lds", "wave_wait_pct", "l2_hit_pct"] + names)]
    for k in order:
        m = mean[k]
        # the tool reports every counter summed over its hardware instances: GRBM_GUI_ACTIVE is the busy clock of
        # each of the 8 XCDs added up, so one eighth of it is the kernel's duration in clocks
        act = m.get("GRBM_GUI_ACTIVE", 0.0) / 8.0
        d = []
        d.append(f"{100 * m['SQ_VALU_MFMA_BUSY_CYCLES'] / (act * 1024):.1f}" if act and "SQ_VALU_MFMA_BUSY_CYCLES" in m else "-")
        d.append(f"{100 * m['SQ_LDS_IDX_ACTIVE'] / (act * 256):.1f}" if act and "SQ_LDS_IDX_ACTIVE" in m else "-")
        d.append(f"{100 * m['SQ_LDS_BANK_CONFLICT'] / m['SQ_LDS_IDX_ACTIVE']:.1f}" if m.get("SQ_LDS_IDX_ACTIVE") and "SQ_LDS_BANK_CONFLICT" in m else "-")
        d.append(f"{100 * m['TCC_HIT_sum'] / (m['TCC_HIT_sum'] + m['TCC_MISS_sum']):.1f}" if m.get("TCC_HIT_sum") is not None and (m.get("TCC_HIT_sum", 0) + m.get("TCC_MISS_sum", 0)) > 0 else "-")
        d.insert(3, f"{100 * m['SQ_WAIT_ANY'] / m['SQ_WAVE_CYCLES']:.1f}" if m.get("SQ_WAVE_CYCLES") and "SQ_WAIT_ANY" in m else "-")
        n = max(v[1] for v in agg[k].values())
        lines.append(f"{k} | {n} | " + " | ".join(d + [f"{m[c]:.0f}" if c in m else "-" for c in names]))
    open(out_path, "w").write("\n".join(lines) + "\n")


if __name__ == "__main__":
    if sys.argv[1] == "counters":
        counters(sys.argv[2:-3], *sys.argv[-3:])
    elif sys.argv[1] == "layers":
        layers(*sys.argv[2:7])
    elif sys.argv[1] == "stats":
        stats(*sys.argv[2:6])
    elif sys.argv[1] == "traffic":
        traffic(*sys.argv[2:9])
    else:
        raise SystemExit(__doc__)
