#!/usr/bin/env python3
"""Throughput of the gate-routed, weight-sliced forward pass on one MI355X.

One step = one ds_forward pass (gate, bucketing, every sliced layer, classifier,
un-permute) over a batch of 256 synthetic ImageNet-shaped images with mixed routes,
inputs and weights resident in HBM.  Prints one JSON line:
images/s (mean over the timed steps, with the median and the 10th / 90th percentile
of the single steps beside it), the roofline fraction of the dominant kernel class
(measured with HIP events around every launch of it inside the timed region) and of
each of its kernels against the roof its launches select, and the CPU oracle timed
on a bounded sample of the same workload.  Without --workload the headline is
config 4 (DS-ResNet) and configs 3 and 5 are measured after it (other_workloads).
Defaults: 20 warm-up and 100 timed steps.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_BF16_TFLOPS = 2500.0   # dense bf16 matrix-core peak of MI355X
PEAK_HBM_GBS = 8000.0


def build_workload(name: str, B: int, mix: str = "uniform"):
    import numpy as np
    import workloads as WL
    S = WL.BASE_SEED

    def bias(seed, T, amp=4.0, late=False):
        # "skewed": half of the batch takes the smallest route at an early (or only) gate and the
        # largest route at a late gate; the other half stays spread over all routes
        favour = -1 if mix == "uniform" else (T - 1 if late else 0)
        return WL.seeded_logit_bias(seed, B, T, amp=amp, favour=favour)

    if name == "mbnet":
        arch = WL.mbnet_arch()
        params = WL.mbnet_params(arch, S + 3)
        lb = bias(S + 203, arch["T"])[None]
        label = "config3: DS-MBNet (MobileNetV1-shaped, 14 width routes), bf16"
    elif name == "mbnet_pp":
        arch = WL.mbnet_pp_arch()
        params = WL.mbnet_params(arch, S + 8)
        lb = bias(S + 208, arch["T"])[None]
        label = "DS-MBNet++ (12 routes over channels [288:640:32] / [800:1152:32] and depthwise kernel size 3/5/7), bf16"
    elif name == "resnet":
        arch = WL.resnet_arch()
        params = WL.resnet_params(arch, S + 4)
        lb = np.stack([bias(S + 204 + s, 4, amp=16.0, late=s >= 2) for s in range(4)])
        label = "config4: DS-ResNet (ResNet-50-shaped, 4 gates x 4 width ratios), bf16"
    elif name == "resnet_pp":
        arch = WL.resnet_arch(blocks=(3, 4, 8, 3), routes="pp")
        params = WL.resnet_params(arch, S + 9)
        lb = np.stack([bias(S + 209 + s, 9, amp=16.0) for s in range(4)])
        label = "DS-ResNet++ (one gate, 9 paths over stage widths [128:256:32] .. [1024:2048:128] and block counts), bf16"
    elif name == "vit":
        arch = WL.vit_arch()
        params = WL.vit_params(arch, S + 5)
        lb = bias(S + 205, arch["T"])[None]
        label = "config5: DS-ViT (DeiT-S-shaped, 48 routes over embed/heads/MLP), bf16"
    elif name == "vit_stem":
        arch = WL.vit_arch(stem_dim=24, patch=8)
        params = WL.vit_params(arch, S + 6)
        lb = bias(S + 206, arch["T"], amp=16.0)[None]
        label = "DS-ViT++ stem (conv + 2 depthwise-separable blocks at 24 channels, gate on its map) + config5's network, bf16"
    elif name == "vit_pp":
        arch = WL.vit_arch(embed=416, heads=8, head_dim=48, mlp=1664, depth=14, routes="pp", stem_dim=24, patch=8)
        params = WL.vit_params(arch, S + 7)
        lb = bias(S + 207, arch["T"], amp=16.0)[None]
        label = ("DS-ViT++ supernet (stem, embed 192..416, 4..8 heads of 48, MLP ratio 3..4, depth 12..14; "
                 "8 nested routes), bf16")
    else:
        raise SystemExit(f"unknown workload {name}")
    imgs = WL.images(S + 100 + {"mbnet": 3, "resnet": 4, "vit": 5, "vit_stem": 6, "vit_pp": 7, "mbnet_pp": 8, "resnet_pp": 9}[name], B)
    return arch, params, imgs, lb.astype("float32"), label


def cpu_baseline(name, arch, params, imgs, lb, budget_s=15.0):
    """Times the oracle as it stands on a bounded sample of the same batch."""
    from oracle import ds_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([d.get("num_threads", 1) for d in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    t0 = time.perf_counter()
    n = 0
    while n < imgs.shape[0] and (time.perf_counter() - t0 < budget_s or n < 2):
        if name in ("mbnet", "mbnet_pp"):
            O.forward_mbnet(arch, params, imgs[n], logit_bias=lb[0, n])
        elif name in ("resnet", "resnet_pp"):
            O.forward_resnet(arch, params, imgs[n], logit_bias=lb[:, n])
        elif name in ("vit_stem", "vit_pp"):
            O.forward_vit_stem(arch, params, imgs[n], logit_bias=lb[0, n])
        else:
            O.forward_vit(arch, params, imgs[n], O.gate_route(lb[0, n]))
        n += 1
    dt = time.perf_counter() - t0
    return {"value": n / dt, "unit": "images/s", "cores": int(threads), "kind": "oracle",
            "sample": f"first {n} images of the same batch, one image at a time, float64 numpy ({dt:.1f} s); cores = the "
                      f"threads of numpy's BLAS pool (its matmul calls are the only parallel part; no parallelism over samples)"}


def run_linear(args):
    """Config 2: the sliced linear sweep (64 images x 197 tokens, embedding slices 192..384, output slices 4x that).
    A step buckets the images by their slice and runs the one grouped GEMM over the four buckets."""
    import numpy as np
    import torch
    import workloads as WL
    import paper_2109_10060_amd as ds

    ds.load()
    dev = "cuda:0"
    B = 64 if args.batch == 256 else args.batch          # config 2 is defined at 64 images; --batch overrides
    c = WL.config2(B=B)
    x = torch.from_numpy(c["x"]).to(dev).to(torch.bfloat16).contiguous()
    w = torch.from_numpy(c["w"]).to(dev).to(torch.bfloat16).contiguous()
    bias = torch.from_numpy(c["bias"]).to(dev).contiguous()
    route = torch.from_numpy(c["route"]).to(dev).contiguous()
    y = torch.zeros((B, c["N"], 4 * c["K"]), dtype=torch.bfloat16, device=dev)

    def step():
        perm, _inv, off = ds.ds_route_bucket(route, c["T"])
        g = ds.make_groups(off, perm, c["k_in"].tolist(), c["k_out"].tolist())
        ds.ds_sliced_linear(x, w, bias, g, y=y)

    for _ in range(args.warmup):
        step()
    ds.ds_profile_reset()
    every = max(1, args.event_every)
    sampled = 0
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for i in range(args.steps):
        on = (not args.no_kernel_events) and i % every == min(every // 2, args.steps - 1)
        if on:
            ds.ds_profile_enable(True)
            sampled += 1
        step()
        if on:
            ds.ds_profile_enable(False)
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = max((time.perf_counter() - t0) * 1e3, e0.elapsed_time(e1)) / args.steps
    prof = ds.ds_profile_read() if sampled else {}
    # the same step with cold caches: a 1 GiB device fill between steps evicts L2 and the memory-side cache, so the
    # operands and the weight come from HBM; each step is timed on its own
    scratch = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    cold = []
    for i in range(min(20, args.steps)):
        scratch.fill_(i & 1)
        a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a0.record()
        step()
        a1.record()
        torch.cuda.synchronize()
        cold.append(a0.elapsed_time(a1))
    cold.sort()
    del scratch
    k_in = c["k_in"][c["route"]].astype(np.float64)
    k_out = c["k_out"][c["route"]].astype(np.float64)
    flops = 2.0 * c["N"] * float(np.sum(k_in * k_out))
    nbytes = 2.0 * c["N"] * float(np.sum(k_in) + np.sum(k_out)) + 2.0 * float(k_in.max() * k_out.max())
    roofline = None
    if prof and prof["gemm"][1]:
        ms, n = prof["gemm"]
        tf = flops * sampled / (ms * 1e-3) / 1e12
        gbs = nbytes * sampled / (ms * 1e-3) / 1e9
        # 240 FLOP per byte: below the ridge, so the bound that applies is HBM; both views are given
        roofline = {"kernel": "gemm_kernel", "bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": gbs / PEAK_HBM_GBS, "traffic": None, "algorithmic_bytes_per_launch": nbytes,
                    "launches_per_step": n / sampled, "avg_launch_us": ms * 1e3 / n, "steps_sampled": sampled,
                    "share_of_step": ms / (ms_per_step * sampled),
                    "mfma_view": {"achieved": tf, "peak": PEAK_MFMA_BF16_TFLOPS, "unit": "TFLOP/s",
                                  "frac": tf / PEAK_MFMA_BF16_TFLOPS}}
    out = {
        "metric": "images/sec at batch 256 (mixed gate widths)", "value": B / (ms_per_step * 1e-3), "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "config2: sliced linear sweep (197 tokens per image, slices 192/256/320/384 -> 4x), "
                               "bucket + one grouped GEMM, operands warm in the caches", "batch": B,
                   "route_histogram": [np.bincount(c["route"], minlength=4).tolist()]},
        "roofline": roofline,
        "cold_caches": {"ms_per_step_median": cold[len(cold) // 2], "ms_per_step_min": cold[0], "steps": len(cold),
                        "flush": "1 GiB device fill before every step"},
    }
    if not args.no_cpu_baseline:
        from oracle import ds_oracle as O
        t1 = time.perf_counter()
        n = 0
        while time.perf_counter() - t1 < 10.0:             # whole passes over the batch, about 10 s of CPU work
            for i in range(B):
                t = int(c["route"][i])
                O.sliced_linear(c["x"][i][:, :c["k_in"][t]], c["w"], c["bias"], int(c["k_out"][t]))
            n += B
        dt = time.perf_counter() - t1
        try:
            from threadpoolctl import threadpool_info
            threads = max([d.get("num_threads", 1) for d in threadpool_info()] or [1])
        except Exception:
            threads = os.cpu_count() or 1
        out["cpu_baseline"] = {"value": n / dt, "unit": "images/s", "cores": int(threads), "kind": "oracle",
                               "sample": f"{n // B} passes over the same {B} images, one by one, float64 numpy ({dt:.1f} s)"}
    print(json.dumps(out))


GEMM_CLASSES = ("gemm", "gemm_taps", "conv3", "thin")          # kernel classes whose launches are the cost model's gemm / gemm_taps records
KERNEL_OF = {"gemm": "gemm_kernel", "gemm_taps": "gemm_kernel", "conv3": "conv3_kernel", "thin": "thin_kernel"}
RIDGE = PEAK_MFMA_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)     # flop per byte above which the matrix peak is the roof


def rates(flops, nbytes, ms, contraction):
    """Algorithmic rates of `flops` / `nbytes` done in `ms`, and the fraction of the roof that applies: a contraction whose
    flop per byte lies above the ridge is held against the bf16 matrix peak, everything else against HBM bandwidth."""
    t = ms * 1e-3
    tf, gbs = flops / t / 1e12, nbytes / t / 1e9
    ai = flops / max(nbytes, 1.0)
    roof = "mfma" if contraction and ai >= RIDGE else "hbm"
    return {"tflops": tf, "algorithmic_gbs": gbs, "flop_per_byte": ai, "roof": roof,
            "frac": tf / PEAK_MFMA_BF16_TFLOPS if roof == "mfma" else gbs / PEAK_HBM_GBS,
            "frac_mfma": tf / PEAK_MFMA_BF16_TFLOPS, "frac_hbm": gbs / PEAK_HBM_GBS}


def match_launches(cost, launches, sampled):
    """Joins the recorded launches (class, ms) of `sampled` identical steps with the cost model's per-launch records, class
    by class in launch order.  Returns the cost records with 'kernel' and 'us' (mean over the sampled steps) filled in."""
    per_step = len(launches) // sampled
    rows = [dict(r) for r in cost.launches]
    want = {}
    for i, r in enumerate(rows):
        want.setdefault("gemm*" if r["kind"] in ("gemm", "gemm_taps") else r["kind"], []).append(i)
    for cls, idx in want.items():
        got = [[(k, ms) for k, ms in launches[s0 * per_step:(s0 + 1) * per_step]
                if (k in GEMM_CLASSES if cls == "gemm*" else k == cls)] for s0 in range(sampled)]
        if any(len(g) != len(idx) for g in got):
            continue                                   # this class is launched differently from the model (gate, head): totals only
        for k, i in enumerate(idx):
            rows[i]["kernel"] = KERNEL_OF.get(got[0][k][0], got[0][k][0])
            rows[i]["us"] = 1e3 * sum(g[k][1] for g in got) / sampled
    return rows


def run_net(workload, args, steps, warmup, with_cpu_baseline):
    import numpy as np
    import torch
    import paper_2109_10060_amd as ds
    from paper_2109_10060_amd import cost as C

    dev = "cuda:0"
    B = args.batch
    arch, params, imgs, lb, label = build_workload(workload, B, args.mix)
    net = {"mbnet": ds.build_mbnet, "mbnet_pp": ds.build_mbnet, "resnet": ds.build_resnet, "resnet_pp": ds.build_resnet, "vit": ds.build_vit,
           "vit_stem": ds.build_vit, "vit_pp": ds.build_vit}[workload](arch, params, dev)
    x = torch.from_numpy(imgs).to(dev).to(torch.bfloat16).contiguous()
    lbg = torch.from_numpy(lb).to(dev).contiguous()
    logits = torch.empty((B, net.num_classes), dtype=torch.float32, device=dev)
    routes = torch.empty((net.n_gates, B), dtype=torch.int32, device=dev)
    ws = net.workspace(B, args.parts)

    def step():
        if args.parts == 1:
            ds.ds_forward(net, x, logit_bias=lbg, logits=logits, routes=routes, ws=ws)
        else:
            ds.ds_forward_parts(net, x, args.parts, logit_bias=lbg, logits=logits, routes=routes, ws=ws)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    # per-kernel HIP events are recorded on a sample of the timed steps (every --event-every-th):
    # the event packets keep consecutive kernels from overlapping, so bracketing every step would
    # lower the throughput being measured
    ds.ds_profile_reset()
    every = max(1, args.event_every)
    sampled = 0
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    sampled_steps = set()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        on = (not args.no_kernel_events) and i % every == min(every // 2, steps - 1)
        if on:
            ds.ds_profile_enable(True)
            sampled += 1
            sampled_steps.add(i)
        step()
        if on:
            ds.ds_profile_enable(False)
        marks[i + 1].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    gpu_ms = marks[0].elapsed_time(marks[steps])
    ms_per_step = max(wall_ms, gpu_ms) / steps
    # spread of the individual steps (those without kernel events, which cost 13-16 %)
    per = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps) if i not in sampled_steps) or [ms_per_step]
    pick = lambda q: per[min(len(per) - 1, int(q * len(per)))]
    prof = ds.ds_profile_read() if sampled else {}
    launches = ds.ds_profile_launches() if sampled else []

    rt = routes.cpu().numpy()
    cost = {"mbnet": C.mbnet_cost, "mbnet_pp": C.mbnet_cost, "resnet": C.resnet_cost, "resnet_pp": C.resnet_cost, "vit": C.vit_cost, "vit_stem": C.vit_cost,
            "vit_pp": C.vit_cost}[workload](arch, rt)
    roofline = None
    kernels = {}
    if prof:
        rows = match_launches(cost, launches, sampled) if args.parts == 1 else []
        if args.layers_json:
            json.dump(rows, open(args.layers_json, "w"))
        # the grouped GEMM class (linear / 1x1 / KxK layers) as one figure, as the dominant kernel of every network, ...
        gsel = [r for r in rows if r["kind"] in ("gemm", "gemm_taps") and "us" in r]
        ms = sum(prof[k][0] for k in GEMM_CLASSES)
        n = sum(prof[k][1] for k in GEMM_CLASSES)
        flops = (cost["gemm"]["flops"] + cost["gemm_taps"]["flops"]) * sampled
        nbytes = (cost["gemm"]["bytes"] + cost["gemm_taps"]["bytes"]) * sampled
        traffic = None
        tfile = os.path.join(ROOT, "profiles", f"gemm_traffic_{workload}_b256.txt")
        if os.path.exists(tfile) and B == 256:
            from paper_2109_10060_amd.profiling import kernel_source_hash
            t = json.load(open(tfile))
            if t.get("source_hash") == kernel_source_hash():   # stale once the kernel changes
                traffic = t["hbm_bytes_per_launch"]
        if n and ms > 0:
            tf = flops / (ms * 1e-3) / 1e12
            gbs = nbytes / (ms * 1e-3) / 1e9
            roofline = {"kernel": "gemm_kernel+conv3_kernel+thin_kernel", "bound": "mfma", "achieved": tf, "peak": PEAK_MFMA_BF16_TFLOPS,
                        "unit": "TFLOP/s", "frac": tf / PEAK_MFMA_BF16_TFLOPS, "traffic": traffic,
                        "algorithmic_bytes_per_launch": nbytes / n,
                        "launches_per_step": n / sampled, "avg_launch_us": ms * 1e3 / n,
                        "steps_sampled": sampled, "share_of_step": ms / (ms_per_step * sampled),
                        "hbm_view": {"achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS}}
            # ... and each of its three kernels against the roof its own launches select: the launches whose flop per byte
            # lies above the ridge against the matrix peak, the others against HBM bandwidth
            per_kernel = {}
            for kern in ("gemm_kernel", "conv3_kernel", "thin_kernel"):
                mine = [r for r in gsel if r["kernel"] == kern]
                if not mine:
                    continue
                entry = {"launches_per_step": len(mine), "ms_per_step": sum(r["us"] for r in mine) * 1e-3}
                for roof in ("mfma", "hbm"):
                    part = [r for r in mine if ("mfma" if r["flops"] / max(r["bytes"], 1.0) >= RIDGE else "hbm") == roof]
                    if part:
                        t_ms = sum(r["us"] for r in part) * 1e-3
                        rr = rates(sum(r["flops"] for r in part), sum(r["bytes"] for r in part), t_ms, True)
                        entry[roof + "_bound_launches"] = {"launches": len(part), "ms_per_step": t_ms, "tflops": rr["tflops"],
                                                           "algorithmic_gbs": rr["algorithmic_gbs"],
                                                           "frac": rr["frac_mfma"] if roof == "mfma" else rr["frac_hbm"]}
                per_kernel[kern] = entry
            roofline["per_kernel"] = per_kernel
            # the class as a whole under each roof: the launches above the ridge against the matrix peak, the rest against HBM
            by_roof = {}
            for roof in ("mfma", "hbm"):
                part = [r for r in gsel if ("mfma" if r["flops"] / max(r["bytes"], 1.0) >= RIDGE else "hbm") == roof]
                if part:
                    t_ms = sum(r["us"] for r in part) * 1e-3
                    rr = rates(sum(r["flops"] for r in part), sum(r["bytes"] for r in part), t_ms, True)
                    by_roof[roof] = {"launches": len(part), "ms_per_step": t_ms, "tflops": rr["tflops"],
                                     "algorithmic_gbs": rr["algorithmic_gbs"],
                                     "frac": rr["frac_mfma"] if roof == "mfma" else rr["frac_hbm"]}
            roofline["by_roof"] = by_roof
        # every kernel class with its algorithmic rates (same events, same sampled steps)
        merged = dict(prof)
        for k, (t, cnt) in merged.items():
            if not cnt:
                continue
            ck = {"conv3": "gemm_taps", "thin": "gemm"}.get(k, k)
            c = cost.get(ck, {"flops": 0.0, "bytes": 0.0}) if k not in ("conv3", "thin", "gemm", "gemm_taps") else None
            if c is None:
                mine = [r for r in gsel if (r["kernel"], r["kind"]) == (KERNEL_OF[k], "gemm_taps" if k in ("gemm_taps", "conv3") else "gemm")
                        or (k == "conv3" and r["kernel"] == "conv3_kernel") or (k == "thin" and r["kernel"] == "thin_kernel")]
                c = {"flops": sum(r["flops"] for r in mine), "bytes": sum(r["bytes"] for r in mine)}
            per_step_ms = t / sampled
            kernels[k] = {"ms_per_step": per_step_ms, "launches_per_step": cnt / sampled,
                          **{kk: vv for kk, vv in rates(c["flops"], c["bytes"], per_step_ms, k in GEMM_CLASSES or k == "attention").items()
                             if kk in ("tflops", "algorithmic_gbs", "roof", "frac")}}
        if args.breakdown:
            for k, v in kernels.items():
                sys.stderr.write(f"{k:10s} {v['ms_per_step']:8.3f} ms/step {int(v['launches_per_step']):4d} launches  "
                                 f"{v['tflops']:8.1f} TFLOP/s {v['algorithmic_gbs']:8.0f} GB/s  {v['roof']} {v['frac']:.3f}\n")

    out = {
        "metric": "images/sec at batch 256 (mixed gate widths)", "value": B / (ms_per_step * 1e-3), "unit": "images/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "ms_per_step_median": pick(0.5), "ms_per_step_p10": pick(0.1), "ms_per_step_p90": pick(0.9),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": label, "batch": B, "image": arch["image"], "route_mix": args.mix, "parts": args.parts,
                   "route_histogram": [np.bincount(r, minlength=net.T).tolist() for r in rt]},
        "roofline": roofline,
        "kernels": kernels,
    }
    if with_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(workload, arch, params, imgs, lb)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="", choices=["", "mbnet", "resnet", "vit", "vit_stem", "vit_pp", "mbnet_pp", "resnet_pp", "linear"],
                    help="default: config 4 (DS-ResNet) as the headline line, with configs 3 (DS-MBNet) and 5 (DS-ViT) measured "
                         "after it and reported under other_workloads; naming a workload runs that one only")
    ap.add_argument("--batch", type=int, default=256)
    ap.add_argument("--parts", type=int, default=1,
                    help="run the batch as this many concurrent shares (ds_forward_parts, 1..4); 1 = ds_forward")
    ap.add_argument("--mix", default="uniform", choices=["uniform", "skewed"],
                    help="route mix: every route about equally often (default), or half of the batch on the smallest "
                         "route at early gates / the largest route at late gates")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="do not bracket kernel launches with HIP events (roofline is then null)")
    ap.add_argument("--event-every", type=int, default=5,
                    help="bracket the kernels of every N-th timed step with HIP events (1 = every step)")
    ap.add_argument("--breakdown", action="store_true", help="print the per-kernel-class table to stderr")
    ap.add_argument("--layers-json", default="", metavar="PATH",
                    help="write the per-launch work list of one step with the measured duration of each launch")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="only run a plain device copy of MIB mebibytes 5 times (reference for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py measures one GPU: the library has no multi-GPU path (--gpus must be 1)")

    if args.workload == "linear" and not args.copy_calibration:
        return run_linear(args)

    import torch
    import paper_2109_10060_amd as ds

    ds.load()
    if args.copy_calibration:
        n = args.copy_calibration << 20
        src = torch.empty(n, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes": n, "repeats": 5}))
        return
    out = run_net(args.workload or "resnet", args, args.steps, args.warmup, not args.no_cpu_baseline)
    if not args.workload:
        # configs 3 and 5 ride along in the default line (same protocol, fewer steps, no CPU leg), so that the recorded run
        # carries the depthwise / LayerNorm / attention kernels as well
        others = {}
        layers_json, args.layers_json = args.layers_json, ""
        for w in ("mbnet", "vit"):
            r = run_net(w, args, max(10, args.steps // 2), max(3, args.warmup // 2), False)
            others[w] = {k: r[k] for k in ("value", "unit", "ms_per_step", "ms_per_step_median", "steps", "warmup", "config",
                                           "roofline", "kernels")}
        args.layers_json = layers_json
        out["other_workloads"] = others
        if args.parts == 1:
            # the same batch through ds_forward_parts: four shares on streams of the library fill each other's launch ramps
            # and tails; reported beside the headline, which stays on ds_forward because overlapping kernels have no
            # duration of their own to hold against a roofline
            a4 = argparse.Namespace(**vars(args))
            a4.parts, a4.no_kernel_events, a4.layers_json = 4, True, ""
            r = run_net("resnet", a4, max(10, args.steps // 2), max(3, args.warmup // 2), False)
            out["concurrent_shares"] = {"entry_point": "ds_forward_parts", "parts": 4,
                                        **{k: r[k] for k in ("value", "unit", "ms_per_step", "ms_per_step_median", "steps", "warmup")}}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
