"""Algorithmic work of one ds_forward pass, per kernel class, for a given route assignment.

flops: 2 x multiply-adds the method itself must do on the valid slices (not the dense work
it avoids).  bytes: each kernel reads its valid input once and writes its valid output once
(bf16), reads a residual once where it has one, and reads the union of the weight slices
once per launch.  These are the numerators of the roofline fractions bench.py reports.
"""
from __future__ import annotations

from collections import defaultdict

import numpy as np


class Cost(defaultdict):
    """Per kernel class totals (self[kind]) and, in launch order, one record per launch (self.launches)."""

    def __init__(self):
        super().__init__(lambda: {"flops": 0.0, "bytes": 0.0, "launches": 0})
        self.launches = []

    def add(self, kind, flops, nbytes, name="", shape="", merge=False):
        """merge: the work rides along in the previous launch of this kind (a chained layer): no new launch."""
        e = self[kind]
        e["flops"] += float(flops)
        e["bytes"] += float(nbytes)
        if merge:
            last = next(r for r in reversed(self.launches) if r["kind"] == kind)
            last["flops"] += float(flops)
            last["bytes"] += float(nbytes)
            last["name"] += " + " + name
            return
        e["launches"] += 1
        self.launches.append({"kind": kind, "name": name, "shape": shape, "flops": float(flops), "bytes": float(nbytes)})


def _osz(n, k, s, p):
    return (n + 2 * p - k) // s + 1


def _gemm(cost, kind, rows_in, rows_out, kk, k_in, k_out, residual=False, out_bytes=2, chained=False, name=""):
    """k_in, k_out: per-sample arrays of valid widths.  chained: the layer runs inside the launch that
    produced its input rows, so it adds flops, its output and its weights, but no input read and no launch."""
    k_in, k_out = np.asarray(k_in, np.float64), np.asarray(k_out, np.float64)
    flops = 2.0 * rows_out * kk * np.sum(k_in * k_out)
    nbytes = (0.0 if chained else 2.0 * rows_in * np.sum(k_in)) + out_bytes * rows_out * np.sum(k_out) * (2 if residual else 1)
    nbytes += 2.0 * kk * float(np.max(k_in)) * float(np.max(k_out))
    live = k_in * k_out > 0
    shape = (f"rows {int(rows_out) * int(live.sum())} k {int(k_in[live].min()) if live.any() else 0}..{int(k_in.max())}"
             f"{'x' + str(int(kk)) if kk > 1 else ''} n {int(k_out[live].min()) if live.any() else 0}..{int(k_out.max())}")
    cost.add(kind, flops, nbytes, name=name, shape=shape, merge=chained)


def mbnet_cost(arch, routes) -> Cost:
    routes = np.asarray(routes).reshape(-1)
    B = routes.shape[0]
    c = Cost()
    r = _osz(arch["image"], 3, 2, 1)
    so = arch["stem_out"]
    c.add("stem", 2.0 * B * r * r * 27 * so, B * (3 * arch["image"] ** 2 * 2 + r * r * so * 2), name="stem 3x3/2")
    for i, (_ci, _co, s) in enumerate(arch["blocks"]):
        rin = r
        r = _osz(r, 3, s, 1)
        ci, co = arch["cin"][routes, i].astype(np.float64), arch["cout"][routes, i].astype(np.float64)
        kk = arch["ksize"][routes, i].astype(np.float64) ** 2 if "ksize" in arch else 9.0
        cif, cof = int(_ci), int(_co)
        if (i < arch["gate_after"] and "ksize" not in arch and cif % 8 == 0 and cif <= 128 and cof % 8 == 0
                and cof <= 128 and r % (4 if s == 1 else 2) == 0):
            # an unsliced block the library runs as one kernel (depthwise map kept in LDS): counted as one launch
            # of the depthwise class that reads the block's input and writes the pointwise output
            c.add("dwconv", 2.0 * r * r * (kk * ci).sum() + 2.0 * r * r * np.sum(ci * co),
                  2.0 * rin * rin * ci.sum() + 2.0 * r * r * co.sum() + 2.0 * cif * cof, name=f"ds{i} dw+pw fused",
                  shape=f"{rin}x{rin}x{cif} -> {r}x{r}x{cof}")
        else:
            c.add("dwconv", 2.0 * r * r * (kk * ci).sum(), 2.0 * (rin * rin + r * r) * ci.sum(), name=f"ds{i} dw",
                  shape=f"{rin}x{rin} s{s} c {int(ci.min())}..{int(ci.max())}")
            _gemm(c, "gemm", r * r, r * r, 1, ci, co, name=f"ds{i} pw")
        if i == arch["gate_after"] - 1:
            c.add("gate", 2.0 * B * (r * r * co[0]), 2.0 * B * r * r * co[0], name="gate pool + MLP")
    cl = arch["cout"][routes, -1].astype(np.float64)
    c.add("head", 2.0 * arch["num_classes"] * cl.sum(), 2.0 * r * r * cl.sum() + 2.0 * arch["num_classes"] * cl.max(),
          name="pool + classifier")
    return c


def resnet_cost(arch, routes) -> Cost:
    routes = np.asarray(routes).reshape(4, -1)
    B = routes.shape[1]
    c = Cost()
    r1 = _osz(arch["image"], 7, 2, 3)
    so = arch["stem_out"]
    c.add("stem", 2.0 * B * r1 * r1 * 147 * so, B * (3 * arch["image"] ** 2 * 2 + r1 * r1 * so * 2), name="stem 7x7/2 (+ max-pool)")
    r = _osz(r1, 3, 2, 1)
    c.add("maxpool", 0.0, 2.0 * B * so * (r1 * r1 + r * r), name="max-pool")
    cprev = np.full(B, so, np.float64)
    for s, nb in enumerate(arch["blocks"]):
        mid = arch["mid"][s][routes[s]].astype(np.float64)
        out = arch["out"][s][routes[s]].astype(np.float64)
        if s == 0 or not arch.get("single_gate"):
            c.add("gate", 2.0 * r * r * cprev.sum(), 2.0 * r * r * cprev.sum(), name=f"s{s} gate pool + MLP")
        # stages with slices of at most 128 channels run a block's last convolution and the next block's first one
        # as one launch (the wide map is written once and not read back)
        mids, outs = arch["mid"][s], arch["out"][s]
        chain = bool(mids.max() <= 128 and outs.max() >= 128 and not (mids % 8).any() and not (outs % 8).any())
        for b in range(nb):
            # dynamic depth: samples whose route has run its blocks of this stage contribute nothing
            on = (arch["nblk"][s][routes[s]] > b).astype(np.float64) if arch.get("nblk") is not None else np.ones(B)
            if not on.any():
                break
            stride = 2 if (b == 0 and s > 0) else 1
            ro = _osz(r, 3, stride, 1)
            cin = (cprev if b == 0 else out) * on
            m, o = mid * on, out * on
            if b == 0:
                _gemm(c, "gemm", ro * ro, ro * ro, 1, cin, o, name=f"s{s}.b{b}.proj")      # 1x1 projection reads only the strided pixels
            _gemm(c, "gemm", r * r, r * r, 1, cin, m, chained=chain and b > 0, name=f"s{s}.b{b}.c1")
            _gemm(c, "gemm_taps", r * r, ro * ro, 9, m, m, name=f"s{s}.b{b}.c2 3x3" + ("/2" if stride == 2 else ""))
            _gemm(c, "gemm", ro * ro, ro * ro, 1, m, o, residual=True, name=f"s{s}.b{b}.c3+res")
            r = ro
        cprev = out
    c.add("head", 2.0 * arch["num_classes"] * cprev.sum(),
          2.0 * r * r * cprev.sum() + 2.0 * arch["num_classes"] * cprev.max(), name="pool + classifier")
    return c


def vit_cost(arch, routes) -> Cost:
    routes = np.asarray(routes).reshape(-1)
    tab = arch["routes"][routes].astype(np.float64)
    de, h, hid = tab[:, 0], tab[:, 1], tab[:, 2]
    hd = h * arch["head_dim"]
    N, B = arch["tokens"], routes.shape[0]
    c = Cost()
    C = arch.get("stem_dim", 0)
    if C:
        r = _osz(arch["image"], 7, 2, 3)
        full = np.full(B, C, np.float64)
        c.add("stem", 2.0 * B * r * r * 147 * C, B * (3 * arch["image"] ** 2 * 2 + r * r * C * 2), name="stem 7x7/2")
        for _ in range(2):
            if C % 8 == 0 and C <= 128 and r % 4 == 0:
                # the block runs as one kernel (depthwise map kept in LDS): one launch of the depthwise class
                c.add("dwconv", 2.0 * B * r * r * 9 * C + 2.0 * B * r * r * C * C, 2.0 * 2 * B * r * r * C + 2.0 * C * C,
                      name="stem dw+pw fused")
            else:
                c.add("dwconv", 2.0 * B * r * r * 9 * C, 2.0 * 2 * B * r * r * C, name="stem dw")
                _gemm(c, "gemm", r * r, r * r, 1, full, full, name="stem pw")
        c.add("gate", 2.0 * B * r * r * C, 2.0 * B * r * r * C, name="gate pool + MLP")
        # the patch projection reads every pixel of the stem's map once
        _gemm(c, "gemm_taps", (N - 1) * arch["patch"] ** 2, N - 1, 1, full, de, name="patch embed conv")
        c["gemm_taps"]["flops"] += 2.0 * (N - 1) * (arch["patch"] ** 2 - 1) * C * de.sum()
    else:
        kp = 3 * arch["patch"] ** 2
        c.add("index", 0.0, 2.0 * 2 * B * (N - 1) * kp, name="patch extraction")
        _gemm(c, "gemm", N - 1, N - 1, 1, np.full(B, kp), de, name="patch embed")
    full = tab[:, :3].copy()
    for l in range(arch["depth"]):
        # dynamic depth: a route that runs fewer than l + 1 blocks contributes nothing to this layer
        on = (tab[:, 3] > l).astype(np.float64) if tab.shape[1] > 3 else np.ones(B)
        if not on.any():
            break
        de, h, hid = full[:, 0] * on, full[:, 1] * on, full[:, 2] * on
        hd = h * arch["head_dim"]
        c.add("layernorm", 8.0 * N * de.sum(), 4.0 * N * de.sum(), name=f"l{l}.ln1")
        k_in, k_out = de, 3 * hd
        _gemm(c, "gemm", N, N, 1, k_in, k_out, name=f"l{l}.qkv")
        c.add("attention", 4.0 * N * N * hd.sum(), 2.0 * 4 * N * hd.sum(), name=f"l{l}.attention")
        _gemm(c, "gemm", N, N, 1, hd, de, residual=True, name=f"l{l}.proj+res")
        c.add("layernorm", 8.0 * N * de.sum(), 4.0 * N * de.sum(), name=f"l{l}.ln2")
        _gemm(c, "gemm", N, N, 1, de, hid, name=f"l{l}.fc1+gelu")
        _gemm(c, "gemm", N, N, 1, hid, de, residual=True, name=f"l{l}.fc2+res")
    de = full[:, 0]
    c.add("layernorm", 8.0 * de.sum(), 4.0 * de.sum(), name="final ln (class token)")
    c.add("head", 2.0 * arch["num_classes"] * de.sum(), 2.0 * de.sum() + 2.0 * arch["num_classes"] * de.max(), name="classifier")
    return c
