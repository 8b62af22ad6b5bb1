"""The algorithmic-work model behind bench.py's roofline numerators, checked against the oracle's multiply-add
counts (which are pinned to the figures the paper prints) and against hand counts of bytes."""
import subprocess
import sys
import os

import numpy as np

import workloads as WL
from oracle import ds_oracle as O
from paper_2109_10060_amd import cost as C

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _macs(cost, kinds):
    return sum(cost[k]["flops"] for k in kinds if k in cost) / 2.0


def test_full_width_flops_equal_the_multiply_add_counts():
    B = 3
    a = WL.mbnet_arch()
    c = C.mbnet_cost(a, np.full(B, a["T"] - 1))
    want = O.madds_mbnet(a, a["cin"][-1], a["cout"][-1], int(a["cout"][-1, -1]))
    assert abs(_macs(c, ["stem", "dwconv", "gemm", "head"]) / B - want) / want < 1e-9
    r = WL.resnet_arch()
    c = C.resnet_cost(r, np.full((4, B), 3))
    want = O.madds_resnet(r, r["mid"][:, 3], r["out"][:, 3])
    assert abs(_macs(c, ["stem", "gemm", "gemm_taps", "head"]) / B - want) / want < 1e-9
    v = WL.vit_arch(routes="diag")
    c = C.vit_cost(v, np.full(B, 3))
    d_e, h, hid = (int(x) for x in v["routes"][3])
    want = O.madds_vit(v, d_e, h, hid)
    assert abs(_macs(c, ["gemm", "attention", "head"]) / B - want) / want < 1e-9


def test_sliced_routes_cost_less_and_depth_routes_skip_layers():
    r = WL.resnet_arch()
    full = C.resnet_cost(r, np.full((4, 8), 3))
    quarter = C.resnet_cost(r, np.zeros((4, 8), np.int64))
    assert quarter["gemm_taps"]["flops"] * 15.9 < full["gemm_taps"]["flops"] < quarter["gemm_taps"]["flops"] * 16.1   # r^2
    d = WL.resnet_arch(routes="depth")
    shallow = C.resnet_cost(d, np.full((4, 8), 6))       # ratio 1.0, one block fewer per stage
    deep = C.resnet_cost(d, np.full((4, 8), 7))
    assert shallow["gemm_taps"]["launches"] == deep["gemm_taps"]["launches"] - 4
    v = WL.vit_arch(routes="depth")
    c10 = C.vit_cost(v, np.full(4, 9))                    # widest route, depth - 2
    c12 = C.vit_cost(v, np.full(4, 11))
    assert c12["attention"]["launches"] - c10["attention"]["launches"] == 2
    assert abs(c12["attention"]["flops"] / c10["attention"]["flops"] - 12 / 10) < 1e-9


def test_gemm_bytes_count_each_operand_once():
    # one 1x1 layer, 2 samples of 5 rows, widths 8 -> 16 and 16 -> 32: in + out (bf16) + the union of the weight slices
    c = C.Cost()
    C._gemm(c, "gemm", 5, 5, 1, [8, 16], [16, 32])
    assert c["gemm"]["flops"] == 2 * 5 * (8 * 16 + 16 * 32)
    assert c["gemm"]["bytes"] == 2 * 5 * (8 + 16) + 2 * 5 * (16 + 32) + 2 * 16 * 32


def test_bench_refuses_more_than_one_gpu():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0 and "one GPU" in (p.stderr + p.stdout)
