"""ds_sliced_linear_noalloc (the entry point for callers that cannot allocate device memory) against
ds_sliced_linear and the CPU oracle: two calls in a row on the library's built-in scratch, the second
with a smaller input, so that stale records of the first call's row-tile list would show."""
import ctypes

import numpy as np
import pytest
import torch

import workloads as WL
from oracle import ds_oracle as O

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
TOL_BF16 = 2e-2


def dev(a, dtype=torch.float32):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV).to(dtype).contiguous()


def _case(gpu_lib, c, act, with_res):
    B, N, K = c["B"], c["N"], c["K"]
    perm, inv, off = gpu_lib.ds_route_bucket(dev(c["route"], torch.int32), c["T"])
    g = gpu_lib.make_groups(off, perm, c["k_in"], c["k_out"])
    x, w, bias = dev(c["x"], torch.bfloat16), dev(c["w"], torch.bfloat16), dev(c["bias"])
    res_h = res = None
    if with_res:
        res_h = WL.nets.as_bf16_values(WL.nets.Draw(9).normal((B, N, 4 * K)))
        res = dev(res_h, torch.bfloat16)
    y_ref = torch.full((B, N, 4 * K), float("nan"), dtype=torch.bfloat16, device=DEV)
    y_new = torch.full((B, N, 4 * K), float("nan"), dtype=torch.bfloat16, device=DEV)
    gpu_lib.ds_sliced_linear(x, w, bias, g, act=act, residual=res, y=y_ref)
    if not _case.warm:          # the first call on a device looks up the scratch array (and loads its code object)
        gpu_lib.ds_sliced_linear_noalloc(x, w, bias, g, y_new, act=act, residual=res)
        y_new.fill_(float("nan"))
        _case.warm = True
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    gpu_lib.ds_sliced_linear_noalloc(x, w, bias, g, y_new, act=act, residual=res)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before, "the call changed the device's free memory"
    # same kernels on the same inputs: bit-identical, canaried tails included
    assert torch.equal(y_ref.view(torch.int16), y_new.view(torch.int16))
    yh = y_new.to(torch.float64).cpu().numpy()
    worst = 0.0
    for b in range(B):
        ki, ko = int(c["k_in"][c["route"][b]]), int(c["k_out"][c["route"][b]])
        want = O.sliced_linear(c["x"][b, :, :ki], c["w"], c["bias"], ko)
        if with_res:
            want = want + res_h[b, :, :ko]
        if act == 2:
            want = O.gelu(want)
        want = O.bf16_round(want)
        assert np.all(np.isnan(yh[b, :, ko:])), "tail beyond the valid slice was written"
        worst = max(worst, float(np.max(np.abs(yh[b, :, :ko] - want)) / np.max(np.abs(want))))
    return worst


_case.warm = False


def test_noalloc_two_calls_second_smaller(gpu_lib):
    big = WL.config2(seed=301, B=24, N=197, K=96)            # 37 row tiles + ragged tails, four buckets
    assert _case(gpu_lib, big, act=0, with_res=False) < TOL_BF16
    small = WL.config2(seed=302, B=5, N=37, K=48)            # 2 row tiles: most of the first list is stale now
    assert _case(gpu_lib, small, act=2, with_res=False) < TOL_BF16
    assert _case(gpu_lib, small, act=0, with_res=True) < TOL_BF16


def test_noalloc_rejects_sizes_beyond_the_built_in_scratch_and_accepts_an_empty_batch(gpu_lib):
    lib = gpu_lib.load()
    c = WL.config2(seed=303, B=2, N=8, K=48)
    off = torch.zeros(5, dtype=torch.int32, device=DEV)
    g = gpu_lib.make_groups(off, None, c["k_in"], c["k_out"])
    rows = 128 * 40000                                        # 40000 row tiles per sample
    rc = lib.ds_sliced_linear_noalloc(None, ctypes.c_int64(48), None, ctypes.c_int64(48), 192, 48, None, ctypes.byref(g),
                                      1, rows, 0, None, ctypes.c_int64(0), None, 1, ctypes.c_int64(192), None)
    assert rc == gpu_lib.DS_EWORKSPACE and b"built-in scratch" in lib.ds_last_error()
    x0 = torch.zeros((0, 8, 48), dtype=torch.bfloat16, device=DEV)
    y0 = torch.zeros((0, 8, 192), dtype=torch.bfloat16, device=DEV)
    gpu_lib.ds_sliced_linear_noalloc(x0, dev(c["w"], torch.bfloat16), None, g, y0)
