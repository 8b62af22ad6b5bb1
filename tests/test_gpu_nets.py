"""End-to-end GPU parity of ds_forward against the per-sample CPU oracle.

Small nets: every sample of a mixed-route batch is checked.  Full-size configurations
(batch 256, 224x224): the launch configuration the benchmark times; a seeded sample of
images spanning the routes is recomputed one by one by the oracle, and batch-level
properties (permutation equivariance, bit-exact repeatability, route histogram) are
checked on the whole batch.  At batch 256 the checked images are chosen so that every
route of the network occurs among them (all 14 widths, all 16 route pairs at each stage
boundary, all 48 embed / head / MLP tuples), and besides the logits the outputs of two to
four blocks inside the network (ds_forward_taps) are compared with the oracle's.
Tolerance: max |gpu - oracle| / max |oracle| <= 2e-2 per tensor (bf16 storage, fp32
accumulation); the element-wise form is recorded beside it (tests/parity.py).  Routes
must match the oracle exactly: the seeded logit bias keeps every gate margin far above
the bf16 noise of the features, and the tests assert that no sample needed the exemption
for gates that read bf16 features.
"""
import numpy as np
import pytest
import torch

import workloads as WL
from oracle import ds_oracle as O

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 2e-2
S = WL.BASE_SEED


def dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV).to(dtype).contiguous()


from tests.parity import both as _both  # noqa: E402


def relerr(got, want):
    """The stated bound's form, max |gpu - oracle| / max |oracle|; the element-wise form is recorded beside it."""
    return _both(got, want)[0]


def _taps_gpu(gpu_lib, net, xg, shapes, **kw):
    """Runs ds_forward_taps; shapes: {block: (rows, C_stored)}.  Buffers start as NaN, so unwritten tails show."""
    B = xg.shape[0]
    bufs = {k: torch.full((B, r, c), float("nan"), dtype=torch.bfloat16, device=DEV) for k, (r, c) in shapes.items()}
    logits, routes = gpu_lib.ds_forward_taps(net, xg, bufs, **kw)
    torch.cuda.synchronize()
    return logits, routes, bufs


def _check_tap(buf, b, want_chw):
    """buf[b]: [rows, C_stored] channels-last; want_chw: the oracle's [c, H, W] (or [tokens, c]) block output."""
    want = np.asarray(want_chw, np.float64)
    want = want.reshape(want.shape[0], -1).T if want.ndim == 3 else want
    c = want.shape[1]
    got = buf[b].to(torch.float64).cpu().numpy()
    assert np.all(np.isnan(got[:, c:])), "tap tail beyond the valid slice was written"
    return relerr(got[:, :c], want)


# ------------------------------------------------------------------ DS-MBNet
def _mb_case(gpu_lib, arch, params, imgs, lb, check, tap_blocks=()):
    net = gpu_lib.build_mbnet(arch, params, DEV)
    B = imgs.shape[0]
    xg, lbg = dev(imgs, torch.bfloat16), dev(lb[None], torch.float32)
    logits, routes = gpu_lib.ds_forward(net, xg, logit_bias=lbg)
    torch.cuda.synchronize()
    bufs = {}
    if tap_blocks:
        res = arch["image"] // 2
        shapes = {}
        for i, (_ci, co, st) in enumerate(arch["blocks"]):
            res = (res - 1) // st + 1
            if i in tap_blocks:
                shapes[i] = (res * res, co)
        l1, r1, bufs = _taps_gpu(gpu_lib, net, xg, shapes, logit_bias=lbg)
        assert torch.equal(l1, logits) and torch.equal(r1, routes)      # taps do not disturb the pass
    lg, rt = logits.cpu().numpy(), routes.cpu().numpy()[0]
    worst = 0.0
    for b in check:
        taps = {}
        want, t, z = O.forward_mbnet(arch, params, imgs[b], logit_bias=lb[b], taps=taps)
        assert O.gate_margin(z) > 1e-2
        assert rt[b] == t, (b, rt[b], t)
        worst = max(worst, relerr(lg[b], want))
        for i in tap_blocks:
            worst = max(worst, _check_tap(bufs[i], b, taps[f"ds{i}"]))
    assert worst < TOL, worst
    # teacher-forced routes give the same result as the free-running gate when routes agree
    l2, r2 = gpu_lib.ds_forward(net, xg, route_override=routes.clone(), logit_bias=lbg)
    assert torch.equal(l2, logits) and torch.equal(r2, routes)
    return net, xg, lbg, logits, routes


def test_mbnet_small_all_samples(gpu_lib):
    arch = WL.mbnet_arch(image=64, width_div=4)
    params = WL.mbnet_params(arch, S + 30)
    B = 31
    imgs = WL.images(S + 31, B, 64)
    lb = WL.seeded_logit_bias(S + 32, B, arch["T"])
    _, _, _, _, routes = _mb_case(gpu_lib, arch, params, imgs, lb, range(B))
    assert len(set(routes.cpu().numpy()[0].tolist())) == arch["T"]       # every width occurs


@pytest.mark.parametrize("B", [16, 5])
def test_mbnet_full_width_small_images_all_samples(gpu_lib, B):
    # the stored widths of the paper's network (32 .. 1024) on 64x64 images: the unsliced blocks in front of the gate
    # take the fused depthwise + pointwise kernel on 32x32, 16x16 and 8x8 maps (whole tiles, two tiles per sample, and
    # a ragged tile of 64 pixels), with whole samples per die (B = 16) and in plain tile order (B = 5)
    arch = WL.mbnet_arch(image=64)
    params = WL.mbnet_params(arch, S + 33)
    imgs = WL.images(S + 34, B, 64)
    lb = WL.seeded_logit_bias(S + 35, B, arch["T"])
    _mb_case(gpu_lib, arch, params, imgs, lb, range(B))


def test_mbnet_config3_batch256(gpu_lib):
    arch = WL.mbnet_arch()
    params = WL.mbnet_params(arch, S + 3)
    B = 256
    imgs = WL.images(S + 103, B)
    lb = WL.seeded_logit_bias(S + 203, B, arch["T"])
    target = np.argmax(lb, axis=1)
    # 32 images: the first two of every width, then the last images of the batch
    check = sorted({int(b) for t in range(14) for b in np.where(target == t)[0][:2]} | {252, 253, 254, 255})
    assert len(check) == 32 and set(target[check].tolist()) == set(range(14))
    net, xg, lbg, logits, routes = _mb_case(gpu_lib, arch, params, imgs, lb, check, tap_blocks=(2, 5, 12))
    rt = routes.cpu().numpy()[0]
    assert np.array_equal(rt, target)
    assert np.bincount(rt, minlength=14).min() >= 18
    # permuting the batch permutes the logits, bit for bit (bucketing is invisible)
    pi = torch.randperm(B, generator=torch.Generator().manual_seed(1)).to(DEV)
    l3, r3 = gpu_lib.ds_forward(net, xg[pi].contiguous(), logit_bias=lbg[:, pi].contiguous())
    assert torch.equal(l3, logits[pi]) and torch.equal(r3, routes[:, pi])


def test_mbnet_pp_small_all_samples(gpu_lib):
    # DS-MBNet++: 5x5 depthwise filters before the gate, stored 7x7 filters used at kernel size 3, 5 or 7 after it
    arch = WL.mbnet_pp_arch(image=64, width_div=2)
    params = WL.mbnet_params(arch, S + 33)
    B = 29
    imgs = WL.images(S + 34, B, 64)
    lb = WL.seeded_logit_bias(S + 35, B, arch["T"])
    net, xg, lbg, logits, routes = _mb_case(gpu_lib, arch, params, imgs, lb, range(B))
    assert len(set(routes.cpu().numpy()[0].tolist())) == arch["T"]


def test_mbnet_pp_batch256(gpu_lib):
    arch = WL.mbnet_pp_arch()
    params = WL.mbnet_params(arch, S + 36)
    B = 256
    imgs = WL.images(S + 136, B)
    lb = WL.seeded_logit_bias(S + 236, B, arch["T"])
    target = np.argmax(lb, axis=1)
    check = sorted({int(b) for t in range(12) for b in np.where(target == t)[0][:2]})      # every path twice
    _mb_case(gpu_lib, arch, params, imgs, lb, check, tap_blocks=(5, 12))


# ------------------------------------------------------------------ DS-ResNet
def _rn_case(gpu_lib, arch, params, imgs, lb, check, tap_stage_ends=False, max_exempt=0):
    """max_exempt: how many checked samples may take the exemption for gates that read bf16 features (a route
    that differs from the oracle's where the oracle's margin is inside that noise); 0 under the seeded bias."""
    net = gpu_lib.build_resnet(arch, params, DEV)
    xg, lbg = dev(imgs, torch.bfloat16), dev(lb, torch.float32)
    logits, routes = gpu_lib.ds_forward(net, xg, logit_bias=lbg)
    torch.cuda.synchronize()
    bufs, tap_of = {}, {}
    if tap_stage_ends:
        res, blk, shapes = arch["image"] // 4, 0, {}
        for s, nb in enumerate(arch["blocks"]):
            res = res if s == 0 else (res - 1) // 2 + 1
            blk += nb
            shapes[blk - 1] = (res * res, 4 * int(arch["widths"][s]))
            tap_of[blk - 1] = f"s{s}.b{nb - 1}"
        l1, r1, bufs = _taps_gpu(gpu_lib, net, xg, shapes, logit_bias=lbg)
        assert torch.equal(l1, logits) and torch.equal(r1, routes)
    lg, rt = logits.cpu().numpy(), routes.cpu().numpy()
    worst, exempt = 0.0, 0
    for b in check:
        taps = {}
        want, ro, zs = O.forward_resnet(arch, params, imgs[b], logit_bias=lb[:, b], taps=taps)
        if rt[:, b].tolist() != ro:
            # mid-network gates read bf16 features, so a gate may only disagree where the oracle's
            # margin is within that noise; activations are then compared under the GPU's routes
            exempt += 1
            s0 = next(s for s in range(4) if rt[s, b] != ro[s])
            assert O.gate_margin(zs[s0]) < 2e-2 * np.max(np.abs(zs[s0])), (b, rt[:, b], ro, zs[s0])
            taps = {}
            want, _, _ = O.forward_resnet(arch, params, imgs[b], logit_bias=lb[:, b], route_override=rt[:, b], taps=taps)
        worst = max(worst, relerr(lg[b], want))
        for blk, name in tap_of.items():
            if name in taps:            # a route of lesser depth stops before the stage's last stored block
                worst = max(worst, _check_tap(bufs[blk], b, taps[name]))
    assert worst < TOL, worst
    assert exempt <= max_exempt, f"{exempt} checked samples needed the bf16-gate exemption"
    return net, xg, lbg, logits, routes


def _cover_boundary_pairs(rt, n):
    """Indices of n samples such that every (route of stage s-1, route of stage s) pair that occurs in rt [4, B] is
    among them, chosen greedily; filled up with the first samples not yet taken."""
    B = rt.shape[1]
    need = {(s, int(rt[s - 1, b]), int(rt[s, b])) for s in range(1, 4) for b in range(B)} | {(0, 0, int(r)) for r in rt[0]}
    keys = lambda b: {(s, int(rt[s - 1, b]), int(rt[s, b])) for s in range(1, 4)} | {(0, 0, int(rt[0, b]))}
    pick = []
    while need:
        b = max(range(B), key=lambda i: (len(keys(i) & need), -i))
        pick.append(b)
        need -= keys(b)
    pick += [b for b in range(B) if b not in pick][:max(0, n - len(pick))]
    return sorted(pick)


def _rn_bias(seed, B, T):
    return np.stack([WL.seeded_logit_bias(seed + s, B, T, amp=16.0) for s in range(4)])


def test_resnet_small_all_samples(gpu_lib):
    arch = WL.resnet_arch(image=64, width_div=2, blocks=(2, 2, 2, 2))
    params = WL.resnet_params(arch, S + 40)
    B = 37
    imgs = WL.images(S + 41, B, 64)
    lb = _rn_bias(S + 42, B, 4)
    net, xg, lbg, logits, routes = _rn_case(gpu_lib, arch, params, imgs, lb, range(B))
    # forcing the oracle's routes reproduces the free-running logits
    l2, _ = gpu_lib.ds_forward(net, xg, route_override=routes.clone())
    assert torch.equal(l2, logits)
    # a uniform batch on the largest route equals the static full network
    full = torch.full((4, B), 3, dtype=torch.int32, device=DEV)
    l3, _ = gpu_lib.ds_forward(net, xg, route_override=full)
    want, _, _ = O.forward_resnet(arch, params, imgs[5], route_override=[3, 3, 3, 3])
    assert relerr(l3[5].cpu().numpy(), want) < TOL


def test_resnet_chained_blocks_ragged_rows_all_samples(gpu_lib):
    # three blocks per early stage at 48 x 48 input: 144 and 36 rows per sample, so the row tiles of the launches that
    # run a block's last convolution together with the next block's first one straddle samples and end in a partial tile
    arch = WL.resnet_arch(image=48, width_div=2, blocks=(3, 3, 1, 1))
    params = WL.resnet_params(arch, S + 140)
    B = 21
    imgs = WL.images(S + 141, B, 48)
    lb = _rn_bias(S + 142, B, 4)
    _rn_case(gpu_lib, arch, params, imgs, lb, range(B))


def test_resnet_dynamic_depth_small_all_samples(gpu_lib):
    # 8 routes per stage: 4 widths x (all blocks | one block fewer); 64 groups per stage.  Samples on a
    # shallow route must come through the skipped blocks untouched while their neighbours are updated.
    arch = WL.resnet_arch(image=64, width_div=2, blocks=(2, 3, 3, 1), routes="depth")
    params = WL.resnet_params(arch, S + 45)
    B = 41
    imgs = WL.images(S + 46, B, 64)
    lb = _rn_bias(S + 47, B, 8)
    net, xg, lbg, logits, routes = _rn_case(gpu_lib, arch, params, imgs, lb, range(B))
    rt = routes.cpu().numpy()
    assert len(np.unique(rt % 2)) == 2          # both depths occur
    # a batch that is shallow everywhere, and one where whole stages have nothing left to run
    for pick in ([0, 2, 4, 6], [6, 6, 6, 6], [7, 7, 7, 7]):
        ov = torch.tensor(pick, dtype=torch.int32, device=DEV)[:, None].expand(4, B).contiguous()
        l2, _ = gpu_lib.ds_forward(net, xg, route_override=ov)
        want, _, _ = O.forward_resnet(arch, params, imgs[3], route_override=pick)
        assert relerr(l2[3].cpu().numpy(), want) < TOL, pick
    # an ill-formed depth table is rejected
    bad = dict(arch, nblk=arch["nblk"].copy())
    bad["nblk"][1, 2] = 4
    with pytest.raises(Exception):
        gpu_lib.ds_forward(gpu_lib.build_resnet(bad, params, DEV), xg, logit_bias=lbg)


def test_resnet_pp_single_gate_small_and_batch256(gpu_lib):
    # DS-ResNet++: one gate steers width and block count of all four stages (9 paths)
    arch = WL.resnet_arch(image=64, blocks=(3, 4, 8, 3), routes="pp")     # full widths: the table's steps of 32 need them
    params = WL.resnet_params(arch, S + 48)
    B = 19
    imgs = WL.images(S + 49, B, 64)
    lb = _rn_bias(S + 50, B, 9)
    net, xg, lbg, logits, routes = _rn_case(gpu_lib, arch, params, imgs, lb, range(B))
    rt = routes.cpu().numpy()
    assert (rt == rt[0]).all() and len(set(rt[0].tolist())) == 9
    arch = WL.resnet_arch(blocks=(3, 4, 8, 3), routes="pp")
    params = WL.resnet_params(arch, S + 51)
    B = 256
    imgs = WL.images(S + 151, B)
    lb = _rn_bias(S + 251, B, 9)
    target = np.argmax(lb[0], axis=1)
    check = [int(np.where(target == t)[0][0]) for t in range(9)]            # every path once
    net, xg, lbg, logits, routes = _rn_case(gpu_lib, arch, params, imgs, lb, check, tap_stage_ends=True)
    rt = routes.cpu().numpy()
    assert (rt == rt[0]).all() and np.array_equal(rt[0], target)


def test_resnet_config4_batch256(gpu_lib):
    arch = WL.resnet_arch()
    params = WL.resnet_params(arch, S + 4)
    B = 256
    imgs = WL.images(S + 104, B)
    lb = _rn_bias(S + 204, B, 4)
    target = np.argmax(lb, axis=2)                                  # [4, B]
    # 32 images covering all 4 first-stage routes and all 16 (previous, own) route pairs of every later stage
    check = _cover_boundary_pairs(target, 32)
    assert len(check) == 32
    net, xg, lbg, logits, routes = _rn_case(gpu_lib, arch, params, imgs, lb, check, tap_stage_ends=True)
    rt = routes.cpu().numpy()
    for s in range(1, 4):
        assert len({(int(rt[s - 1, b]), int(rt[s, b])) for b in check}) == 16
    assert np.mean(rt == target) > 0.97                              # the seeded bias decides nearly every gate
    for s in range(1, 4):
        assert len(set(zip(rt[s - 1].tolist(), rt[s].tolist()))) == 16   # all 16 (r_prev, r) boundary pairs occur
    pi = torch.randperm(B, generator=torch.Generator().manual_seed(2)).to(DEV)
    l3, r3 = gpu_lib.ds_forward(net, xg[pi].contiguous(), logit_bias=lbg[:, pi].contiguous())
    assert torch.equal(l3, logits[pi]) and torch.equal(r3, routes[:, pi])


# ------------------------------------------------------------------ DS-ViT
def _vit_taps(gpu_lib, arch, net, xg, lbg, logits, routes, tap_layers):
    if not tap_layers:
        return {}
    shapes = {l: (arch["tokens"], arch["embed"]) for l in tap_layers}
    l1, r1, bufs = _taps_gpu(gpu_lib, net, xg, shapes, logit_bias=lbg)
    assert torch.equal(l1, logits) and torch.equal(r1, routes)
    return bufs


def _vit_case(gpu_lib, arch, params, imgs, lb, check, tap_layers=()):
    net = gpu_lib.build_vit(arch, params, DEV)
    xg, lbg = dev(imgs, torch.bfloat16), dev(lb[None], torch.float32)
    logits, routes = gpu_lib.ds_forward(net, xg, logit_bias=lbg)
    torch.cuda.synchronize()
    bufs = _vit_taps(gpu_lib, arch, net, xg, lbg, logits, routes, tap_layers)
    lg, rt = logits.cpu().numpy(), routes.cpu().numpy()[0]
    assert np.array_equal(rt, [O.gate_route(z) for z in lb])
    worst = 0.0
    for b in check:
        taps = {}
        want = O.forward_vit(arch, params, imgs[b], int(rt[b]), taps=taps)
        worst = max(worst, relerr(lg[b], want))
        for l in tap_layers:
            if f"l{l}" in taps:
                worst = max(worst, _check_tap(bufs[l], b, taps[f"l{l}"]))
    assert worst < TOL, worst
    return net, xg, lbg, logits, routes


@pytest.mark.parametrize("routes", ["cross", "diag"])
def test_vit_small_all_samples(gpu_lib, routes):
    arch = WL.vit_arch(image=64, patch=16, depth=2, routes=routes)      # 17 tokens, DeiT-S widths
    params = WL.vit_params(arch, S + 50)
    B = 53
    imgs = WL.images(S + 51, B, 64)
    lb = WL.seeded_logit_bias(S + 52, B, arch["T"])
    _vit_case(gpu_lib, arch, params, imgs, lb, range(B))


def test_vit_dynamic_depth_small_all_samples(gpu_lib):
    # 12 routes = 4 nested widths x 3 depths (2, 3 or 4 of the 4 stored blocks): rows of a route that has
    # finished must pass through the remaining blocks untouched
    arch = WL.vit_arch(image=64, patch=16, depth=4, routes="depth")
    params = WL.vit_params(arch, S + 60)
    B = 40
    imgs = WL.images(S + 61, B, 64)
    lb = WL.seeded_logit_bias(S + 62, B, arch["T"])
    net, xg, lbg, logits, routes = _vit_case(gpu_lib, arch, params, imgs, lb, range(B))
    assert len(set(routes.cpu().numpy()[0].tolist())) == arch["T"]
    # a depth of 0 blocks is legal: embedding, final LayerNorm and classifier only
    arch0 = dict(arch, routes=arch["routes"].copy())
    arch0["routes"][:, 3] = 0
    _vit_case(gpu_lib, arch0, params, imgs[:6], lb[:6], range(6))


def _vit_stem_case(gpu_lib, arch, params, imgs, lb, check, tap_layers=(), max_exempt=0):
    net = gpu_lib.build_vit(arch, params, DEV)
    xg, lbg = dev(imgs, torch.bfloat16), dev(lb[None], torch.float32)
    logits, routes = gpu_lib.ds_forward(net, xg, logit_bias=lbg)
    torch.cuda.synchronize()
    bufs = _vit_taps(gpu_lib, arch, net, xg, lbg, logits, routes, tap_layers)
    lg, rt = logits.cpu().numpy(), routes.cpu().numpy()[0]
    worst, exempt = 0.0, 0
    for b in check:
        taps = {}
        want, ro, z = O.forward_vit_stem(arch, params, imgs[b], logit_bias=lb[b], taps=taps)
        if int(rt[b]) != ro:
            # the gate reads bf16 stem features: it may only disagree inside that noise
            exempt += 1
            assert O.gate_margin(z) < 2e-2 * np.max(np.abs(z)), (b, rt[b], ro, z)
            taps = {}
            want, _, _ = O.forward_vit_stem(arch, params, imgs[b], logit_bias=lb[b], route_override=int(rt[b]), taps=taps)
        worst = max(worst, relerr(lg[b], want))
        for l in tap_layers:
            if f"l{l}" in taps:
                worst = max(worst, _check_tap(bufs[l], b, taps[f"l{l}"]))
    assert worst < TOL, worst
    assert exempt <= max_exempt, f"{exempt} checked samples needed the bf16-gate exemption"
    return net, xg, lbg, logits, routes


@pytest.mark.parametrize("stem_dim,routes", [(24, "diag"), (8, "depth")])
def test_vit_stem_small_all_samples(gpu_lib, stem_dim, routes):
    # 64x64 images -> 32x32 stem map -> 4x4 patches of 8x8 (+ class token): 17 tokens, DeiT-S widths
    arch = WL.vit_arch(image=64, patch=8, depth=2, routes=routes, stem_dim=stem_dim)
    assert arch["tokens"] == 17
    params = WL.vit_params(arch, S + 70)
    B = 29
    imgs = WL.images(S + 71, B, 64)
    lb = WL.seeded_logit_bias(S + 72, B, arch["T"], amp=16.0)
    net, xg, lbg, logits, rt = _vit_stem_case(gpu_lib, arch, params, imgs, lb, range(B))
    assert len(set(rt.cpu().numpy()[0].tolist())) == arch["T"]
    # forced routes reproduce the free-running logits; the gate also runs without any bias
    l2, _ = gpu_lib.ds_forward(net, xg, route_override=rt.clone())
    assert torch.equal(l2, logits)
    l3, r3 = gpu_lib.ds_forward(net, xg)
    want, ro, z = O.forward_vit_stem(arch, params, imgs[2])
    if int(r3[0, 2]) == ro:
        assert relerr(l3[2].cpu().numpy(), want) < TOL
    else:
        assert O.gate_margin(z) < 2e-2 * np.max(np.abs(z))


def test_vit_stem_batch256(gpu_lib):
    # the paper's stem at its real shape: 224x224 -> 112x112x24 -> 14x14 patches of 8x8, 197 tokens
    arch = WL.vit_arch(stem_dim=24, patch=8, depth=2)
    assert arch["tokens"] == 197 and arch["T"] == 48
    params = WL.vit_params(arch, S + 75)
    B = 256
    imgs = WL.images(S + 175, B)
    lb = WL.seeded_logit_bias(S + 275, B, arch["T"], amp=16.0)
    target = np.argmax(lb, axis=1)
    check = sorted({int(np.where(target == t)[0][0]) for t in range(0, 48, 3)} | {200})      # 16 routes + one more
    net, xg, lbg, logits, routes = _vit_stem_case(gpu_lib, arch, params, imgs, lb, check, tap_layers=(0, 1))
    pi = torch.randperm(B, generator=torch.Generator().manual_seed(4)).to(DEV)
    l3, r3 = gpu_lib.ds_forward(net, xg[pi].contiguous(), logit_bias=lbg[:, pi].contiguous())
    assert torch.equal(l3, logits[pi]) and torch.equal(r3, routes[:, pi])


def test_vit_pp_small_all_samples(gpu_lib):
    # the DS-ViT++ supernet shape in small: stem, 8 stored heads of 48, embedding up to 416, MLP ratios 3 / 3.5 / 4,
    # 8 nested routes that also differ in depth (2..4 of 4 stored blocks)
    arch = WL.vit_arch(image=64, patch=8, embed=416, heads=8, head_dim=48, mlp=1664, depth=4, routes="pp", stem_dim=24)
    assert arch["tokens"] == 17 and arch["T"] == 8
    params = WL.vit_params(arch, S + 80)
    B = 27
    imgs = WL.images(S + 81, B, 64)
    lb = WL.seeded_logit_bias(S + 82, B, arch["T"], amp=16.0)
    net, xg, lbg, logits, rt = _vit_stem_case(gpu_lib, arch, params, imgs, lb, range(B))
    assert len(set(rt.cpu().numpy()[0].tolist())) == arch["T"]


def test_vit_pp_batch256(gpu_lib):
    # DS-ViT++ at the sizes of its routing-space table: 224x224 images, stem at 24 channels, 197 tokens, embedding
    # 192..416, 4..8 heads of 48, depth 12..14
    arch = WL.vit_arch(embed=416, heads=8, head_dim=48, mlp=1664, depth=14, routes="pp", stem_dim=24, patch=8)
    assert arch["tokens"] == 197
    params = WL.vit_params(arch, S + 85)
    B = 256
    imgs = WL.images(S + 185, B)
    lb = WL.seeded_logit_bias(S + 285, B, arch["T"], amp=16.0)
    target = np.argmax(lb, axis=1)
    check = [int(np.where(target == t)[0][0]) for t in range(8)]            # every path once
    net, xg, lbg, logits, routes = _vit_stem_case(gpu_lib, arch, params, imgs, lb, check, tap_layers=(5, 11, 13))
    assert np.bincount(routes.cpu().numpy()[0], minlength=8).min() >= 28


def test_vit_config5_batch256(gpu_lib):
    arch = WL.vit_arch()
    params = WL.vit_params(arch, S + 5)
    B = 256
    imgs = WL.images(S + 105, B)
    lb = WL.seeded_logit_bias(S + 205, B, arch["T"])
    target = np.argmax(lb, axis=1)
    check = sorted({int(np.where(target == t)[0][0]) for t in range(48)})   # one image of every (embed, heads, MLP) route
    assert len(check) == 48
    net, xg, lbg, logits, routes = _vit_case(gpu_lib, arch, params, imgs, lb, check, tap_layers=(0, 5, 11))
    assert np.bincount(routes.cpu().numpy()[0], minlength=48).min() >= 5
    pi = torch.randperm(B, generator=torch.Generator().manual_seed(3)).to(DEV)
    l3, r3 = gpu_lib.ds_forward(net, xg[pi].contiguous(), logit_bias=lbg[:, pi].contiguous())
    assert torch.equal(l3, logits[pi]) and torch.equal(r3, routes[:, pi])
    l4, _ = gpu_lib.ds_forward(net, xg, route_override=routes.clone())
    assert torch.equal(l4, logits)


# ------------------------------------------------------------------ degenerate batches
def test_single_sample_batches_all_networks(gpu_lib):
    # one sample: every route group but one is empty, tile lists hold a single group, buckets have one slot
    arch = WL.mbnet_arch(image=64, width_div=4)
    params = WL.mbnet_params(arch, S + 30)
    _mb_case(gpu_lib, arch, params, WL.images(S + 90, 1, 64), WL.seeded_logit_bias(S + 91, 1, arch["T"]), [0])
    arch = WL.resnet_arch(image=64, width_div=2, blocks=(2, 1, 2, 1), routes="depth")
    params = WL.resnet_params(arch, S + 40)
    _rn_case(gpu_lib, arch, params, WL.images(S + 92, 1, 64), _rn_bias(S + 93, 1, 8), [0])
    arch = WL.vit_arch(image=64, patch=16, depth=2, routes="cross")
    params = WL.vit_params(arch, S + 50)
    _vit_case(gpu_lib, arch, params, WL.images(S + 94, 1, 64), WL.seeded_logit_bias(S + 95, 1, arch["T"]), [0])
    arch = WL.vit_arch(image=64, patch=8, embed=416, heads=8, head_dim=48, mlp=1664, depth=3, routes="pp", stem_dim=24)
    params = WL.vit_params(arch, S + 80)
    _vit_stem_case(gpu_lib, arch, params, WL.images(S + 96, 1, 64), WL.seeded_logit_bias(S + 97, 1, arch["T"], amp=16.0), [0])
    # an empty batch is a no-op
    net = gpu_lib.build_vit(arch, params, DEV)
    empty = torch.zeros((0, 3, 64, 64), dtype=torch.bfloat16, device=DEV)
    logits, routes = gpu_lib.ds_forward(net, empty, logit_bias=torch.zeros((1, 0, arch["T"]), dtype=torch.float32, device=DEV))
    assert logits.shape == (0, arch["num_classes"]) and routes.shape == (1, 0)


# ------------------------------------------------------------------ the batch as concurrent parts
@pytest.mark.gpu
@pytest.mark.parametrize("kind", ["resnet", "mbnet", "vit"])
def test_forward_parts_equals_forward(gpu_lib, kind):
    """ds_forward_parts cuts the batch into shares that run on streams of the library; every output is per sample,
    so logits and routes must equal ds_forward's (the gate's pooled sums are split differently for another batch
    size, hence a rounding-level tolerance on the logits), the caller's gate-major arrays are addressed with the
    whole batch as their stride, and bytes beyond the arrays stay untouched."""
    B = 37
    if kind == "resnet":
        arch = WL.resnet_arch(image=64, width_div=2, blocks=(2, 2, 2, 2))
        params = WL.resnet_params(arch, S + 40)
        lb = _rn_bias(S + 42, B, 4)
        net = gpu_lib.build_resnet(arch, params, DEV)
    elif kind == "mbnet":
        arch = WL.mbnet_arch(image=64, width_div=4)
        params = WL.mbnet_params(arch, S + 30)
        lb = WL.seeded_logit_bias(S + 32, B, arch["T"])[None]
        net = gpu_lib.build_mbnet(arch, params, DEV)
    else:
        arch = WL.vit_arch(image=64, patch=16, depth=2, routes="diag")
        params = WL.vit_params(arch, S + 50)
        lb = WL.seeded_logit_bias(S + 52, B, arch["T"])[None]
        net = gpu_lib.build_vit(arch, params, DEV)
    imgs = WL.images(S + 41, B, 64)
    xg = torch.from_numpy(imgs).to(DEV).to(torch.bfloat16).contiguous()
    lbg = torch.from_numpy(np.ascontiguousarray(lb, dtype=np.float32)).to(DEV)
    want_l, want_r = gpu_lib.ds_forward(net, xg, logit_bias=lbg)
    torch.cuda.synchronize()
    for parts in (1, 2, 3, 4):
        logits = torch.full((B + 1, net.num_classes), float("nan"), dtype=torch.float32, device=DEV)
        routes = torch.full((net.n_gates, B), -7, dtype=torch.int32, device=DEV)
        gpu_lib.ds_forward_parts(net, xg, parts, logit_bias=lbg, logits=logits, routes=routes)
        # two calls in a row share the side streams; the second must wait for the first
        gpu_lib.ds_forward_parts(net, xg, parts, logit_bias=lbg, logits=logits, routes=routes)
        torch.cuda.synchronize()
        assert torch.equal(routes, want_r), parts
        assert torch.all(torch.isnan(logits[B]))
        assert relerr(logits[:B].cpu().numpy(), want_l.cpu().numpy()) < 1e-5, parts
    # teacher-forced routes through the parts path
    l2, r2 = gpu_lib.ds_forward_parts(net, xg, 3, route_override=want_r.clone(), logit_bias=lbg)
    assert torch.equal(r2, want_r) and relerr(l2.cpu().numpy(), want_l.cpu().numpy()) < 1e-5
    # too small a workspace is refused before anything is launched
    with pytest.raises(gpu_lib.DsError):
        gpu_lib.ds_forward_parts(net, xg, 2, logit_bias=lbg, ws=torch.empty(256, dtype=torch.uint8, device=DEV))


@pytest.mark.gpu
def test_forward_parts_from_two_host_threads(gpu_lib):
    """The side streams and fork / join events of ds_forward_parts are one set per device; calls from two host
    threads, each on a stream and workspace of its own, take turns enqueueing and both equal ds_forward."""
    import threading
    B = 29
    arch = WL.vit_arch(image=64, patch=16, depth=2, routes="diag")
    net = gpu_lib.build_vit(arch, WL.vit_params(arch, S + 50), DEV)
    xs, lbs, wants, outs, wss, streams = [], [], [], [], [], []
    for t in range(2):
        xg = torch.from_numpy(WL.images(S + 60 + t, B, 64)).to(DEV).to(torch.bfloat16).contiguous()
        lb = WL.seeded_logit_bias(S + 62 + t, B, arch["T"])[None]
        lbs.append(torch.from_numpy(np.ascontiguousarray(lb, dtype=np.float32)).to(DEV))
        xs.append(xg)
        wants.append(gpu_lib.ds_forward(net, xg, logit_bias=lbs[t]))
        outs.append((torch.empty((B, net.num_classes), dtype=torch.float32, device=DEV),
                     torch.empty((net.n_gates, B), dtype=torch.int32, device=DEV)))
        wss.append(net.workspace(B, 3))
        streams.append(torch.cuda.Stream())
    torch.cuda.synchronize()
    errors = []

    def work(t):
        try:
            with torch.cuda.stream(streams[t]):
                for _ in range(8):
                    gpu_lib.ds_forward_parts(net, xs[t], 3, logit_bias=lbs[t], logits=outs[t][0], routes=outs[t][1], ws=wss[t])
        except Exception as e:  # surfaced in the main thread below
            errors.append(e)

    threads = [threading.Thread(target=work, args=(t,)) for t in range(2)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for t in range(2):
        assert torch.equal(outs[t][1], wants[t][1]), t
        assert relerr(outs[t][0].cpu().numpy(), wants[t][0].cpu().numpy()) < 1e-5, t
