"""Pins for the oracle's network assemblies and multiply-add model.

The assemblies are checked against library routines (torch CPU, float64) applied
layer by layer to explicitly copied weight slices on test-sized networks, and the
multiply-add model against the counts the paper prints (tests/golden/paper_madds.txt).
"""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads as WL
from oracle import ds_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_madds.txt")


def t64(a):
    return torch.from_numpy(np.ascontiguousarray(np.asarray(a, np.float64)))


def _gold():
    out = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        name, val, tol = line.split()[:3]
        out[name] = (float(val), float(tol))
    return out


# ------------------------------------------------------------------ multiply-add model
def _mb_scaled(frac_num, frac_den):
    a = WL.mbnet_arch()
    sc = lambda c: c * frac_num // frac_den
    arch = dict(a, stem_out=sc(a["stem_out"]))
    cin = [sc(ci) for ci, _, _ in a["blocks"]]
    cout = [sc(co) for _, co, _ in a["blocks"]]
    return O.madds_mbnet(arch, cin, cout, cout[-1])


def _rn_scaled(frac_num, frac_den):
    a = WL.resnet_arch()
    sc = lambda c: c * frac_num // frac_den
    arch = dict(a, stem_out=sc(a["stem_out"]))
    mids = [sc(w) for w in a["widths"]]
    return O.madds_resnet(arch, mids, [4 * m for m in mids])


def test_madds_model_reproduces_paper_counts():
    g = _gold()
    got = {
        "mobilenetv1_1.0x": _mb_scaled(1, 1), "mobilenetv1_0.75x": _mb_scaled(3, 4),
        "mobilenetv1_0.5x": _mb_scaled(1, 2),
        "resnet50_1.0x": _rn_scaled(1, 1), "resnet50_0.75x": _rn_scaled(3, 4), "resnet50_0.5x": _rn_scaled(1, 2),
    }
    v = WL.vit_arch()
    got["deit_s"] = O.madds_vit(v, 384, 6, 1536)
    for k, val in got.items():
        want, tol = g[k]
        assert abs(val - want) / want <= tol, (k, val, want)


def test_madds_route_tables_are_nested_and_largest_route_is_the_full_net():
    a = WL.mbnet_arch()
    m = [O.madds_mbnet(a, a["cin"][t], a["cout"][t], int(a["cout"][t, -1])) for t in range(a["T"])]
    assert all(m[i] < m[i + 1] for i in range(len(m) - 1))      # routes ordered by complexity
    assert m[-1] == _mb_scaled(1, 1)
    assert a["cout"][:, 6].tolist() == [176, 208, 232, 256, 280, 304, 336, 360, 384, 408, 432, 464, 488, 512]
    assert a["cout"][:, 12].tolist() == [360, 408, 464, 512, 560, 616, 664, 720, 768, 816, 872, 920, 976, 1024]
    r = WL.resnet_arch()
    assert O.madds_resnet(r, r["mid"][:, 3], r["out"][:, 3]) == _rn_scaled(1, 1)
    v = WL.vit_arch()
    assert v["T"] == 48 and tuple(v["routes"][-1]) == (384, 6, 1536) and tuple(v["routes"][0]) == (192, 3, 384)


# ------------------------------------------------------------------ library-built references
def _bn(x, bn, t, c, eps):
    return F.batch_norm(x, t64(bn["mean"][t, :c]), t64(bn["var"][t, :c]), t64(bn["gamma"][:c]),
                        t64(bn["beta"][:c]), False, 0.0, eps)


def _ref_mbnet(arch, p, img, t):
    eps = arch["bn_eps"]
    x = t64(img)[None]
    x = F.relu(_bn(F.conv2d(x, t64(p["stem.w"]), stride=2, padding=1), p["stem.bn"], 0, arch["stem_out"], eps))
    for i, (_a, _b, s) in enumerate(arch["blocks"]):
        tb = t if i >= arch["gate_after"] else 0
        ci, co = int(arch["cin"][t, i]), int(arch["cout"][t, i])
        wd = p[f"ds{i}.dw.w"][:ci]
        k = int(arch["ksize"][t, i]) if "ksize" in arch else 3
        k0 = (wd.shape[-1] - k) // 2
        wd = wd[:, :, k0:k0 + k, k0:k0 + k].copy()              # the route's centred block of the stored filter
        x = F.relu(_bn(F.conv2d(x, t64(wd), stride=s, padding=(k - 1) // 2, groups=ci),
                       p[f"ds{i}.dw.bn"], tb, ci, eps))
        x = F.relu(_bn(F.conv2d(x, t64(p[f"ds{i}.pw.w"][:co, :ci])), p[f"ds{i}.pw.bn"], tb, co, eps))
    c = x.shape[1]
    return F.linear(x.mean((2, 3)), t64(p["fc.w"][:, :c]), t64(p["fc.b"]))[0].numpy()


def _ref_resnet(arch, p, img, routes):
    eps = arch["bn_eps"]
    x = t64(img)[None]
    x = F.relu(_bn(F.conv2d(x, t64(p["stem.w"]), stride=2, padding=3), p["stem.bn"], 0, arch["stem_out"], eps))
    x = F.max_pool2d(x, 3, 2, 1)
    for s, nb in enumerate(arch["blocks"]):
        t = routes[s]
        mid, out = int(arch["mid"][s, t]), int(arch["out"][s, t])
        for b in range(nb):
            bp = f"s{s}.b{b}"
            st = 2 if (b == 0 and s > 0) else 1
            ci = x.shape[1]
            sc = x
            if b == 0:
                sc = _bn(F.conv2d(x, t64(p[bp + ".proj.w"][:out, :ci]), stride=st), p[bp + ".proj.bn"], t, out, eps)
            y = F.relu(_bn(F.conv2d(x, t64(p[bp + ".c1.w"][:mid, :ci])), p[bp + ".c1.bn"], t, mid, eps))
            y = F.relu(_bn(F.conv2d(y, t64(p[bp + ".c2.w"][:mid, :mid]), stride=st, padding=1), p[bp + ".c2.bn"], t, mid, eps))
            y = _bn(F.conv2d(y, t64(p[bp + ".c3.w"][:out, :mid])), p[bp + ".c3.bn"], t, out, eps)
            x = F.relu(y + sc)
    c = x.shape[1]
    return F.linear(x.mean((2, 3)), t64(p["fc.w"][:, :c]), t64(p["fc.b"]))[0].numpy()


def _ref_vit(arch, p, img, route):
    d, h, hid = (int(v) for v in arch["routes"][route])
    dh, eps = arch["head_dim"], arch["ln_eps"]
    hd = h * dh
    tok = F.conv2d(t64(img)[None], t64(p["embed.w"][:d]), t64(p["embed.b"][:d]), stride=arch["patch"])
    tok = tok.flatten(2).transpose(1, 2)[0] + t64(p["pos"][1:, :d])
    x = torch.cat([(t64(p["cls"][:d]) + t64(p["pos"][0, :d]))[None], tok], 0)
    N = x.shape[0]
    for l in range(arch["depth"]):
        q_ = f"l{l}"
        a = F.layer_norm(x, (d,), t64(p[q_ + ".ln1.g"][:d]), t64(p[q_ + ".ln1.b"][:d]), eps)
        q, k, v = (F.linear(a, t64(p[q_ + f".w{n}"][:hd, :d]), t64(p[q_ + f".b{n}"][:hd])) for n in "qkv")
        sp = lambda z: z.reshape(N, h, dh).transpose(0, 1)
        o = F.scaled_dot_product_attention(sp(q), sp(k), sp(v)).transpose(0, 1).reshape(N, hd)
        x = x + F.linear(o, t64(p[q_ + ".wproj"][:d, :hd]), t64(p[q_ + ".bproj"][:d]))
        m = F.layer_norm(x, (d,), t64(p[q_ + ".ln2.g"][:d]), t64(p[q_ + ".ln2.b"][:d]), eps)
        m = F.gelu(F.linear(m, t64(p[q_ + ".fc1.w"][:hid, :d]), t64(p[q_ + ".fc1.b"][:hid])))
        x = x + F.linear(m, t64(p[q_ + ".fc2.w"][:d, :hid]), t64(p[q_ + ".fc2.b"][:d]))
    f = F.layer_norm(x[:1], (d,), t64(p["ln.g"][:d]), t64(p["ln.b"][:d]), eps)
    return F.linear(f[0], t64(p["head.w"][:, :d]), t64(p["head.b"])).numpy()


# ------------------------------------------------------------------ assemblies
@pytest.mark.parametrize("t", [0, 6, 13])
def test_mbnet_assembly_matches_library_layers(t):
    arch = WL.mbnet_arch(image=32, width_div=8)
    p = WL.mbnet_params(arch, 11)
    img = WL.images(12, 1, 32)[0]
    got, rt, _ = O.forward_mbnet(arch, p, img, route_override=t, store="f64")
    assert rt == t
    np.testing.assert_allclose(got, _ref_mbnet(arch, p, img, t), rtol=1e-9, atol=1e-9)


@pytest.mark.parametrize("t", [0, 5, 11])
def test_mbnet_pp_assembly_matches_library_layers(t):
    arch = WL.mbnet_pp_arch(image=32, width_div=2)
    assert arch["T"] == 12 and sorted(set(arch["ksize"][:, 7].tolist())) == [3, 5, 7] and set(arch["ksize"][:, 2].tolist()) == {5}
    p = WL.mbnet_params(arch, 13)
    assert p["ds1.dw.w"].shape[-1] == 5 and p["ds7.dw.w"].shape[-1] == 7
    img = WL.images(14, 1, 32)[0]
    got, rt, _ = O.forward_mbnet(arch, p, img, route_override=t, store="f64")
    assert rt == t
    np.testing.assert_allclose(got, _ref_mbnet(arch, p, img, t), rtol=1e-9, atol=1e-9)


def test_mbnet_pp_channel_lists_are_the_papers():
    # lower half of the DS-MBNet routing-space table: [288:640:32] and [800:1152:32], 12 paths (Section 5.2)
    a = WL.mbnet_pp_arch()
    assert a["cout"][:, 5].tolist() == list(range(288, 641, 32)) and a["cout"][:, 12].tolist() == list(range(800, 1153, 32))
    assert a["T"] == 12 and [b[1] for b in a["blocks"][:5]] == [32, 48, 48, 96, 96] and a["stem_out"] == 16


def test_mbnet_gate_picks_the_biased_route_and_bf16_storage_stays_close():
    arch = WL.mbnet_arch(image=32, width_div=8)
    p = WL.mbnet_params(arch, 11)
    img = WL.images(12, 2, 32)
    lb = WL.seeded_logit_bias(5, 2, arch["T"])
    for b in range(2):
        lo, t, z = O.forward_mbnet(arch, p, img[b], logit_bias=lb[b], store="bf16")
        assert t == int(np.argmax(z)) and z.shape == (arch["T"],)
        hi, t2, _ = O.forward_mbnet(arch, p, img[b], route_override=t, store="f64")
        assert np.max(np.abs(lo - hi)) / np.max(np.abs(hi)) < 2e-2
    taps = {}
    O.forward_mbnet(arch, p, img[0], route_override=3, store="bf16", taps=taps)
    for v in taps.values():
        assert np.array_equal(O.bf16_round(v), v)              # stored tensors are bf16 values


@pytest.mark.parametrize("routes", [(0, 0, 0, 0), (3, 3, 3, 3), (1, 3, 0, 2)])
def test_resnet_assembly_matches_library_layers(routes):
    arch = WL.resnet_arch(image=32, width_div=8, blocks=(2, 1, 2, 1))
    p = WL.resnet_params(arch, 21)
    img = WL.images(22, 1, 32)[0]
    got, rt, _ = O.forward_resnet(arch, p, img, route_override=routes, store="f64")
    assert tuple(rt) == routes
    np.testing.assert_allclose(got, _ref_resnet(arch, p, img, routes), rtol=1e-9, atol=1e-9)


def test_resnet_free_running_gates_follow_logit_bias():
    arch = WL.resnet_arch(image=32, width_div=8, blocks=(1, 1, 1, 1))
    p = WL.resnet_params(arch, 21)
    img = WL.images(22, 1, 32)[0]
    lb = np.stack([WL.seeded_logit_bias(30 + s, 1, 4)[0] for s in range(4)])
    _, rt, zs = O.forward_resnet(arch, p, img, logit_bias=lb, store="bf16")
    assert rt == [int(np.argmax(z)) for z in zs]


@pytest.mark.parametrize("route", [0, 17, 47])
def test_vit_assembly_matches_library_layers(route):
    arch = WL.vit_arch(image=32, patch=8, embed=48, heads=6, head_dim=8, mlp=192, depth=2)
    p = WL.vit_params(arch, 31)
    img = WL.images(32, 1, 32)[0]
    got = O.forward_vit(arch, p, img, route, store="f64")
    np.testing.assert_allclose(got, _ref_vit(arch, p, img, route), rtol=1e-9, atol=1e-10)


def test_vit_bf16_storage_stays_close():
    arch = WL.vit_arch(image=32, patch=8, embed=48, heads=6, head_dim=8, mlp=192, depth=2, routes="diag")
    p = WL.vit_params(arch, 31)
    img = WL.images(32, 1, 32)[0]
    for route in range(4):
        lo = O.forward_vit(arch, p, img, route, store="bf16")
        hi = O.forward_vit(arch, p, img, route, store="f64")
        assert np.max(np.abs(lo - hi)) / np.max(np.abs(hi)) < 2e-2


def test_seeded_logit_bias_makes_every_route_occur():
    for B, T in [(256, 14), (256, 48), (64, 4)]:
        lb = WL.seeded_logit_bias(7, B, T)
        r = np.argmax(lb, axis=1)
        cnt = np.bincount(r, minlength=T)
        assert cnt.min() >= B // T and cnt.max() <= B // T + 1


def test_vit_route_depth_equals_truncated_network():
    # a route of depth L must give what the same network cut down to its first L blocks gives, and a
    # route whose depth is the stored depth must equal the plain three-entry route (the skipped
    # blocks are identities because of the residual connections)
    arch = WL.vit_arch(image=32, patch=8, embed=48, heads=6, head_dim=8, mlp=192, depth=4, routes="depth")
    p = WL.vit_params(arch, 31)
    img = WL.images(32, 1, 32)[0]
    plain = WL.vit_arch(image=32, patch=8, embed=48, heads=6, head_dim=8, mlp=192, depth=4, routes="diag")
    assert arch["T"] == 12 and arch["routes"].shape == (12, 4)
    for t in range(arch["T"]):
        d_e, h, hidden, blocks = (int(v) for v in arch["routes"][t])
        assert 2 <= blocks <= 4
        cut = dict(plain, depth=blocks)
        want = O.forward_vit(cut, p, img, t // 3, store="f64")
        got = O.forward_vit(arch, p, img, t, store="f64")
        np.testing.assert_array_equal(got, want)
    # deeper routes differ from shallower ones (the extra blocks do something)
    a = O.forward_vit(arch, p, img, 0, store="f64")
    b = O.forward_vit(arch, p, img, 2, store="f64")
    assert np.max(np.abs(a - b)) > 1e-6


def test_resnet_route_depth_equals_truncated_network():
    # a stage whose route runs n blocks must give what a network storing only n blocks in that stage
    # gives with the same weights and the same per-route BN rows (the skipped blocks are identities
    # through their residuals)
    blocks = (2, 3, 2, 2)
    arch = WL.resnet_arch(image=32, width_div=8, blocks=blocks, routes="depth")
    plain = {k: v for k, v in arch.items() if k != "nblk"}
    assert arch["T"] == 8 and arch["nblk"].shape == (4, 8) and arch["nblk"].min() == 1
    p = WL.resnet_params(arch, 23)
    img = WL.images(32, 1, 32)[0]
    rng = np.random.default_rng(5)
    cases = [[0, 0, 0, 0], [7, 7, 7, 7], [1, 2, 4, 6]] + [list(rng.integers(0, 8, 4)) for _ in range(3)]
    for rt in cases:
        got, r_got, _ = O.forward_resnet(arch, p, img, route_override=rt, store="f64")
        cut = dict(plain, blocks=[int(arch["nblk"][s][rt[s]]) for s in range(4)])
        want, _, _ = O.forward_resnet(cut, p, img, route_override=rt, store="f64")
        assert list(r_got) == [int(t) for t in rt]
        np.testing.assert_array_equal(got, want)
    # the shallow and the deep route of one ratio differ (the extra block does something)
    a, _, _ = O.forward_resnet(arch, p, img, route_override=[6, 6, 6, 6], store="f64")
    b, _, _ = O.forward_resnet(arch, p, img, route_override=[7, 7, 7, 7], store="f64")
    assert np.max(np.abs(a - b)) > 1e-6


# ------------------------------------------------------------------ DS-ViT++ stem (Section 3.4)
def test_patch_stem_madds_reproduce_the_papers_stem_table():
    # Section 3.4's table of patch-embedding designs: the 4-convolution stem at width 64 costs 1.3 G
    # more than a plain 16x16 patch projection (6.8 G vs 5.5 G), the [c, ds, ds, c] stem at width 24
    # only 0.1 G more (5.6 G vs 5.5 G); embedding width 384 as in the small ViT variants
    plain = O.madds_patch_stem(224, 384, 0, ["c"], [16], [16])
    lv = O.madds_patch_stem(224, 384, 64, ["c", "c", "c", "c"], [7, 3, 3, 8], [2, 1, 1, 8])
    ours = O.madds_patch_stem(224, 384, 24, ["c", "ds", "ds", "c"], [7, 3, 3, 8], [2, 1, 1, 8])
    assert plain == 196 * 768 * 384
    assert abs((lv - plain) - 1.3e9) < 0.05e9
    assert abs((ours - plain) - 0.1e9) < 0.05e9
    assert round(lv / 1e9, 1) in (1.3, 1.4)           # the text quotes the stem alone at 1.3 G


def _ref_vit_stem(arch, p, img, t):
    eps, C = arch["bn_eps"], arch["stem_dim"]
    x = t64(img)[None]
    x = F.relu(_bn(F.conv2d(x, t64(p["stem.c0.w"]), stride=2, padding=3), p["stem.c0.bn"], 0, C, eps))
    for i in (1, 2):
        x = F.relu(_bn(F.conv2d(x, t64(p[f"stem.ds{i}.dw.w"]), padding=1, groups=C), p[f"stem.ds{i}.dw.bn"], 0, C, eps))
        x = F.relu(_bn(F.conv2d(x, t64(p[f"stem.ds{i}.pw.w"])), p[f"stem.ds{i}.pw.bn"], 0, C, eps))
    pooled = x.mean((2, 3))[0]
    hid = F.relu(F.linear(pooled, t64(p["gate.w1"]), t64(p["gate.b1"])))
    z = F.linear(hid, t64(p["gate.w2"]), t64(p["gate.b2"])).numpy()
    # the rest is the plain network fed with the stem's feature map instead of the image
    q = dict(p)
    plain = {k: v for k, v in arch.items() if k != "stem_dim"}
    return _ref_vit(plain, q, x[0].numpy(), t), z


@pytest.mark.parametrize("t", [0, 5, 11])
def test_vit_stem_assembly_matches_library_layers(t):
    arch = WL.vit_arch(image=32, patch=4, embed=48, heads=6, head_dim=8, mlp=192, depth=2, routes="depth",
                       stem_dim=8)
    assert arch["tokens"] == 17
    # drop the depth entry for the library reference (it runs every block): compare on full-depth routes
    arch3 = dict(arch, routes=arch["routes"][:, :3].copy())
    p = WL.vit_params(arch3, 77)
    img = WL.images(78, 1, 32)[0]
    got, rt, z = O.forward_vit_stem(arch3, p, img, route_override=t, store="f64")
    want, z_ref = _ref_vit_stem(arch3, p, img, t)
    assert rt == t
    np.testing.assert_allclose(z, z_ref, rtol=1e-9, atol=1e-9)
    np.testing.assert_allclose(got, want, rtol=1e-9, atol=1e-9)


def test_vit_stem_patch_projection_is_a_linear_layer_on_patches_and_gate_follows_bias():
    arch = WL.vit_arch(image=32, patch=4, embed=48, heads=6, head_dim=8, mlp=192, depth=1, routes="diag",
                       stem_dim=8)
    p = WL.vit_params(arch, 79)
    rng = np.random.default_rng(3)
    x = rng.standard_normal((8, 16, 16))
    for d_e in (24, 48):
        conv = O.sliced_conv2d(x, p["embed.w"], d_e, 4, 0).reshape(d_e, -1).T
        lin = O.sliced_linear(O.patchify(x, 4), np.asarray(p["embed.w"], np.float64).reshape(48, -1), None, d_e)
        np.testing.assert_allclose(conv, lin, rtol=1e-12, atol=1e-12)
    img = WL.images(80, 3, 32)
    lb = WL.seeded_logit_bias(6, 3, arch["T"], amp=16.0)
    for b in range(3):
        lo, t, z = O.forward_vit_stem(arch, p, img[b], logit_bias=lb[b], store="bf16")
        assert t == int(np.argmax(z)) == int(np.argmax(lb[b])) and z.shape == (arch["T"],)
        hi, _, _ = O.forward_vit_stem(arch, p, img[b], route_override=t, store="f64")
        assert np.max(np.abs(lo - hi)) / np.max(np.abs(hi)) < 2e-2


def test_resnet_pp_single_gate_steers_every_stage():
    # DS-ResNet++: the first block's gate decides width and depth of all four stages (Section 5.2); the table's ranges
    blocks = (3, 4, 8, 3)
    full = WL.resnet_arch(blocks=blocks, routes="pp")
    assert full["T"] == 9 and full["single_gate"]
    assert full["out"][0].tolist() == [128, 128, 160, 160, 192, 192, 224, 224, 256]
    assert (full["out"][1][0], full["out"][1][-1], full["out"][2][0], full["out"][2][-1]) == (256, 512, 512, 1024)
    assert (full["out"][3][0], full["out"][3][-1]) == (1024, 2048)
    assert [(int(r.min()), int(r.max())) for r in full["nblk"]] == [(2, 3), (2, 4), (5, 8), (2, 3)]
    arch = WL.resnet_arch(image=32, width_div=8, blocks=blocks, routes="pp")
    p = WL.resnet_params(arch, 29)
    img = WL.images(33, 1, 32)[0]
    multi = {k: v for k, v in arch.items() if k != "single_gate"}
    for t in (0, 4, 8):
        lb = np.zeros((4, 9), np.float32)
        lb[0, t] = 50.0                                    # stage-1 gate picks t
        lb[1:, (t + 3) % 9] = 50.0                         # the other gates would pick something else
        got, rt, zs = O.forward_resnet(arch, p, img, logit_bias=lb, store="f64")
        assert rt == [t, t, t, t] and len(zs) == 4
        want, _, _ = O.forward_resnet(multi, p, img, route_override=[t, t, t, t], store="f64")
        np.testing.assert_array_equal(got, want)
        # and against library layers on a network cut to the route's block counts
        cut = {k: v for k, v in multi.items() if k != "nblk"}
        cut["blocks"] = [int(arch["nblk"][s][t]) for s in range(4)]
        np.testing.assert_allclose(got, _ref_resnet(cut, p, img, [t, t, t, t]), rtol=1e-9, atol=1e-9)
