"""Network descriptions (layer lists, route tables) and seeded random parameters.

Everything here is data: shapes, integer slice tables and random tensors drawn
from a seeded CPU generator in a fixed order.  Values meant for bf16 storage are
rounded once to bf16 (round-to-nearest-even) and handed out as float32 arrays
holding exactly those bf16 values, so every consumer starts from the same bits.

Shapes follow the routing spaces of the paper's Section 5.2 ("Architecture
details") and its routing-space tables, restricted to channel / embedding /
head / MLP slicing.
"""
from __future__ import annotations

import numpy as np
import torch

BASE_SEED = 210910060


# --------------------------------------------------------------------------
# random helpers (no arithmetic of the method)
# --------------------------------------------------------------------------
class Draw:
    """Sequential draws from one seeded CPU generator."""

    def __init__(self, seed: int):
        self.g = torch.Generator(device="cpu")
        self.g.manual_seed(int(seed))

    def normal(self, shape, std=1.0, mean=0.0) -> np.ndarray:
        t = torch.empty(tuple(shape), dtype=torch.float32)
        t.normal_(mean=float(mean), std=float(std), generator=self.g)
        return t.numpy()

    def uniform(self, shape, lo, hi) -> np.ndarray:
        t = torch.empty(tuple(shape), dtype=torch.float32)
        t.uniform_(float(lo), float(hi), generator=self.g)
        return t.numpy()

    def randint(self, n, high) -> np.ndarray:
        return torch.randint(0, int(high), (int(n),), generator=self.g).numpy().astype(np.int32)

    def permutation(self, n) -> np.ndarray:
        return torch.randperm(int(n), generator=self.g).numpy().astype(np.int64)


def as_bf16_values(a: np.ndarray) -> np.ndarray:
    """Round a float32 array once to bf16 (RNE); return float32 holding those values."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(torch.bfloat16).to(torch.float32).numpy()


def bn_tables(d: Draw, T: int, C: int) -> dict:
    """Affine parameters shared by all routes plus per-route running statistics."""
    return {
        "gamma": d.uniform((C,), 0.5, 1.5),
        "beta": d.normal((C,), std=0.1),
        "mean": d.normal((T, C), std=0.1),
        "var": d.uniform((T, C), 0.5, 1.5),
    }


def seeded_logit_bias(seed: int, B: int, T: int, amp: float = 4.0, favour: int = -1, share: float = 0.5) -> np.ndarray:
    """Per-sample additive gate logits: small noise plus `amp` on a seeded target route,
    so that every route occurs about B/T times and margins are far above rounding noise.
    With favour >= 0 the first `share` of a seeded order of the samples targets route `favour`
    instead (a skewed mix: about share + (1 - share)/T of the batch on one route)."""
    d = Draw(seed)
    noise = d.normal((B, T), std=0.1)
    pi = d.permutation(B)
    target = (pi % T).astype(np.int64)
    if favour >= 0:
        target[pi < int(round(share * B))] = favour
    bias = noise.copy()
    bias[np.arange(B), target] += float(amp)
    return bias.astype(np.float32)


def images(seed: int, B: int, size: int = 224, bf16: bool = True) -> np.ndarray:
    """Synthetic ImageNet-shaped batch, N(0,1) pixels, NCHW."""
    d = Draw(seed)
    x = d.normal((B, 3, size, size))
    return as_bf16_values(x) if bf16 else x


def _kaiming(d: Draw, shape) -> np.ndarray:
    fan_in = int(np.prod(shape[1:]))
    return d.normal(shape, std=(2.0 / fan_in) ** 0.5)


# --------------------------------------------------------------------------
# DS-MBNet: MobileNetV1 with one gate after the 5th depthwise-separable block
# --------------------------------------------------------------------------
def _round8(C: int, i: int) -> int:
    # nearest multiple of 8 to C*(0.35+0.05 i), ties up, integer only
    return 8 * ((C * (35 + 5 * i) + 400) // 800)


def mbnet_arch(image: int = 224, width_div: int = 1) -> dict:
    """Layer list of the MobileNetV1-shaped dynamic net.

    `width_div` shrinks every stored channel count (test-sized nets); 1 gives
    the standard 32..1024 channels.  cin/cout are [T, 13] integer tables: the
    valid channels of block i on route t.  Blocks 1-5 are fixed; blocks 6-13 and
    the classifier's input width follow the route.
    """
    base = [(32, 64, 1), (64, 128, 2), (128, 128, 1), (128, 256, 2), (256, 256, 1),
            (256, 512, 2), (512, 512, 1), (512, 512, 1), (512, 512, 1), (512, 512, 1),
            (512, 512, 1), (512, 1024, 2), (1024, 1024, 1)]
    blocks = [(ci // width_div, co // width_div, s) for ci, co, s in base]
    T = 14
    cin = np.zeros((T, 13), np.int32)
    cout = np.zeros((T, 13), np.int32)
    for t in range(T):
        for i, (ci, co, _s) in enumerate(blocks):
            cin[t, i] = ci if i < 6 else _round8(ci, t)
            cout[t, i] = co if i < 5 else _round8(co, t)
    return {
        "name": "mbnet", "image": image, "stem_out": 32 // width_div, "blocks": blocks,
        "gate_after": 5, "gate_hidden": blocks[4][1] // 4, "T": T,
        "cin": cin, "cout": cout, "num_classes": 1000, "bn_eps": 1e-5,
    }


def mbnet_pp_arch(image: int = 224, width_div: int = 1) -> dict:
    """DS-MBNet++ (lower half of the DS-MBNet routing-space table): stem 16, depthwise-separable blocks
    32 / 48, 48 / 96, 96 with 5x5 depthwise filters (fixed), then six blocks at [288:640:32] and two at
    [800:1152:32] channels whose depthwise filters are stored 7x7 and used at kernel size 3, 5 or 7.
    12 routes: route t has the t-th entry of both channel lists and kernel size 3 (t < 4), 5 (t < 8) or 7;
    padding is (k - 1) / 2 throughout, so every route keeps the resolution.  ksize is [T, 13], kfull [13]."""
    d = width_div
    c1max, c2max = 640 // d, 1152 // d
    blocks = [(16 // d, 32 // d, 1), (32 // d, 48 // d, 2), (48 // d, 48 // d, 1), (48 // d, 96 // d, 2),
              (96 // d, 96 // d, 1), (96 // d, c1max, 2)] + [(c1max, c1max, 1)] * 5 + [(c1max, c2max, 2), (c2max, c2max, 1)]
    T = 12
    cin = np.zeros((T, 13), np.int32)
    cout = np.zeros((T, 13), np.int32)
    ksize = np.zeros((T, 13), np.int32)
    kfull = [5] * 5 + [7] * 8
    for t in range(T):
        c1, c2 = (288 + 32 * t) // d, (800 + 32 * t) // d
        for i, (ci, co, _s) in enumerate(blocks):
            cin[t, i] = ci if i < 6 else (c1 if i < 12 else c2)
            cout[t, i] = co if i < 5 else (c1 if i < 11 else c2)
            ksize[t, i] = 5 if i < 5 else (3, 5, 7)[t // 4]
    return {
        "name": "mbnet", "image": image, "stem_out": 16 // d, "blocks": blocks,
        "gate_after": 5, "gate_hidden": blocks[4][1] // 4, "T": T,
        "cin": cin, "cout": cout, "kfull": kfull, "ksize": ksize, "num_classes": 1000, "bn_eps": 1e-5,
    }


def mbnet_params(arch: dict, seed: int) -> dict:
    d = Draw(seed)
    T = arch["T"]
    p = {}
    so = arch["stem_out"]
    p["stem.w"] = as_bf16_values(_kaiming(d, (so, 3, 3, 3)))
    p["stem.bn"] = bn_tables(d, 1, so)
    for i, (ci, co, _s) in enumerate(arch["blocks"]):
        Tb = 1 if i < arch["gate_after"] else T
        kf = arch["kfull"][i] if "kfull" in arch else 3
        p[f"ds{i}.dw.w"] = as_bf16_values(_kaiming(d, (ci, 1, kf, kf)))
        p[f"ds{i}.dw.bn"] = bn_tables(d, Tb, ci)
        p[f"ds{i}.pw.w"] = as_bf16_values(_kaiming(d, (co, ci, 1, 1)))
        p[f"ds{i}.pw.bn"] = bn_tables(d, Tb, co)
    cg = arch["blocks"][arch["gate_after"] - 1][1]
    hid = arch["gate_hidden"]
    p["gate.w1"] = d.normal((hid, cg), std=cg ** -0.5)
    p["gate.b1"] = d.normal((hid,), std=0.1)
    p["gate.w2"] = d.normal((T, hid), std=hid ** -0.5)
    p["gate.b2"] = d.normal((T,), std=0.1)
    cf = arch["blocks"][-1][1]
    p["fc.w"] = as_bf16_values(d.normal((arch["num_classes"], cf), std=cf ** -0.5))
    p["fc.b"] = d.normal((arch["num_classes"],), std=0.1)
    return p


# --------------------------------------------------------------------------
# DS-ResNet: ResNet-50 with a gate in the first block of each stage
# --------------------------------------------------------------------------
def resnet_arch(image: int = 224, width_div: int = 1, blocks=(3, 4, 6, 3), routes: str = "width") -> dict:
    """Bottleneck stages with mid width w*q/4 and output width 4w*q/4, q=1..4.

    mid[s][t], out[s][t] are the valid channel counts of stage s on route t.  The 7x7 stem and
    the max-pool are never sliced.  routes="width": 4 routes, one per ratio; "pp": the 9 paths of
    DS-ResNet++ under a single gate; "depth": 8 routes,
    route t has ratio index t // 2 and runs nblk[s][t] = blocks[s] - 1 + t % 2 (at least 1)
    blocks of stage s.
    """
    widths = [64 // width_div, 128 // width_div, 256 // width_div, 512 // width_div]
    mid = np.array([[w * q // 4 for q in (1, 2, 3, 4)] for w in widths], np.int32)
    extra = {}
    if routes == "pp":
        # DS-ResNet++ (lower half of the DS-ResNet routing-space table): one gate in the first block steers the
        # width and the number of blocks of all four stages; 9 nested paths along stage outputs [128:256:32],
        # [256:512:32], [512:1024:64], [1024:2048:128] and block counts [2:3], [2:4], [5:8], [2:3]
        # (use blocks=(3, 4, 8, 3)).  Stage 1 has five widths for nine paths: two paths share each.
        d = width_div
        outs = [[(128 + 32 * (i // 2)) // d for i in range(9)], [(256 + 32 * i) // d for i in range(9)],
                [(512 + 64 * i) // d for i in range(9)], [(1024 + 128 * i) // d for i in range(9)]]
        mid = np.array(outs, np.int32) // 4
        nb = list(blocks)
        extra["nblk"] = np.array([[nb[0] - 1 + (i >= 5) for i in range(9)], [nb[1] - 2 + i // 3 for i in range(9)],
                                  [nb[2] - 3 + i // 3 + (i == 8) for i in range(9)], [nb[3] - 1 + (i >= 5) for i in range(9)]],
                                 np.int32).clip(1, None)
        extra["single_gate"] = True
    elif routes == "depth":
        mid = np.repeat(mid, 2, axis=1)
        extra["nblk"] = np.array([[max(1, nb - 1 + t % 2) for t in range(8)] for nb in blocks], np.int32)
    else:
        assert routes == "width"
    out = 4 * mid
    return {
        **extra,
        "name": "resnet", "image": image, "stem_out": 64 // width_div, "widths": widths,
        "blocks": list(blocks), "T": mid.shape[1], "mid": mid, "out": out.astype(np.int32),
        "gate_hidden": [max(1, (64 // width_div) // 4)] + [max(1, 4 * w // 4) for w in widths[:-1]],
        "num_classes": 1000, "bn_eps": 1e-5,
    }


def resnet_params(arch: dict, seed: int) -> dict:
    d = Draw(seed)
    T = arch["T"]
    p = {}
    so = arch["stem_out"]
    p["stem.w"] = as_bf16_values(_kaiming(d, (so, 3, 7, 7)))
    p["stem.bn"] = bn_tables(d, 1, so)
    cprev = so
    for s, (w, nb) in enumerate(zip(arch["widths"], arch["blocks"])):
        hid = arch["gate_hidden"][s]
        p[f"s{s}.gate.w1"] = d.normal((hid, cprev), std=cprev ** -0.5)
        p[f"s{s}.gate.b1"] = d.normal((hid,), std=0.1)
        p[f"s{s}.gate.w2"] = d.normal((T, hid), std=hid ** -0.5)
        p[f"s{s}.gate.b2"] = d.normal((T,), std=0.1)
        for b in range(nb):
            cin = cprev if b == 0 else 4 * w
            pre = f"s{s}.b{b}"
            p[pre + ".c1.w"] = as_bf16_values(_kaiming(d, (w, cin, 1, 1)))
            p[pre + ".c1.bn"] = bn_tables(d, T, w)
            p[pre + ".c2.w"] = as_bf16_values(_kaiming(d, (w, w, 3, 3)))
            p[pre + ".c2.bn"] = bn_tables(d, T, w)
            p[pre + ".c3.w"] = as_bf16_values(_kaiming(d, (4 * w, w, 1, 1)))
            p[pre + ".c3.bn"] = bn_tables(d, T, 4 * w)
            # small gain on the last batch-norm of the residual branch (the training recipe starts
            # it at zero): keeps the random-init net's activations from doubling at every block
            p[pre + ".c3.bn"]["gamma"] = (0.25 * p[pre + ".c3.bn"]["gamma"]).astype(np.float32)
            if b == 0:
                p[pre + ".proj.w"] = as_bf16_values(_kaiming(d, (4 * w, cin, 1, 1)))
                p[pre + ".proj.bn"] = bn_tables(d, T, 4 * w)
        cprev = 4 * w
    p["fc.w"] = as_bf16_values(d.normal((arch["num_classes"], cprev), std=cprev ** -0.5))
    p["fc.b"] = d.normal((arch["num_classes"],), std=0.1)
    return p


# --------------------------------------------------------------------------
# DS-ViT: DeiT-S-shaped transformer, one route per image chosen before the patch embed
# --------------------------------------------------------------------------
def vit_arch(image: int = 224, patch: int = 16, embed: int = 384, heads: int = 6,
             head_dim: int = 64, mlp: int = 1536, depth: int = 12, routes: str = "cross",
             stem_dim: int = 0) -> dict:
    """routes[t] = (d_e, h, hidden): embedding slice, head count and MLP hidden slice.

    "cross": every combination of 4 embedding slices, 4 head counts and MLP
    ratios 2,3,4 (hidden = ratio * d_e); "diag": 4 nested routes; "pp": 8 nested routes of the
    DS-ViT++ space (use embed=416, heads=8, head_dim=48, mlp=1664, depth=14); "depth": the 4 nested
    routes, each at 3 depths (depth - 2, depth - 1, depth), as (d_e, h, hidden, blocks).

    stem_dim > 0: the convolutional stem of Section 3.4 (7x7 stride-2 convolution and two
    depthwise-separable blocks at stem_dim channels, then the gate) precedes the patch embedding,
    which then is a patch x patch stride-patch convolution over the stem's half-resolution map.
    """
    step = embed // 6
    de_list = [3 * step, 4 * step, 5 * step, 6 * step]
    h_list = [heads - 3, heads - 2, heads - 1, heads]
    if routes == "cross":
        table = [(de, h, r * de) for de in de_list for h in h_list for r in (2, 3, 4)]
    elif routes == "diag":
        table = [(de_list[0], h_list[0], 2 * de_list[0]), (de_list[1], h_list[1], 3 * de_list[1]),
                 (de_list[2], h_list[2], 3 * de_list[2]), (de_list[3], h_list[3], 4 * de_list[3])]
    elif routes == "pp":
        # the DS-ViT++ routing space (its table in Section 5.2): embedding 192..416 in steps of 32, Q-K-V width
        # 48 h with h = 4..8 heads, MLP ratio 3 / 3.5 / 4, depth - 2 .. depth blocks; 8 nested routes along
        # the diagonal of that space, scaled to the stored sizes given
        s13 = embed // 13
        table = []
        for i in range(8):
            de = 6 * s13 + i * s13
            h = heads - 4 + (i * 4 + 3) // 7
            ratio2 = 6 + (i * 2 + 3) // 7                      # twice the MLP ratio: 6, 7 or 8
            table.append((de, h, ratio2 * de // 2, depth - 2 + (i * 2 + 3) // 7))
    elif routes == "depth":
        diag = [(de_list[0], h_list[0], 2 * de_list[0]), (de_list[1], h_list[1], 3 * de_list[1]),
                (de_list[2], h_list[2], 3 * de_list[2]), (de_list[3], h_list[3], 4 * de_list[3])]
        table = [(*r, depth - k) for r in diag for k in (2, 1, 0)]
    else:
        raise ValueError(routes)
    n_tok = (image // patch) ** 2 + 1
    extra = {}
    if stem_dim:
        n_tok = (image // 2 // patch) ** 2 + 1
        extra = {"stem_dim": stem_dim, "gate_hidden": 16, "bn_eps": 1e-5}
    return {
        **extra,
        "name": "vit", "image": image, "patch": patch, "embed": embed, "heads": heads,
        "head_dim": head_dim, "mlp": mlp, "depth": depth, "tokens": n_tok,
        "routes": np.array(table, np.int32), "T": len(table), "num_classes": 1000, "ln_eps": 1e-6,
    }


def vit_params(arch: dict, seed: int) -> dict:
    d = Draw(seed)
    D, Hd, M = arch["embed"], arch["heads"] * arch["head_dim"], arch["mlp"]
    P = arch["patch"]
    std = 0.02
    bf = as_bf16_values
    p = {}
    C = arch.get("stem_dim", 0)
    p["embed.w"] = bf(d.normal((D, C if C else 3, P, P), std=std))
    p["embed.b"] = d.normal((D,), std=std)
    p["cls"] = bf(d.normal((D,), std=std))
    p["pos"] = bf(d.normal((arch["tokens"], D), std=std))
    for l in range(arch["depth"]):
        pre = f"l{l}"
        p[pre + ".ln1.g"] = 1.0 + d.normal((D,), std=std)
        p[pre + ".ln1.b"] = d.normal((D,), std=std)
        for nm in ("q", "k", "v"):
            p[pre + f".w{nm}"] = bf(d.normal((Hd, D), std=std))
            p[pre + f".b{nm}"] = d.normal((Hd,), std=std)
        p[pre + ".wproj"] = bf(d.normal((D, Hd), std=std))
        p[pre + ".bproj"] = d.normal((D,), std=std)
        p[pre + ".ln2.g"] = 1.0 + d.normal((D,), std=std)
        p[pre + ".ln2.b"] = d.normal((D,), std=std)
        p[pre + ".fc1.w"] = bf(d.normal((M, D), std=std))
        p[pre + ".fc1.b"] = d.normal((M,), std=std)
        p[pre + ".fc2.w"] = bf(d.normal((D, M), std=std))
        p[pre + ".fc2.b"] = d.normal((D,), std=std)
    p["ln.g"] = 1.0 + d.normal((D,), std=std)
    p["ln.b"] = d.normal((D,), std=std)
    p["head.w"] = bf(d.normal((arch["num_classes"], D), std=std))
    p["head.b"] = d.normal((arch["num_classes"],), std=std)
    if C:
        T, hid = arch["T"], arch["gate_hidden"]
        p["stem.c0.w"] = bf(_kaiming(d, (C, 3, 7, 7)))
        p["stem.c0.bn"] = bn_tables(d, 1, C)
        for i in (1, 2):
            p[f"stem.ds{i}.dw.w"] = bf(_kaiming(d, (C, 1, 3, 3)))
            p[f"stem.ds{i}.dw.bn"] = bn_tables(d, 1, C)
            p[f"stem.ds{i}.pw.w"] = bf(_kaiming(d, (C, C, 1, 1)))
            p[f"stem.ds{i}.pw.bn"] = bn_tables(d, 1, C)
        p["gate.w1"] = d.normal((hid, C), std=C ** -0.5)
        p["gate.b1"] = d.normal((hid,), std=0.1)
        p["gate.w2"] = d.normal((T, hid), std=hid ** -0.5)
        p["gate.b2"] = d.normal((T,), std=0.1)
    return p
