"""CPU oracle for gate-routed, weight-sliced inference (DS-Net++, arXiv 2109.10060).

TEST INFRASTRUCTURE ONLY.  This module is a plain, slow, per-sample statement
of what the method computes, in float64 numpy.  It is used by the tests, by the
smoke check and by the benchmark's CPU-baseline leg; the product path never
imports it, and it shares no code with the HIP kernels.

Every layer is the textbook dense layer evaluated on the leading block of the
stored weight (Section 3.2, weight slicing, Eq. 8; Section 3.3, Eq. 9-10 and the
split batch-norm of Eq. 14; Section 3.4, Eq. 15-19; Section 3.5, Eq. 21-22).
There is no bucketing, tiling, permutation or fusion here: a batch is a Python
loop over independent samples (Eq. 1 is stated per input).

Storage precision: `store="bf16"` rounds a value to bfloat16 (nearest-even)
wherever the bf16 contract keeps a tensor in memory or feeds a bf16 matrix
operand: every conv/linear output after its epilogue, LayerNorm outputs, Q, K, V,
the softmax probabilities before P.V and the attention output.  Pooled vectors,
gate logits and classifier logits stay unrounded.  `store="f64"` rounds nothing.

All functions below are pinned by tests/test_oracle_*.py (closed forms,
brute-force loops, library routines on copied slices, masked-full == sliced,
prefix nesting, additivity, multiply-add counts printed in the paper).
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64


# --------------------------------------------------------------------------
# storage rounding
# --------------------------------------------------------------------------
def bf16_round(x):
    """Nearest bfloat16 (8 significant bits, ties to even) of float64 values."""
    x = np.asarray(x, F64)
    m, e = np.frexp(x)                 # x = m * 2**e, 0.5 <= |m| < 1
    q = np.rint(m * 256.0)             # 8 significant bits; rint rounds half to even
    return np.ldexp(q, e - 8)


def _store(x, store):
    if store == "bf16":
        return bf16_round(x)
    if store == "f64":
        return np.asarray(x, F64)
    raise ValueError(store)


# --------------------------------------------------------------------------
# routing agent (Section 3.5)
# --------------------------------------------------------------------------
def gate_encoder(x):
    """Eq. 21: spatial mean of each valid channel.  x: [c, H, W] -> [c]."""
    x = np.asarray(x, F64)
    return x.sum(axis=(1, 2)) / float(x.shape[1] * x.shape[2])


def gate_logits(pooled, w1, b1, w2, b2, logit_bias=None):
    """Eq. 22 scores before the softmax: W2 . relu(W1[:, :c] . pooled + b1) + b2.

    The first layer is input-sliced to the c valid channels (the gate MLP is
    itself a dynamic layer).  An optional per-sample additive term stands in
    for a trained gate's preference.
    """
    pooled = np.asarray(pooled, F64)
    c = pooled.shape[0]
    h = np.asarray(w1, F64)[:, :c] @ pooled
    if b1 is not None:
        h = h + np.asarray(b1, F64)
    h = np.maximum(h, 0.0)
    z = np.asarray(w2, F64) @ h
    if b2 is not None:
        z = z + np.asarray(b2, F64)
    if logit_bias is not None:
        z = z + np.asarray(logit_bias, F64)
    return z


def gate_hidden(pooled, w1, b1):
    """Hidden vector shared by the two heads of the gate: relu(W1[:, :c] . pooled + b1)."""
    pooled = np.asarray(pooled, F64)
    c = pooled.shape[0]
    h = np.asarray(w1, F64)[:, :c] @ pooled
    if b1 is not None:
        h = h + np.asarray(b1, F64)
    return np.maximum(h, 0.0)


def gate_attention_scale(x, w1, b1, w3, b3=None):
    """Channel-attention head of the double-headed gate (Section 3.5, Eq. 23): the hidden vector of
    the routing MLP is projected back to the channels by a third matrix W3 [C_I, C_mlp] and passed
    through delta(s) = 1 + tanh(s).  x: [c, H, W] with c valid channels; W1 is input-sliced to its
    first c columns and W3 output-sliced to its first c rows (both are dynamic layers of the
    sample's width).  Returns the per-channel factor [c]."""
    x = np.asarray(x, F64)
    c = x.shape[0]
    h = gate_hidden(gate_encoder(x), w1, b1)
    s = np.asarray(w3, F64)[:c] @ h
    if b3 is not None:
        s = s + np.asarray(b3, F64)[:c]
    return 1.0 + np.tanh(s)


def gate_attention(x, w1, b1, w3, b3=None):
    """Eq. 23: the re-weighted feature map X * delta(...), broadcast over the pixels."""
    x = np.asarray(x, F64)
    return x * gate_attention_scale(x, w1, b1, w3, b3)[:, None, None]


def gate_route(z):
    """Inference-time routing: index of the largest score (softmax is monotone, so
    it is skipped).  Ties go to the lowest index, i.e. the smaller sub-network; a
    NaN score is never selected; all-NaN gives route 0."""
    best, arg = None, 0
    for t, v in enumerate(np.asarray(z, F64).tolist()):
        if math.isnan(v):
            continue
        if best is None or v > best:
            best, arg = v, t
    return arg


def gate_margin(z):
    """Gap between the two largest scores (used to exempt near-ties from bit-exactness)."""
    s = np.sort(np.asarray(z, F64))
    return float(s[-1] - s[-2]) if s.size > 1 else float("inf")


def route_bucket(route, T):
    """Stable bucket-major ordering of a batch by route id.

    offsets[t] = number of samples with route < t (exclusive prefix sum of the
    histogram); perm lists sample indices bucket by bucket, ascending inside a
    bucket; inv_perm[perm[j]] = j.
    """
    route = [int(r) for r in route]
    B = len(route)
    for r in route:
        if r < 0 or r >= T:
            raise ValueError("route id out of range")
    offsets = [0] * (T + 1)
    perm = []
    for t in range(T):
        offsets[t] = len(perm)
        for b in range(B):
            if route[b] == t:
                perm.append(b)
    offsets[T] = len(perm)
    inv = [0] * B
    for j, b in enumerate(perm):
        inv[b] = j
    return (np.array(perm, np.int32), np.array(inv, np.int32), np.array(offsets, np.int32))


# --------------------------------------------------------------------------
# sliced layers (Sections 3.2-3.4)
# --------------------------------------------------------------------------
def sliced_linear(x, w, b, k_out):
    """Eq. 8: y[:k_out] = W[:k_out, :k_in] x + b[:k_out]; x: [..., k_in]."""
    x = np.asarray(x, F64)
    k_in = x.shape[-1]
    y = x @ np.asarray(w, F64)[:k_out, :k_in].T
    if b is not None:
        y = y + np.asarray(b, F64)[:k_out]
    return y


def sliced_conv2d(x, w, c_out, stride=1, pad=0):
    """Eq. 9: W[:c_out, :c_in] * X for one sample.  x: [c_in, H, W]; w: [C_O, C_I, K, K].

    Written as the sum over the K*K taps of a channel contraction on the
    shifted, strided view of the zero-padded input.
    """
    x = np.asarray(x, F64)
    w = np.asarray(w, F64)
    c_in, H, W = x.shape
    K = w.shape[2]
    Ho = (H + 2 * pad - K) // stride + 1
    Wo = (W + 2 * pad - K) // stride + 1
    xp = np.pad(x, ((0, 0), (pad, pad), (pad, pad)))
    y = np.zeros((c_out, Ho, Wo), F64)
    for u in range(K):
        for v in range(K):
            view = xp[:, u:u + stride * (Ho - 1) + 1:stride, v:v + stride * (Wo - 1) + 1:stride]
            y += np.tensordot(w[:c_out, :c_in, u, v], view, axes=([1], [0]))
    return y


def sliced_dwconv2d(x, w, stride=1, pad=1):
    """Eq. 10, first scheme with one channel per group: channel c of the output is
    filter c applied to channel c of the input, for the c_in valid channels."""
    x = np.asarray(x, F64)
    w = np.asarray(w, F64)
    c, H, W = x.shape
    K = w.shape[2]
    Ho = (H + 2 * pad - K) // stride + 1
    Wo = (W + 2 * pad - K) // stride + 1
    xp = np.pad(x, ((0, 0), (pad, pad), (pad, pad)))
    y = np.zeros((c, Ho, Wo), F64)
    for u in range(K):
        for v in range(K):
            view = xp[:, u:u + stride * (Ho - 1) + 1:stride, v:v + stride * (Wo - 1) + 1:stride]
            y += w[:c, 0, u, v][:, None, None] * view
    return y


def spatial_dwconv2d(x, w, k, dilation=1, stride=1, pad=0):
    """Depthwise convolution with a spatially sliced filter (Section 3.2).

    Kernel size (Eq. 11): the centred k x k block W[:, :, k0:k0+k, k0:k0+k], k0 = (K - k) / 2, of the
    stored K x K filter.  Dilation (Eq. 12): every `dilation`-th tap of that block, W[..., ::l, ::l];
    the taps keep their spacing, i.e. the n = ceil(k / l) selected taps per axis act as an n x n
    convolution of dilation l.  Padding (Eq. 13): `pad` zeros per side (the input padded to the
    maximum and cropped back is the same thing), which sets the output resolution
    (H + 2 pad - span) / stride + 1 with span = (n - 1) l + 1.
    x: [c, H, W] valid channels; w: [C, 1, K, K]."""
    x = np.asarray(x, F64)
    w = np.asarray(w, F64)
    c, H, W = x.shape
    K = w.shape[2]
    assert (K - k) % 2 == 0 and 1 <= k <= K and dilation >= 1
    k0 = (K - k) // 2
    taps = list(range(k0, k0 + k, dilation))
    span = (len(taps) - 1) * dilation + 1
    Ho = (H + 2 * pad - span) // stride + 1
    Wo = (W + 2 * pad - span) // stride + 1
    xp = np.pad(x, ((0, 0), (pad, pad), (pad, pad)))
    y = np.zeros((c, Ho, Wo), F64)
    for i, u in enumerate(taps):
        for j, v in enumerate(taps):
            a, b = i * dilation, j * dilation
            view = xp[:, a:a + stride * (Ho - 1) + 1:stride, b:b + stride * (Wo - 1) + 1:stride]
            y += w[:c, 0, u, v][:, None, None] * view
    return y


def re_sbn(x, bn, t, eps):
    """Eq. 14: gamma[:c] * (x - mu_t) / sigma_t + beta[:c] with route t's statistics;
    sigma_t = sqrt(var_t + eps).  x: [c, H, W]."""
    x = np.asarray(x, F64)
    c = x.shape[0]
    g = np.asarray(bn["gamma"], F64)[:c, None, None]
    b = np.asarray(bn["beta"], F64)[:c, None, None]
    mu = np.asarray(bn["mean"], F64)[t, :c, None, None]
    sd = np.sqrt(np.asarray(bn["var"], F64)[t, :c, None, None] + eps)
    return g * ((x - mu) / sd) + b


def re_sbn_recalibrate(samples, routes, T, C):
    """Re-calibration of the split batch-norm statistics (the paragraph above Eq. 14): for every route t,
    mu_t and sigma_t^2 of each valid channel are re-estimated over a calibration set, here as the mean and
    the biased variance over all pixels of all samples that take route t (the population statistics; for
    batches of equal size the mean is the average of the batch means, and the variance is the average of
    the batch variances plus the variance of the batch means).
    samples[b]: [c_b, H, W] pre-normalisation features with the valid channels of its route; routes[b] in
    [0, T).  Returns (mean [T, C], var [T, C], count [T] pixels per route); entries of channels a route
    does not reach, and of routes without samples, stay at mean 0, variance 1."""
    mean = np.zeros((T, C), F64)
    var = np.ones((T, C), F64)
    count = np.zeros(T, np.int64)
    for t in range(T):
        xs = [np.asarray(x, F64) for x, r in zip(samples, routes) if int(r) == t]
        if not xs:
            continue
        c = xs[0].shape[0]
        flat = np.concatenate([x.reshape(c, -1) for x in xs], axis=1)        # [c, pixels of all samples]
        count[t] = flat.shape[1]
        mean[t, :c] = flat.mean(axis=1)
        var[t, :c] = ((flat - mean[t, :c, None]) ** 2).mean(axis=1)
    return mean, var, count


def relu(x):
    return np.maximum(x, 0.0)


def maxpool3x3s2(x):
    """3x3 max-pool, stride 2, padding 1 (padding never wins the max)."""
    c, H, W = x.shape
    Ho, Wo = (H + 2 - 3) // 2 + 1, (W + 2 - 3) // 2 + 1
    xp = np.full((c, H + 2, W + 2), -np.inf, F64)
    xp[:, 1:-1, 1:-1] = x
    y = np.full((c, Ho, Wo), -np.inf, F64)
    for u in range(3):
        for v in range(3):
            y = np.maximum(y, xp[:, u:u + 2 * (Ho - 1) + 1:2, v:v + 2 * (Wo - 1) + 1:2])
    return y


def layernorm_sliced(x, g, b, eps):
    """LayerNorm over the d valid features only, with gamma[:d], beta[:d]; x: [N, d]."""
    x = np.asarray(x, F64)
    d = x.shape[-1]
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * np.asarray(g, F64)[:d] + np.asarray(b, F64)[:d]


def gelu(x):
    return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0)))


def softmax_rows(s):
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=-1, keepdims=True)


def sliced_mhsa(x, wq, bq, wk, bk, wv, bv, wproj, bproj, h, head_dim, store="f64"):
    """Eq. 16-18 for one sample.  x: [N, d_e]; Wq/Wk/Wv: [H*Dh, D_e]; Wproj: [D_e, H*Dh].

    Q, K, V use rows [:h*Dh] and columns [:d_e]; head j owns rows j*Dh..(j+1)*Dh;
    scores are scaled by 1/sqrt(Dh); the projection uses Wproj[:d_e, :h*Dh].
    """
    x = np.asarray(x, F64)
    d_e = x.shape[-1]
    hd = h * head_dim
    q = _store(sliced_linear(x, wq, bq, hd), store)
    k = _store(sliced_linear(x, wk, bk, hd), store)
    v = _store(sliced_linear(x, wv, bv, hd), store)
    heads = []
    for j in range(h):
        sl = slice(j * head_dim, (j + 1) * head_dim)
        s = (q[:, sl] @ k[:, sl].T) / math.sqrt(head_dim)
        p = _store(softmax_rows(s), store)
        heads.append(p @ v[:, sl])
    a = _store(np.concatenate(heads, axis=-1), store)
    return sliced_linear(a, wproj, bproj, d_e)


# --------------------------------------------------------------------------
# network assemblies (Section 5.2), one sample at a time
# --------------------------------------------------------------------------
def _conv_bn_relu(x, w, bn, t, eps, c_out, stride, pad, store, act=True, residual=None):
    y = re_sbn(sliced_conv2d(x, w, c_out, stride, pad), bn, t, eps)
    if residual is not None:
        y = y + residual
    if act:
        y = relu(y)
    return _store(y, store)


def forward_mbnet(arch, p, image, logit_bias=None, route_override=None, store="bf16", taps=None):
    """DS-MBNet: stem, 5 fixed depthwise-separable blocks, gate, 8 sliced blocks,
    pool, classifier with sliced input width.  Returns (logits[1000], route, gate scores).
    With arch["ksize"] (DS-MBNet++) the depthwise filters are stored larger and a route also
    picks their kernel size."""
    eps = arch["bn_eps"]
    x = _conv_bn_relu(np.asarray(image, F64), p["stem.w"], p["stem.bn"], 0, eps,
                      arch["stem_out"], 2, 1, store)
    t, z = 0, None
    for i, (_ci, _co, s) in enumerate(arch["blocks"]):
        if i == arch["gate_after"]:
            z = gate_logits(gate_encoder(x), p["gate.w1"], p["gate.b1"], p["gate.w2"], p["gate.b2"],
                            logit_bias)
            t = gate_route(z) if route_override is None else int(route_override)
        tb = t if i >= arch["gate_after"] else 0
        c_in = int(arch["cin"][t, i])
        c_out = int(arch["cout"][t, i])
        assert x.shape[0] == c_in
        if "ksize" in arch:
            # DS-MBNet++: the route's centred block of the stored filter (Eq. 11) at the padding that keeps
            # the resolution
            k = int(arch["ksize"][t, i])
            y = spatial_dwconv2d(x, p[f"ds{i}.dw.w"], k, 1, s, (k - 1) // 2)
        else:
            y = sliced_dwconv2d(x, p[f"ds{i}.dw.w"], s, 1)
        y = re_sbn(y, p[f"ds{i}.dw.bn"], tb, eps)
        x = _store(relu(y), store)
        x = _conv_bn_relu(x, p[f"ds{i}.pw.w"], p[f"ds{i}.pw.bn"], tb, eps, c_out, 1, 0, store)
        if taps is not None:
            taps[f"ds{i}"] = x
    pooled = gate_encoder(x)
    logits = sliced_linear(pooled, p["fc.w"], p["fc.b"], arch["num_classes"])
    return logits, t, z


def forward_resnet(arch, p, image, logit_bias=None, route_override=None, store="bf16", taps=None):
    """DS-ResNet: 7x7 stem, max-pool, four bottleneck stages.  The first block of a
    stage runs the gate on its input; the stage's mid width, output width and
    projection shortcut follow that route; later blocks inherit it.
    logit_bias / route_override: [4, T] / [4] per stage.  Returns (logits, routes[4], scores).

    arch["single_gate"]: only the first stage's gate decides; the later stages follow its route
    (their scores are still returned for reference).
    arch["nblk"][s][t], when present, is the number of blocks of stage s that route t runs
    (dynamic depth, Section 3.4 / Guideline I of Section 3.1): the first block always runs, since
    it changes resolution and width; the skipped later blocks are identities through their
    residual connections."""
    eps = arch["bn_eps"]
    x = _conv_bn_relu(np.asarray(image, F64), p["stem.w"], p["stem.bn"], 0, eps,
                      arch["stem_out"], 2, 3, store)
    x = maxpool3x3s2(x)
    routes, scores = [], []
    for s, nb in enumerate(arch["blocks"]):
        pre = f"s{s}"
        lb = None if logit_bias is None else logit_bias[s]
        z = gate_logits(gate_encoder(x), p[pre + ".gate.w1"], p[pre + ".gate.b1"],
                        p[pre + ".gate.w2"], p[pre + ".gate.b2"], lb)
        t = gate_route(z) if route_override is None else int(route_override[s])
        if arch.get("single_gate") and s > 0:
            t = routes[0]          # DS-ResNet++: the gate of the first block steers all four stages (Section 5.2)
        routes.append(t)
        scores.append(z)
        mid, out = int(arch["mid"][s, t]), int(arch["out"][s, t])
        run = nb if arch.get("nblk") is None else int(arch["nblk"][s][t])
        assert 1 <= run <= nb
        for b in range(run):
            bp = f"{pre}.b{b}"
            stride = 2 if (b == 0 and s > 0) else 1
            if b == 0:
                sc = _conv_bn_relu(x, p[bp + ".proj.w"], p[bp + ".proj.bn"], t, eps, out, stride, 0,
                                   store, act=False)
            else:
                sc = x
            y = _conv_bn_relu(x, p[bp + ".c1.w"], p[bp + ".c1.bn"], t, eps, mid, 1, 0, store)
            y = _conv_bn_relu(y, p[bp + ".c2.w"], p[bp + ".c2.bn"], t, eps, mid, stride, 1, store)
            x = _conv_bn_relu(y, p[bp + ".c3.w"], p[bp + ".c3.bn"], t, eps, out, 1, 0, store,
                              residual=sc)
            if taps is not None:
                taps[bp] = x
    pooled = gate_encoder(x)
    logits = sliced_linear(pooled, p["fc.w"], p["fc.b"], arch["num_classes"])
    return logits, routes, scores


def patchify(image, patch):
    """[3, H, W] -> [N, 3*patch*patch], patches in raster order, features ordered (c, u, v)
    to match a [D, 3, patch, patch] embedding filter flattened row-major."""
    c, H, W = image.shape
    gh, gw = H // patch, W // patch
    x = np.asarray(image, F64).reshape(c, gh, patch, gw, patch)
    return x.transpose(1, 3, 0, 2, 4).reshape(gh * gw, c * patch * patch)


def _vit_body(arch, p, tok, route, store, taps):
    """Class token, position embedding, the route's blocks, final LayerNorm and classifier for
    one sample whose patch tokens tok [N-1, d_e] (before the position embedding) are given."""
    r = [int(v) for v in arch["routes"][route]]
    d_e, h, hidden = r[:3]
    n_blocks = r[3] if len(r) > 3 else arch["depth"]
    eps = arch["ln_eps"]
    pos = np.asarray(p["pos"], F64)
    tok = tok + pos[1:, :d_e]
    cls = (np.asarray(p["cls"], F64)[:d_e] + pos[0, :d_e])[None, :]
    x = _store(np.concatenate([cls, tok], axis=0), store)
    for l in range(n_blocks):
        pre = f"l{l}"
        a = _store(layernorm_sliced(x, p[pre + ".ln1.g"], p[pre + ".ln1.b"], eps), store)
        att = sliced_mhsa(a, p[pre + ".wq"], p[pre + ".bq"], p[pre + ".wk"], p[pre + ".bk"],
                          p[pre + ".wv"], p[pre + ".bv"], p[pre + ".wproj"], p[pre + ".bproj"],
                          h, arch["head_dim"], store)
        x = _store(x + att, store)
        m = _store(layernorm_sliced(x, p[pre + ".ln2.g"], p[pre + ".ln2.b"], eps), store)
        hdn = _store(gelu(sliced_linear(m, p[pre + ".fc1.w"], p[pre + ".fc1.b"], hidden)), store)
        x = _store(x + sliced_linear(hdn, p[pre + ".fc2.w"], p[pre + ".fc2.b"], d_e), store)
        if taps is not None:
            taps[pre] = x
    f = _store(layernorm_sliced(x[:1], p["ln.g"], p["ln.b"], eps), store)
    return sliced_linear(f[0], p["head.w"], p["head.b"], arch["num_classes"])


def forward_vit(arch, p, image, route, store="bf16", taps=None):
    """DS-ViT with the route given (chosen before the patch embedding): sliced patch
    embedding (Eq. 15), class token and position embedding sliced to d_e, pre-LN
    blocks with sliced MHSA (Eq. 16-18) and sliced MLP (Eq. 19), final LayerNorm,
    classifier on the class token with sliced input width.

    A route may carry a fourth entry, its depth (Section 3.4 lists depth among the dimensions
    the DS-ViT++ gate controls): the route runs the first `depth` stored blocks and skips the
    rest, which the residual connections turn into identities (Guideline I of Section 3.1)."""
    d_e = int(arch["routes"][route][0])
    w_embed = np.asarray(p["embed.w"], F64).reshape(arch["embed"], -1)
    tok = sliced_linear(patchify(image, arch["patch"]), w_embed, p["embed.b"], d_e)
    return _vit_body(arch, p, tok, route, store, taps)


def forward_vit_stem(arch, p, image, logit_bias=None, route_override=None, store="bf16", taps=None):
    """DS-ViT++ with the efficient stem of Section 3.4: a strided convolution and two
    depthwise-separable blocks (each layer followed by batch-norm and ReLU, never sliced, width
    arch["stem_dim"]) run before the gate; the gate (Eq. 21-22) reads the stem's feature map and
    picks the route; the patch embedding is the stem's last convolution (kernel = stride =
    arch["patch"], no padding), its filters sliced to the route's d_e (Eq. 15 with the stem's
    channels as input).  Returns (logits, route, gate scores)."""
    eps = arch["bn_eps"]
    C = arch["stem_dim"]
    x = _conv_bn_relu(np.asarray(image, F64), p["stem.c0.w"], p["stem.c0.bn"], 0, eps, C, 2, 3, store)
    for i in (1, 2):
        y = re_sbn(sliced_dwconv2d(x, p[f"stem.ds{i}.dw.w"], 1, 1), p[f"stem.ds{i}.dw.bn"], 0, eps)
        x = _store(relu(y), store)
        x = _conv_bn_relu(x, p[f"stem.ds{i}.pw.w"], p[f"stem.ds{i}.pw.bn"], 0, eps, C, 1, 0, store)
    if taps is not None:
        taps["stem"] = x
    z = gate_logits(gate_encoder(x), p["gate.w1"], p["gate.b1"], p["gate.w2"], p["gate.b2"], logit_bias)
    t = gate_route(z) if route_override is None else int(route_override)
    d_e = int(arch["routes"][t][0])
    y = sliced_conv2d(x, p["embed.w"], d_e, arch["patch"], 0)           # [d_e, gh, gw]
    tok = y.reshape(d_e, -1).T + np.asarray(p["embed.b"], F64)[:d_e]
    return _vit_body(arch, p, tok, t, store, taps), t, z


# --------------------------------------------------------------------------
# multiply-add counts (the complexity measure of Section 4.2)
# --------------------------------------------------------------------------
def _osz(n, k, s, p):
    return (n + 2 * p - k) // s + 1


def madds_mbnet(arch, cin, cout, fc_in):
    """Multiply-adds of one MobileNetV1-shaped forward with the given per-block widths."""
    r = _osz(arch["image"], 3, 2, 1)
    total = r * r * 27 * arch["stem_out"]
    for i, (_a, _b, s) in enumerate(arch["blocks"]):
        r = _osz(r, 3, s, 1)
        total += r * r * 9 * int(cin[i]) + r * r * int(cin[i]) * int(cout[i])
    return total + fc_in * arch["num_classes"]


def madds_resnet(arch, mids, outs):
    """Multiply-adds of one ResNet-50-shaped forward; mids/outs: per-stage widths."""
    r = _osz(arch["image"], 7, 2, 3)
    total = r * r * 147 * arch["stem_out"]
    r = _osz(r, 3, 2, 1)
    cprev = arch["stem_out"]
    for s, nb in enumerate(arch["blocks"]):
        m, o = int(mids[s]), int(outs[s])
        for b in range(nb):
            stride = 2 if (b == 0 and s > 0) else 1
            ro = _osz(r, 3, stride, 1)
            cin = cprev if b == 0 else o
            total += r * r * cin * m + ro * ro * 9 * m * m + ro * ro * m * o
            if b == 0:
                total += ro * ro * cin * o
            r = ro
        cprev = o
    return total + cprev * arch["num_classes"]


def madds_patch_stem(image, d_e, dim, blocks, kernels, strides):
    """Multiply-adds of a convolutional patch-embedding stem (the table of Section 3.4):
    blocks[i] is "c" (dense convolution) or "ds" (depthwise + pointwise), all at width `dim`
    except the last layer, which projects to d_e; padding keeps n/stride output pixels."""
    r, cin, total = image, 3, 0
    for i, (kind, k, s) in enumerate(zip(blocks, kernels, strides)):
        cout = d_e if i == len(blocks) - 1 else dim
        r = r // s
        if kind == "c":
            total += r * r * k * k * cin * cout
        else:
            total += r * r * k * k * cin + r * r * cin * cout
        cin = cout
    return total


def madds_vit(arch, d_e, h, hidden):
    """Multiply-adds of one DS-ViT forward on route (d_e, h, hidden)."""
    N = arch["tokens"]
    hd = h * arch["head_dim"]
    total = (N - 1) * 3 * arch["patch"] ** 2 * d_e
    per_layer = 3 * N * d_e * hd + 2 * N * N * hd + N * hd * d_e + 2 * N * d_e * hidden
    return total + arch["depth"] * per_layer + d_e * arch["num_classes"]
