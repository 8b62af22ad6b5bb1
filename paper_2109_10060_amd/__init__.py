"""Thin ctypes binding over libdsnet.so (HIP kernels for gfx950).

Every function here has the name of the C entry point it forwards to (see
include/dsnet.h) and does argument marshalling only: it checks tensor dtypes,
allocates outputs and workspaces with torch, and passes raw device pointers plus
the current HIP stream.  All arithmetic of the method runs in the library's
kernels.  There is no CPU or eager fallback: if the shared library is missing
or cannot be loaded, load() raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

from .net import Net, build_mbnet, build_resnet, build_vit  # noqa: F401  (re-exported)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdsnet.so")

DS_OK = 0
DS_EINVAL, DS_ESHAPE, DS_EALIGN, DS_EUNSUPPORTED, DS_EWORKSPACE, DS_EHIP = -1, -2, -3, -4, -5, -6
DS_F32, DS_BF16 = 0, 1
DS_NCHW, DS_NHWC = 0, 1
DS_ACT_NONE, DS_ACT_RELU, DS_ACT_GELU = 0, 1, 2
DS_MAX_GROUPS = 64
DS_ARCH_MBNET, DS_ARCH_RESNET, DS_ARCH_VIT, DS_ARCH_VIT_STEM = 1, 2, 3, 4

EXPORTS = [
    "ds_last_error", "ds_version", "ds_bn_fold", "ds_bn_stats_workspace", "ds_bn_stats_accumulate", "ds_bn_stats_finish", "ds_gate_workspace", "ds_gate", "ds_gate_double_workspace",
    "ds_gate_double", "ds_route_bucket",
    "ds_sliced_linear_workspace", "ds_sliced_linear", "ds_sliced_linear_noalloc", "ds_sliced_conv_workspace", "ds_sliced_conv",
    "ds_slot_workspace", "ds_sliced_dwconv", "ds_sliced_dwconv_spatial", "ds_sliced_layernorm", "ds_pool_head_workspace", "ds_pool_head", "ds_maxpool", "ds_sliced_mhsa_workspace",
    "ds_sliced_mhsa", "ds_forward_workspace", "ds_forward", "ds_forward_taps", "ds_forward_parts_workspace", "ds_forward_parts", "ds_profile_enable", "ds_profile_reset", "ds_profile_read", "ds_profile_launches",
]


class DsError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libdsnet error {code}: {msg}")
        self.code = code


class ds_groups(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("offsets", ctypes.c_void_p), ("perm", ctypes.c_void_p),
                ("k_in", ctypes.c_int32 * DS_MAX_GROUPS), ("k_out", ctypes.c_int32 * DS_MAX_GROUPS),
                ("table_row", ctypes.c_int32 * DS_MAX_GROUPS)]


class ds_spatial(ctypes.Structure):
    _fields_ = [("ksize", ctypes.c_int32 * DS_MAX_GROUPS), ("dilation", ctypes.c_int32 * DS_MAX_GROUPS),
                ("pad", ctypes.c_int32 * DS_MAX_GROUPS)]


class ds_net(ctypes.Structure):
    _fields_ = [("arch", ctypes.c_int32), ("n_ints", ctypes.c_int32), ("ints", ctypes.POINTER(ctypes.c_int32)),
                ("n_params", ctypes.c_int32), ("params", ctypes.POINTER(ctypes.c_void_p))]


_lib = None


def load(path: Optional[str] = None):
    """Load libdsnet.so; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise RuntimeError(f"{path} not found: build it with `python -m paper_2109_10060_amd.build` "
                           "(there is no fallback path)")
    lib = ctypes.CDLL(path)
    lib.ds_last_error.restype = ctypes.c_char_p
    for name in ("ds_gate_workspace", "ds_sliced_linear_workspace", "ds_sliced_conv_workspace",
                 "ds_slot_workspace", "ds_sliced_mhsa_workspace", "ds_forward_workspace", "ds_forward_parts_workspace", "ds_gate_double_workspace",
                 "ds_bn_stats_workspace", "ds_pool_head_workspace"):
        getattr(lib, name).restype = ctypes.c_size_t
    _lib = lib
    return lib


def _chk(rc: int):
    if rc != DS_OK:
        raise DsError(rc, load().ds_last_error().decode())


def _ptr(t: Optional[torch.Tensor], dtype=None):
    if t is None:
        return ctypes.c_void_p(0)
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA tensors"
    if dtype is not None:
        assert t.dtype == dtype, f"expected {dtype}, got {t.dtype}"
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ws(nbytes: int, like: torch.Tensor) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=like.device)


def make_groups(offsets: torch.Tensor, perm: Optional[torch.Tensor], k_in: Sequence[int],
                k_out: Optional[Sequence[int]] = None, table_row: Optional[Sequence[int]] = None) -> ds_groups:
    g = ds_groups()
    T = len(k_in)
    assert T <= DS_MAX_GROUPS
    g.T = T
    g.offsets = _ptr(offsets, torch.int32).value
    g.perm = _ptr(perm, torch.int32).value if perm is not None else None
    k_out = k_in if k_out is None else k_out
    table_row = range(T) if table_row is None else table_row
    for t in range(T):
        g.k_in[t], g.k_out[t], g.table_row[t] = int(k_in[t]), int(k_out[t]), int(table_row[t])
    return g


# --------------------------------------------------------------------------
# entry points
# --------------------------------------------------------------------------
def ds_bn_fold(gamma, beta, mean, var, eps: float):
    T, C = mean.shape
    scale, shift = torch.empty_like(mean), torch.empty_like(mean)
    _chk(load().ds_bn_fold(_ptr(gamma, torch.float32), _ptr(beta, torch.float32), _ptr(mean, torch.float32),
                           _ptr(var, torch.float32), ctypes.c_float(eps), T, C, _ptr(scale), _ptr(shift), _stream()))
    return scale, shift


def ds_bn_stats_accumulate(x, groups: ds_groups, sum_, sumsq, count):
    """x: [B, HW, C] bf16; sum_, sumsq: [T, C] fp64; count: [T] int64 (all device, updated in place)."""
    lib = load()
    B, HW, C = x.shape
    ws = _ws(lib.ds_bn_stats_workspace(B, HW, C), x)
    _chk(lib.ds_bn_stats_accumulate(_ptr(x, torch.bfloat16), B, HW, C, ctypes.byref(groups), _ptr(sum_, torch.float64),
                                    _ptr(sumsq, torch.float64), _ptr(count, torch.int64), _ptr(ws),
                                    ctypes.c_size_t(ws.numel()), _stream()))


def ds_bn_stats_finish(sum_, sumsq, count, width: Optional[Sequence[int]] = None):
    """Returns (mean, var) fp32 [T, C]."""
    T, C = sum_.shape
    mean = torch.empty((T, C), dtype=torch.float32, device=sum_.device)
    var = torch.empty_like(mean)
    w = (ctypes.c_int32 * T)(*[int(v) for v in width]) if width is not None else None
    _chk(load().ds_bn_stats_finish(_ptr(sum_, torch.float64), _ptr(sumsq, torch.float64), _ptr(count, torch.int64), T, C, w,
                                   _ptr(mean), _ptr(var), _stream()))
    return mean, var


def ds_gate(x, layout, w1, b1, w2, b2, T: int, logit_bias=None, c_in=None, B: Optional[int] = None):
    """Returns (logits [B,T] fp32, route [B] int32)."""
    lib = load()
    if x is not None:
        B = x.shape[0]
        if layout == DS_NCHW:
            C, HW = x.shape[1], x.shape[2] * x.shape[3]
        else:
            C, HW = x.shape[-1], x.numel() // (x.shape[0] * x.shape[-1])
        dt = DS_BF16 if x.dtype == torch.bfloat16 else DS_F32
        dev = x.device
        C_mlp = w1.shape[0]
    else:
        C = HW = C_mlp = 0
        dt = DS_F32
        dev = logit_bias.device
        B = logit_bias.shape[0] if B is None else B
    logits = torch.empty((B, T), dtype=torch.float32, device=dev)
    route = torch.empty((B,), dtype=torch.int32, device=dev)
    nb = lib.ds_gate_workspace(B, C)
    ws = _ws(nb, logits)
    _chk(lib.ds_gate(_ptr(x), dt, layout, B, C, HW, _ptr(c_in), _ptr(w1), _ptr(b1), C_mlp, _ptr(w2), _ptr(b2), T,
                     _ptr(logit_bias), _ptr(logits), _ptr(route), _ptr(ws), ctypes.c_size_t(ws.numel()), _stream()))
    return logits, route


def ds_gate_double(x, layout, w1, b1, w3, b3=None, w2=None, b2=None, T: int = 0, logit_bias=None, c_in=None, y=None):
    """Double-headed gate.  Returns (y, logits or None, route or None); y = x * (1 + tanh(W3 h + b3))."""
    lib = load()
    B = x.shape[0]
    if layout == DS_NCHW:
        C, HW = x.shape[1], x.shape[2] * x.shape[3]
    else:
        C, HW = x.shape[-1], x.numel() // (x.shape[0] * x.shape[-1])
    dt = DS_BF16 if x.dtype == torch.bfloat16 else DS_F32
    C_mlp = w1.shape[0]
    if y is None:
        y = torch.empty_like(x)
    logits = route = None
    if w2 is not None:
        logits = torch.empty((B, T), dtype=torch.float32, device=x.device)
        route = torch.empty((B,), dtype=torch.int32, device=x.device)
    ws = _ws(lib.ds_gate_double_workspace(B, C), x)
    _chk(lib.ds_gate_double(_ptr(x), dt, layout, B, C, HW, _ptr(c_in), _ptr(w1), _ptr(b1), C_mlp, _ptr(w2), _ptr(b2), T,
                            _ptr(logit_bias), _ptr(w3), _ptr(b3), _ptr(logits), _ptr(route), _ptr(y), _ptr(ws),
                            ctypes.c_size_t(ws.numel()), _stream()))
    return y, logits, route


def ds_route_bucket(route: torch.Tensor, T: int):
    """Returns (perm, inv_perm, offsets[T+1]) as int32 device tensors."""
    B = route.shape[0]
    perm = torch.empty((B,), dtype=torch.int32, device=route.device)
    inv = torch.empty((B,), dtype=torch.int32, device=route.device)
    off = torch.empty((T + 1,), dtype=torch.int32, device=route.device)
    _chk(load().ds_route_bucket(_ptr(route, torch.int32), B, T, _ptr(perm), _ptr(inv), _ptr(off), _stream()))
    return perm, inv, off


def ds_sliced_linear(x, w, bias, groups: ds_groups, act=DS_ACT_NONE, residual=None, y=None, y_dtype=torch.bfloat16,
                     n_full: Optional[int] = None):
    """x: [B, rows, x_ld] bf16; w: [N_full, K_full] bf16.  Writes only the valid slices of y."""
    lib = load()
    B, rows, x_ld = x.shape
    N_full, K_full = w.shape
    if y is None:
        y = torch.zeros((B, rows, N_full), dtype=y_dtype, device=x.device)
    ws = _ws(lib.ds_sliced_linear_workspace(B, rows, groups.T), x)
    _chk(lib.ds_sliced_linear(_ptr(x, torch.bfloat16), ctypes.c_int64(x_ld), _ptr(w, torch.bfloat16),
                              ctypes.c_int64(w.stride(0)), N_full, K_full, _ptr(bias), ctypes.byref(groups), B, rows,
                              act, _ptr(residual), ctypes.c_int64(residual.shape[-1] if residual is not None else 0),
                              _ptr(y), DS_BF16 if y.dtype == torch.bfloat16 else DS_F32, ctypes.c_int64(y.shape[-1]),
                              _ptr(ws), ctypes.c_size_t(ws.numel()), _stream()))
    return y


def ds_sliced_linear_noalloc(x, w, bias, groups: ds_groups, y, act=DS_ACT_NONE, residual=None):
    """ds_sliced_linear without a workspace (the library's built-in scratch); y is required, nothing is allocated."""
    B, rows, x_ld = x.shape
    N_full, K_full = w.shape
    _chk(load().ds_sliced_linear_noalloc(_ptr(x, torch.bfloat16), ctypes.c_int64(x_ld), _ptr(w, torch.bfloat16),
                                         ctypes.c_int64(w.stride(0)), N_full, K_full, _ptr(bias), ctypes.byref(groups), B,
                                         rows, act, _ptr(residual),
                                         ctypes.c_int64(residual.shape[-1] if residual is not None else 0), _ptr(y),
                                         DS_BF16 if y.dtype == torch.bfloat16 else DS_F32, ctypes.c_int64(y.shape[-1]),
                                         _stream()))
    return y


def ds_sliced_conv(x, w, scale, shift, groups: ds_groups, stride: int, pad: int, act=DS_ACT_RELU, residual=None,
                   y=None):
    """fp32: x [B,C_I,H,W], w [C_O,C_I,K,K].  bf16: x [B,H,W,C_I], w [C_O,K,K,C_I]."""
    lib = load()
    if x.dtype == torch.float32:
        B, C_I, H, W = x.shape
        C_O, K = w.shape[0], w.shape[2]
        dt, layout = DS_F32, DS_NCHW
    else:
        B, H, W, C_I = x.shape
        C_O, K = w.shape[0], w.shape[1]
        dt, layout = DS_BF16, DS_NHWC
    Ho, Wo = (H + 2 * pad - K) // stride + 1, (W + 2 * pad - K) // stride + 1
    if y is None:
        shp = (B, C_O, Ho, Wo) if layout == DS_NCHW else (B, Ho, Wo, C_O)
        y = torch.zeros(shp, dtype=x.dtype, device=x.device)
    ws = _ws(lib.ds_sliced_conv_workspace(B, Ho, Wo, groups.T), x)
    _chk(lib.ds_sliced_conv(_ptr(x), dt, layout, B, C_I, H, W, _ptr(w, x.dtype), C_O, K, _ptr(scale), _ptr(shift),
                            ctypes.byref(groups), stride, pad, act, _ptr(residual), _ptr(y), _ptr(ws),
                            ctypes.c_size_t(ws.numel()), _stream()))
    return y


def ds_sliced_dwconv(x, w, scale, shift, groups: ds_groups, stride: int, act=DS_ACT_RELU, y=None):
    """x: [B,H,W,C] bf16; w: [3,3,C] bf16."""
    lib = load()
    B, H, W, C = x.shape
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    if y is None:
        y = torch.zeros((B, Ho, Wo, C), dtype=x.dtype, device=x.device)
    ws = _ws(lib.ds_slot_workspace(B), x)
    _chk(lib.ds_sliced_dwconv(_ptr(x, torch.bfloat16), B, C, H, W, _ptr(w, torch.bfloat16), _ptr(scale), _ptr(shift),
                              ctypes.byref(groups), stride, act, _ptr(y), _ptr(ws), ctypes.c_size_t(ws.numel()),
                              _stream()))
    return y


def ds_sliced_dwconv_spatial(x, w, scale, shift, groups: ds_groups, ksize: Sequence[int], dilation: Sequence[int],
                             pad: Sequence[int], stride: int, act=DS_ACT_RELU, y=None):
    """x: [B,H,W,C] bf16; w: [K,K,C] bf16.  y: [B, rows_max, C] with each sample's Ho_t x Wo_t pixels packed at
    the start of its block (rows_max = the largest Ho_t * Wo_t); returns (y, [(Ho_t, Wo_t) per group])."""
    lib = load()
    B, H, W, C = x.shape
    K = w.shape[0]
    sp = ds_spatial()
    res = []
    for t in range(groups.T):
        sp.ksize[t], sp.dilation[t], sp.pad[t] = int(ksize[t]), int(dilation[t]), int(pad[t])
        dl = max(int(dilation[t]), 1)          # an invalid table is reported by the library, not here
        n = (int(ksize[t]) + dl - 1) // dl
        span = (n - 1) * dl + 1
        res.append(((H + 2 * int(pad[t]) - span) // stride + 1, (W + 2 * int(pad[t]) - span) // stride + 1))
    rows_max = max(max(a * b for a, b in res), 1)
    if y is None:
        y = torch.zeros((B, rows_max, C), dtype=x.dtype, device=x.device)
    ws = _ws(lib.ds_slot_workspace(B), x)
    _chk(lib.ds_sliced_dwconv_spatial(_ptr(x, torch.bfloat16), B, C, H, W, _ptr(w, torch.bfloat16), K, _ptr(scale), _ptr(shift),
                                      ctypes.byref(groups), ctypes.byref(sp), stride, act, _ptr(y),
                                      ctypes.c_int64(y.shape[1] * y.shape[2]), _ptr(ws), ctypes.c_size_t(ws.numel()),
                                      _stream()))
    return y, res


def ds_sliced_layernorm(x, gamma, beta, eps: float, groups: ds_groups, y=None):
    lib = load()
    B, rows, ld = x.shape
    if y is None:
        y = torch.zeros_like(x)
    ws = _ws(lib.ds_slot_workspace(B), x)
    _chk(lib.ds_sliced_layernorm(_ptr(x, torch.bfloat16), ctypes.c_int64(ld), _ptr(gamma, torch.float32),
                                 _ptr(beta, torch.float32), ctypes.c_float(eps), ctypes.byref(groups), B, rows,
                                 _ptr(y), ctypes.c_int64(y.shape[-1]), _ptr(ws), ctypes.c_size_t(ws.numel()), _stream()))
    return y


def ds_pool_head(x, w, bias, groups: ds_groups):
    """x: [B, HW, C] bf16; w: [n_out, C] bf16.  Returns logits [B, n_out] fp32."""
    lib = load()
    B, HW, C = x.shape
    n_out = w.shape[0]
    logits = torch.empty((B, n_out), dtype=torch.float32, device=x.device)
    ws = _ws(lib.ds_pool_head_workspace(B, C), x)
    _chk(lib.ds_pool_head(_ptr(x, torch.bfloat16), B, HW, C, _ptr(w, torch.bfloat16), _ptr(bias), n_out, ctypes.byref(groups),
                          _ptr(logits), _ptr(ws), ctypes.c_size_t(ws.numel()), _stream()))
    return logits


def ds_maxpool(x):
    """x: [B, H, W, C] bf16 -> [B, Ho, Wo, C], 3x3 stride 2 padding 1."""
    B, H, W, C = x.shape
    y = torch.empty((B, (H - 1) // 2 + 1, (W - 1) // 2 + 1, C), dtype=x.dtype, device=x.device)
    _chk(load().ds_maxpool(_ptr(x, torch.bfloat16), B, H, W, C, _ptr(y), _stream()))
    return y


def ds_sliced_mhsa(x, wqkv, bqkv, wproj, bproj, H: int, head_dim: int, groups: ds_groups, residual=None, y=None):
    """x: [B,N,D_e] bf16; wqkv: [3,H*Dh,D_e] bf16; wproj: [D_e,H*Dh] bf16."""
    lib = load()
    B, N, D_e = x.shape
    if y is None:
        y = torch.zeros_like(x)
    ws = _ws(lib.ds_sliced_mhsa_workspace(B, N, H, head_dim, groups.T), x)
    _chk(lib.ds_sliced_mhsa(_ptr(x, torch.bfloat16), B, N, D_e, _ptr(wqkv, torch.bfloat16), _ptr(bqkv),
                            _ptr(wproj, torch.bfloat16), _ptr(bproj), H, head_dim, ctypes.byref(groups),
                            _ptr(residual), _ptr(y), _ptr(ws), ctypes.c_size_t(ws.numel()), _stream()))
    return y


def ds_forward(net: "Net", images, route_override=None, logit_bias=None, logits=None, routes=None, ws=None):
    """images: [B,3,S,S] bf16.  Returns (logits [B,classes] fp32, routes [n_gates,B] int32)."""
    lib = load()
    B = images.shape[0]
    if logits is None:
        logits = torch.empty((B, net.num_classes), dtype=torch.float32, device=images.device)
    if routes is None:
        routes = torch.empty((net.n_gates, B), dtype=torch.int32, device=images.device)
    if ws is None:
        ws = net.workspace(B)
    _chk(lib.ds_forward(ctypes.byref(net.c_struct), _ptr(images, torch.bfloat16), B, _ptr(route_override),
                        _ptr(logit_bias), _ptr(logits), _ptr(routes), _ptr(ws), ctypes.c_size_t(ws.numel()), _stream()))
    return logits, routes


def ds_forward_taps(net: "Net", images, taps: dict, route_override=None, logit_bias=None, ws=None):
    """ds_forward that also fills taps[block index] (bf16 [B, rows, C_stored] device tensors, original sample order)
    with the outputs of those blocks.  Returns (logits, routes)."""
    lib = load()
    B = images.shape[0]
    logits = torch.empty((B, net.num_classes), dtype=torch.float32, device=images.device)
    routes = torch.empty((net.n_gates, B), dtype=torch.int32, device=images.device)
    if ws is None:
        ws = net.workspace(B)
    ids = sorted(taps)
    c_ids = (ctypes.c_int32 * max(len(ids), 1))(*ids)
    c_out = (ctypes.c_void_p * max(len(ids), 1))(*[_ptr(taps[i], torch.bfloat16).value for i in ids])
    _chk(lib.ds_forward_taps(ctypes.byref(net.c_struct), _ptr(images, torch.bfloat16), B, _ptr(route_override),
                             _ptr(logit_bias), _ptr(logits), _ptr(routes), len(ids), c_ids, c_out, _ptr(ws),
                             ctypes.c_size_t(ws.numel()), _stream()))
    return logits, routes


def ds_forward_parts(net: "Net", images, parts: int, route_override=None, logit_bias=None, logits=None, routes=None, ws=None):
    """ds_forward with the batch run as `parts` concurrent pieces (the first on the current stream, the others on
    streams of the library).  Same results; ws needs net.workspace(B, parts)."""
    lib = load()
    B = images.shape[0]
    if logits is None:
        logits = torch.empty((B, net.num_classes), dtype=torch.float32, device=images.device)
    if routes is None:
        routes = torch.empty((net.n_gates, B), dtype=torch.int32, device=images.device)
    if ws is None:
        ws = net.workspace(B, parts)
    _chk(lib.ds_forward_parts(ctypes.byref(net.c_struct), _ptr(images, torch.bfloat16), B, _ptr(route_override),
                              _ptr(logit_bias), _ptr(logits), _ptr(routes), _ptr(ws), ctypes.c_size_t(ws.numel()),
                              int(parts), _stream()))
    return logits, routes


KERNEL_CLASSES = ["gemm", "gemm_taps", "attention", "dwconv", "layernorm", "stem", "maxpool", "head", "gate",
                  "bucket", "index", "conv3", "thin"]


def ds_profile_enable(on: bool):
    _chk(load().ds_profile_enable(1 if on else 0))


def ds_profile_reset():
    _chk(load().ds_profile_reset())


def ds_profile_read() -> dict:
    """{kernel class: (total milliseconds, launches)} for the launches recorded since enable."""
    lib = load()
    out = {}
    for k, name in enumerate(KERNEL_CLASSES):
        ms, n = ctypes.c_double(0), ctypes.c_int64(0)
        _chk(lib.ds_profile_read(k, ctypes.byref(ms), ctypes.byref(n)))
        out[name] = (ms.value, n.value)
    return out


def ds_profile_launches() -> list:
    """[(kernel class, milliseconds)] of the recorded launches, in launch order."""
    lib = load()
    n = ctypes.c_int64(0)
    _chk(lib.ds_profile_launches(None, None, ctypes.c_int64(0), ctypes.byref(n)))
    kinds = (ctypes.c_int32 * max(n.value, 1))()
    ms = (ctypes.c_float * max(n.value, 1))()
    _chk(lib.ds_profile_launches(kinds, ms, ctypes.c_int64(n.value), ctypes.byref(n)))
    return [(KERNEL_CLASSES[kinds[i]], float(ms[i])) for i in range(n.value)]
