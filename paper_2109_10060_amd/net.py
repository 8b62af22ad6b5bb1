"""Network descriptors for ds_forward.

Marshalling only: parameters arrive as host arrays in the logical layouts of the
network description (conv filters [C_O, C_I, K, K], depthwise [C, 1, 3, 3], linear
[out, in]); they are moved to the device in the storage layout the kernels read
in place (channels-last filters [C_O, K, K, C_I], depthwise [3, 3, C], stem
[K*K*3, C_O], stacked Q/K/V), split batch-norm statistics are folded to per-route
scale/shift tables by the library's own ds_bn_fold kernel, and the integer
description plus the device pointers are laid out in the order include/dsnet.h
documents for each architecture.
"""
from __future__ import annotations

import ctypes

import numpy as np
import torch


def _dev(a, dtype, device):
    return torch.from_numpy(np.ascontiguousarray(a)).to(device).to(dtype).contiguous()


class Net:
    def __init__(self, arch_id: int, ints, tensors, num_classes: int, n_gates: int, T: int):
        from . import ds_net
        self.arch_id = arch_id
        self.tensors = list(tensors)          # keeps device memory alive
        self.num_classes = num_classes
        self.n_gates = n_gates
        self.T = T
        self._ints = (ctypes.c_int32 * len(ints))(*[int(v) for v in ints])
        self._ptrs = (ctypes.c_void_p * len(self.tensors))(*[t.data_ptr() for t in self.tensors])
        self.c_struct = ds_net(arch_id, len(ints), ctypes.cast(self._ints, ctypes.POINTER(ctypes.c_int32)),
                               len(self.tensors), ctypes.cast(self._ptrs, ctypes.POINTER(ctypes.c_void_p)))
        self.device = self.tensors[0].device

    def workspace_bytes(self, B: int, parts: int = 1) -> int:
        from . import load
        if parts == 1:
            return int(load().ds_forward_workspace(ctypes.byref(self.c_struct), B))
        return int(load().ds_forward_parts_workspace(ctypes.byref(self.c_struct), B, parts))

    def workspace(self, B: int, parts: int = 1) -> torch.Tensor:
        return torch.empty(max(self.workspace_bytes(B, parts), 256), dtype=torch.uint8, device=self.device)


def _fold(bn, eps, device):
    from . import ds_bn_fold
    f32 = torch.float32
    return ds_bn_fold(_dev(bn["gamma"], f32, device), _dev(bn["beta"], f32, device), _dev(bn["mean"], f32, device),
                      _dev(bn["var"], f32, device), eps)


def _ohwi(w, device):
    return _dev(np.transpose(w, (0, 2, 3, 1)), torch.bfloat16, device)


def _stem(w, device):
    co = w.shape[0]
    return _dev(np.transpose(w, (2, 3, 1, 0)).reshape(-1, co), torch.bfloat16, device)


def build_mbnet(arch: dict, p: dict, device="cuda:0") -> Net:
    from . import DS_ARCH_MBNET
    bf, f32 = torch.bfloat16, torch.float32
    eps = arch["bn_eps"]
    nb, T = len(arch["blocks"]), arch["T"]
    ints = [arch["image"], arch["stem_out"], nb, arch["gate_after"], arch["gate_hidden"], T, arch["num_classes"]]
    for ci, co, s in arch["blocks"]:
        ints += [ci, co, s]
    ints += arch["cin"].reshape(-1).tolist() + arch["cout"].reshape(-1).tolist()
    if "ksize" in arch:
        ints += [int(k) for k in arch["kfull"]] + arch["ksize"].reshape(-1).tolist()
    t = [_stem(p["stem.w"], device), *_fold(p["stem.bn"], eps, device)]
    for i in range(nb):
        t.append(_dev(np.transpose(p[f"ds{i}.dw.w"][:, 0], (1, 2, 0)), bf, device))
        t += list(_fold(p[f"ds{i}.dw.bn"], eps, device))
        t.append(_dev(p[f"ds{i}.pw.w"][:, :, 0, 0], bf, device))
        t += list(_fold(p[f"ds{i}.pw.bn"], eps, device))
    t += [_dev(p[k], f32, device) for k in ("gate.w1", "gate.b1", "gate.w2", "gate.b2")]
    t += [_dev(p["fc.w"], bf, device), _dev(p["fc.b"], f32, device)]
    return Net(DS_ARCH_MBNET, ints, t, arch["num_classes"], 1, T)


def build_resnet(arch: dict, p: dict, device="cuda:0") -> Net:
    from . import DS_ARCH_RESNET
    bf, f32 = torch.bfloat16, torch.float32
    eps = arch["bn_eps"]
    T = arch["T"]
    ints = [arch["image"], arch["stem_out"], T, arch["num_classes"], *arch["widths"], *arch["blocks"],
            *arch["gate_hidden"], *arch["mid"].reshape(-1).tolist(), *arch["out"].reshape(-1).tolist()]
    if arch.get("nblk") is not None:
        ints += [int(v) for v in arch["nblk"].reshape(-1)]
        if arch.get("single_gate"):
            ints.append(1)
    t = [_stem(p["stem.w"], device), *_fold(p["stem.bn"], eps, device)]
    for s, nb in enumerate(arch["blocks"]):
        t += [_dev(p[f"s{s}.gate.{k}"], f32, device) for k in ("w1", "b1", "w2", "b2")]
        for b in range(nb):
            pre = f"s{s}.b{b}"
            for c in ("c1", "c2", "c3") + (("proj",) if b == 0 else ()):
                t.append(_ohwi(p[f"{pre}.{c}.w"], device))
                t += list(_fold(p[f"{pre}.{c}.bn"], eps, device))
    t += [_dev(p["fc.w"], bf, device), _dev(p["fc.b"], f32, device)]
    return Net(DS_ARCH_RESNET, ints, t, arch["num_classes"], 4, T)


def build_vit(arch: dict, p: dict, device="cuda:0") -> Net:
    from . import DS_ARCH_VIT, DS_ARCH_VIT_STEM
    bf, f32 = torch.bfloat16, torch.float32
    D = arch["embed"]
    C = arch.get("stem_dim", 0)
    ints = [arch["image"], arch["patch"], D, arch["heads"], arch["head_dim"], arch["mlp"], arch["depth"],
            arch["tokens"], arch["T"], arch["num_classes"]]
    t = []
    if C:
        eps = arch["bn_eps"]
        ints += [arch["routes"].shape[1], C, arch["gate_hidden"]]
        t += [_stem(p["stem.c0.w"], device), *_fold(p["stem.c0.bn"], eps, device)]
        for i in (1, 2):
            t.append(_dev(np.transpose(p[f"stem.ds{i}.dw.w"][:, 0], (1, 2, 0)), bf, device))
            t += list(_fold(p[f"stem.ds{i}.dw.bn"], eps, device))
            t.append(_dev(p[f"stem.ds{i}.pw.w"][:, :, 0, 0], bf, device))
            t += list(_fold(p[f"stem.ds{i}.pw.bn"], eps, device))
        t += [_dev(p[k], f32, device) for k in ("gate.w1", "gate.b1", "gate.w2", "gate.b2")]
        t.append(_ohwi(p["embed.w"], device))
    else:
        t.append(_dev(p["embed.w"].reshape(D, -1), bf, device))
    ints += arch["routes"].reshape(-1).tolist()
    t += [_dev(p["embed.b"], f32, device), _dev(p["cls"], bf, device), _dev(p["pos"], bf, device)]
    for l in range(arch["depth"]):
        q = f"l{l}"
        t += [_dev(p[q + ".ln1.g"], f32, device), _dev(p[q + ".ln1.b"], f32, device),
              _dev(np.stack([p[q + ".wq"], p[q + ".wk"], p[q + ".wv"]]), bf, device),
              _dev(np.stack([p[q + ".bq"], p[q + ".bk"], p[q + ".bv"]]), f32, device),
              _dev(p[q + ".wproj"], bf, device), _dev(p[q + ".bproj"], f32, device),
              _dev(p[q + ".ln2.g"], f32, device), _dev(p[q + ".ln2.b"], f32, device),
              _dev(p[q + ".fc1.w"], bf, device), _dev(p[q + ".fc1.b"], f32, device),
              _dev(p[q + ".fc2.w"], bf, device), _dev(p[q + ".fc2.b"], f32, device)]
    t += [_dev(p["ln.g"], f32, device), _dev(p["ln.b"], f32, device), _dev(p["head.w"], bf, device),
          _dev(p["head.b"], f32, device)]
    return Net(DS_ARCH_VIT_STEM if C else DS_ARCH_VIT, ints, t, arch["num_classes"], 1, arch["T"])
