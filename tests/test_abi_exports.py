"""The C-ABI library loads on a machine without a GPU and exports every symbol that
include/dsnet.h declares; host-side argument validation returns error codes."""
import ctypes
import os
import re

import pytest

import paper_2109_10060_amd as ds

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _lib():
    if not os.path.exists(ds.LIB_PATH):
        from paper_2109_10060_amd.build import build
        build(verbose=False)
    return ds.load()


def test_every_declared_symbol_is_exported():
    lib = _lib()
    header = open(os.path.join(ROOT, "include", "dsnet.h")).read()
    declared = set(re.findall(r"\b(ds_[a-z0-9_]+)\s*\(", header))
    assert {"ds_gate", "ds_route_bucket", "ds_sliced_conv", "ds_sliced_dwconv", "ds_sliced_linear",
            "ds_sliced_mhsa", "ds_forward"} <= declared
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} declared in dsnet.h but not exported"
    assert declared == set(ds.EXPORTS)
    assert lib.ds_version() >= 1


def test_host_validation_returns_codes_without_a_gpu():
    lib = _lib()
    g = ds.ds_groups()
    g.T = 0
    rc = lib.ds_sliced_linear(None, ctypes.c_int64(8), None, ctypes.c_int64(8), 8, 8, None, ctypes.byref(g), 4, 4, 0,
                              None, ctypes.c_int64(0), None, 1, ctypes.c_int64(8), None, ctypes.c_size_t(0), None)
    assert rc == ds.DS_EINVAL and b"T=0" in lib.ds_last_error()
    assert lib.ds_route_bucket(None, 4, 0, None, None, None, None) == ds.DS_EINVAL
    assert lib.ds_route_bucket(None, -1, 4, None, None, None, None) == ds.DS_EINVAL
    assert lib.ds_gate(None, 0, 0, 4, 8, 16, None, None, None, 4, None, None, 0, None, None, None, None,
                       ctypes.c_size_t(0), None) == ds.DS_EINVAL
    g.T = 1
    g.offsets = 1024  # never dereferenced on the host
    g.k_in[0], g.k_out[0] = 12, 8
    rc = lib.ds_sliced_linear(None, ctypes.c_int64(16), None, ctypes.c_int64(16), 8, 16, None, ctypes.byref(g), 4, 4,
                              0, None, ctypes.c_int64(0), None, 1, ctypes.c_int64(8), None, ctypes.c_size_t(0), None)
    assert rc == ds.DS_EALIGN
    g.k_in[0] = 32
    rc = lib.ds_sliced_linear(None, ctypes.c_int64(16), None, ctypes.c_int64(16), 8, 16, None, ctypes.byref(g), 4, 4,
                              0, None, ctypes.c_int64(0), None, 1, ctypes.c_int64(8), None, ctypes.c_size_t(0), None)
    assert rc == ds.DS_EINVAL          # slice larger than the stored weight
    assert lib.ds_sliced_mhsa(None, 2, 300, 64, None, None, None, None, 2, 64, ctypes.byref(g), None, None, None,
                              ctypes.c_size_t(0), None) == ds.DS_EUNSUPPORTED
    assert lib.ds_sliced_linear_workspace(64, 197, 4) >= 16 + 8 * (64 * 197 // 128 + 4)
    # the entry point without a workspace refuses what its built-in scratch cannot hold, before any device call
    g.k_in[0], g.k_out[0] = 16, 8
    rc = lib.ds_sliced_linear_noalloc(None, ctypes.c_int64(16), None, ctypes.c_int64(16), 8, 16, None, ctypes.byref(g), 1,
                                      128 * 40000, 0, None, ctypes.c_int64(0), None, 1, ctypes.c_int64(8), None)
    assert rc == ds.DS_EWORKSPACE and b"built-in scratch" in lib.ds_last_error()


def test_host_validation_of_the_spatial_statistics_and_forward_entry_points():
    lib = _lib()
    g = ds.ds_groups()
    g.T = 1
    g.offsets = 1024  # never dereferenced on the host
    g.k_in[0] = g.k_out[0] = 16
    sp = ds.ds_spatial()
    sp.ksize[0], sp.dilation[0], sp.pad[0] = 4, 1, 1                     # an even block is no centred crop of 7x7
    args = lambda: (None, 2, 16, 8, 8, None, 7, None, None, ctypes.byref(g), ctypes.byref(sp), 1, 1, None,
                    ctypes.c_int64(8 * 8 * 16), None, ctypes.c_size_t(0), None)
    assert lib.ds_sliced_dwconv_spatial(*args()) == ds.DS_EINVAL and b"centred" in lib.ds_last_error()
    sp.ksize[0], sp.dilation[0] = 3, 0
    assert lib.ds_sliced_dwconv_spatial(*args()) == ds.DS_EINVAL
    sp.dilation[0], sp.pad[0] = 1, 0
    a = list(args()); a[6] = 4                                          # stored filter must be odd
    assert lib.ds_sliced_dwconv_spatial(*a) == ds.DS_EUNSUPPORTED
    a = list(args()); a[14] = ctypes.c_int64(16)                        # output block too small for 6x6x16
    assert lib.ds_sliced_dwconv_spatial(*a) == ds.DS_ESHAPE
    assert lib.ds_sliced_dwconv_spatial(*args()) == ds.DS_EINVAL        # everything consistent, tensors null
    # statistics
    assert lib.ds_bn_stats_accumulate(None, 2, 0, 16, ctypes.byref(g), None, None, None, None, ctypes.c_size_t(0), None) == ds.DS_EINVAL
    g.k_in[0] = 12
    assert lib.ds_bn_stats_accumulate(None, 2, 4, 16, ctypes.byref(g), None, None, None, None, ctypes.c_size_t(0), None) == ds.DS_EINVAL
    w = (ctypes.c_int32 * 2)(8, 24)
    assert lib.ds_bn_stats_finish(None, None, None, 2, 16, w, None, None, None) == ds.DS_EINVAL
    assert lib.ds_bn_stats_workspace(4, 64, 32) > 0 and lib.ds_bn_stats_workspace(0, 64, 32) == 0
    # forward: a description whose integer list does not fit the architecture
    ints = (ctypes.c_int32 * 5)(224, 64, 4, 1000, 7)
    params = (ctypes.c_void_p * 1)(0)
    net = ds.ds_net(ds.DS_ARCH_RESNET, 5, ints, 1, params)
    assert lib.ds_forward_workspace(ctypes.byref(net), 4) == 0
    assert lib.ds_forward(ctypes.byref(net), None, 4, None, None, None, None, None, ctypes.c_size_t(0), None) == ds.DS_EINVAL
    assert lib.ds_forward(ctypes.byref(net), None, -1, None, None, None, None, None, ctypes.c_size_t(0), None) == ds.DS_EINVAL
    assert lib.ds_forward(ctypes.byref(net), None, 0, None, None, None, None, None, ctypes.c_size_t(0), None) == ds.DS_OK
    # a MobileNet-shaped description with a block stride of 0, then with a non-positive width: refused on the host
    # (no workspace size, DS_ESHAPE from the forward call) instead of dividing by zero
    def mb(stride, width):
        nb, T = 2, 1
        v = [32, 8, nb, 1, 4, T, 10] + [8, 16, 1, 16, width, stride] + [8, 16] + [16, width]
        arr = (ctypes.c_int32 * len(v))(*v)
        pp = (ctypes.c_void_p * (3 + 6 * nb + 6))(*([256] * (3 + 6 * nb + 6)))      # aligned, never dereferenced
        return ds.ds_net(ds.DS_ARCH_MBNET, len(v), arr, len(pp), pp), arr, pp
    good = mb(2, 16)
    assert lib.ds_forward_workspace(ctypes.byref(good[0]), 4) > 0
    for bad in (mb(0, 16), mb(3, 16), mb(1, 0), mb(1, -8)):
        assert lib.ds_forward_workspace(ctypes.byref(bad[0]), 4) == 0
        assert lib.ds_forward(ctypes.byref(bad[0]), ctypes.c_void_p(256), 4, None, None, ctypes.c_void_p(256), None, None,
                              ctypes.c_size_t(0), None) == ds.DS_ESHAPE
    assert lib.ds_forward_parts_workspace(ctypes.byref(net), 4, 2) == 0 and lib.ds_forward_parts_workspace(ctypes.byref(net), 4, 5) == 0
    assert lib.ds_forward_parts(ctypes.byref(net), None, 4, None, None, None, None, None, ctypes.c_size_t(0), 0, None) == ds.DS_EINVAL
    assert lib.ds_forward_parts(ctypes.byref(net), None, 4, None, None, None, None, None, ctypes.c_size_t(0), 5, None) == ds.DS_EINVAL
    assert lib.ds_forward_parts(ctypes.byref(net), None, 4, None, None, None, None, None, ctypes.c_size_t(0), 2, None) == ds.DS_EINVAL
    assert lib.ds_forward_parts(ctypes.byref(net), None, 0, None, None, None, None, None, ctypes.c_size_t(0), 2, None) == ds.DS_OK


def test_missing_library_fails_loudly(tmp_path):
    import importlib
    old = ds._lib
    ds._lib = None
    try:
        with pytest.raises(RuntimeError, match="no fallback"):
            ds.load(str(tmp_path / "nope.so"))
    finally:
        ds._lib = old
