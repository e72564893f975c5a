"""Host-only checks of the C ABI: the library loads, exports every declared symbol, and
validates descriptors and arguments without touching a GPU."""
import ctypes
import os
import re

import pytest

import paper_2206_07446_amd as nnv
from nnv_workloads import stack, STACK_NAMES
from oracle import layouts as OL

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_header_symbols_exported():
    hdr = open(os.path.join(ROOT, "include", "nnv.h")).read()
    declared = set(re.findall(r"\b(nnv_[a-z_]+)\s*\(", hdr))
    assert declared == set(nnv.EXPORTS)
    lib = nnv.load()
    for name in declared:
        assert getattr(lib, name) is not None


def test_version_and_status_strings():
    assert nnv.nnv_layout_version() == 1
    assert nnv.nnv_status_string(0) == "ok"
    for s in range(-9, 0):
        assert nnv.nnv_status_string(s) not in ("ok", "unknown status")
    assert nnv.nnv_status_string(-99) == "unknown status"


def D(**kw):
    base = dict(n=1, c=16, h=32, w=32, k=16, r=3, s=3, stride_h=1, stride_w=1, pad_h=1, pad_w=1, groups=1, dtype=0)
    base.update(kw)
    return nnv.ConvDesc(**base)


def test_kind_supported_rules():
    d = D()
    assert [nnv.nnv_kind_supported(d, k) for k in range(5)] == [True, True, True, True, False]
    d = D(stride_h=2, stride_w=2)
    assert [nnv.nnv_kind_supported(d, k) for k in range(5)] == [True, True, False, False, False]
    d = D(groups=16)      # depthwise; also a (wasteful) grouped GEMM: one 16-row panel per channel
    assert [nnv.nnv_kind_supported(d, k) for k in range(5)] == [True, True, False, False, True]
    d = D(groups=16, stride_h=2, stride_w=2)
    assert nnv.nnv_kind_supported(d, nnv.DEPTHWISE)
    d = D(r=7, s=7, pad_h=3, pad_w=3, stride_h=2, stride_w=2, c=3)
    assert [nnv.nnv_kind_supported(d, k) for k in range(5)] == [True, True, False, False, False]
    d = D(groups=2)
    assert [nnv.nnv_kind_supported(d, k) for k in range(5)] == [True, True, False, False, False]
    # grouped GEMM: at most 64 groups; float16 with a 3x3 filter needs 32-channel-aligned groups
    assert not nnv.nnv_kind_supported(D(c=128, k=128, groups=128), 1)
    assert not nnv.nnv_kind_supported(D(groups=2, dtype=1), 1)
    assert nnv.nnv_kind_supported(D(c=64, k=64, groups=2, dtype=1), 1)
    assert nnv.nnv_kind_supported(D(groups=2, dtype=1, r=1, s=1, pad_h=0, pad_w=0), 1)
    # float16 Winograd needs at least 16 input channels (accuracy), F(6x6) is float32 only
    assert [nnv.nnv_kind_supported(D(dtype=1), k) for k in (2, 3, 5)] == [True, True, False]
    assert [nnv.nnv_kind_supported(D(c=15, dtype=1), k) for k in (2, 3, 5)] == [False, False, False]
    assert [nnv.nnv_kind_supported(D(c=15), k) for k in (2, 3, 5)] == [True, True, True]
    assert nnv.nnv_transformed_bytes(D(c=15, dtype=1), 3) == 0 and nnv.nnv_workspace_bytes(D(c=15, dtype=1), 3) == 0


@pytest.mark.parametrize("bad", [dict(n=0), dict(c=-1), dict(groups=3), dict(stride_h=0), dict(pad_w=-1),
                                 dict(dtype=2), dict(h=1, w=1, pad_h=0, pad_w=0), dict(k=70000),
                                 dict(pad_h=2 ** 30), dict(pad_w=2 ** 31 - 1), dict(pad_h=2 ** 29, pad_w=2 ** 29)])
def test_bad_descriptors(bad):
    d = D(**bad)
    with pytest.raises(nnv.NnvError) as e:
        nnv.nnv_kind_supported(d, 0)
    assert e.value.status == -2
    assert nnv.nnv_transformed_bytes(d, 0) == 0
    assert nnv.nnv_workspace_bytes(d, 1) == 0


def test_null_and_argument_errors_need_no_gpu():
    lib = nnv.load()
    d = D()
    assert lib.nnv_transform_weights(None, 0, None, None, None) == -1
    assert lib.nnv_transform_weights(ctypes.byref(d), 1, None, None, None) == -1
    assert lib.nnv_transform_weights(ctypes.byref(d), 9, ctypes.c_void_p(256), ctypes.c_void_p(512), None) == -7
    assert lib.nnv_transform_weights(ctypes.byref(d), 4, ctypes.c_void_p(256), ctypes.c_void_p(512), None) == -3
    assert lib.nnv_transform_weights(ctypes.byref(d), 1, ctypes.c_void_p(260), ctypes.c_void_p(512), None) == -5
    assert lib.nnv_conv_forward(ctypes.byref(d), 1, None, None, None, None, None, 0, None) == -1
    assert lib.nnv_conv_forward(ctypes.byref(d), 3, ctypes.c_void_p(256), ctypes.c_void_p(256), None,
                                ctypes.c_void_p(256), ctypes.c_void_p(256), 16, None) == -4
    assert lib.nnv_time_layer(ctypes.byref(d), 1, None, None, None, None, None, 0, None, 0, 1, 1, None, None) == -1
    t = nnv.Timing()
    assert lib.nnv_time_layer(ctypes.byref(d), 1, ctypes.c_void_p(256), ctypes.c_void_p(256), ctypes.c_void_p(256),
                              ctypes.c_void_p(256), None, 0, None, 0, 1, 0, None, ctypes.byref(t)) == -7
    assert lib.nnv_transform_weights_grouped(-1, None, None, None, None, None) == -7
    assert lib.nnv_transform_weights_grouped(0, None, None, None, None, None) == 0


KNAME = {0: "direct", 1: "im2col_gemm", 2: "wino_f2", 3: "wino_f4", 4: "depthwise", 5: "wino_f6"}


@pytest.mark.parametrize("name", STACK_NAMES)
def test_transformed_bytes_match_oracle_layout_sizes(name):
    for layer in stack(name):
        for half in (False, True):
            d = nnv.make_desc(layer, nnv.F16 if half else nnv.F32)
            for kind in range(6):
                if not nnv.nnv_kind_supported(d, kind):
                    assert nnv.nnv_transformed_bytes(d, kind) == 0
                    continue
                exp = OL.transformed_bytes(KNAME[kind], layer.k, layer.cg, layer.r, layer.s, half, layer.groups)
                assert nnv.nnv_transformed_bytes(d, kind) == exp, (layer.name, kind, half)


def test_winograd_size_ratio_unpadded():
    """alpha^2/9 growth of 3x3 weights (16/9, 4) when no padding is needed."""
    d = D(c=64, k=64)
    raw = 64 * 64 * 9 * 4
    assert nnv.nnv_transformed_bytes(d, nnv.WINO_F2) * 9 == raw * 16
    assert nnv.nnv_transformed_bytes(d, nnv.WINO_F4) * 9 == raw * 36
    assert nnv.nnv_transformed_bytes(d, nnv.WINO_F6) * 9 == raw * 64    # the 7.1x of the paper's 8x8-tile example
    assert nnv.nnv_transformed_bytes(d, nnv.IM2COL_GEMM) == raw


def test_cache_argument_and_file_errors_need_no_gpu(tmp_path):
    """The cache reader validates its arguments and the file header before it touches the device."""
    lib = nnv.load()
    d = D()
    p = str(tmp_path / "w.nnvc").encode()
    dev = ctypes.c_void_p(256)
    assert lib.nnv_cache_read(None, ctypes.byref(d), 1, dev, 0, None, None) == -1
    assert lib.nnv_cache_read(p, ctypes.byref(d), 9, dev, 0, None, None) == -7
    assert lib.nnv_cache_read(p, ctypes.byref(d), 4, dev, 0, None, None) == -3
    assert lib.nnv_cache_read(p, ctypes.byref(d), 1, ctypes.c_void_p(260), 0, None, None) == -5
    assert lib.nnv_cache_read(p, ctypes.byref(d), 1, dev, 0, None, None) == -8          # no such file
    assert lib.nnv_cache_write(None, ctypes.byref(d), 1, dev, None) == -1
    open(p, "wb").write(b"short")
    assert lib.nnv_cache_read(p, ctypes.byref(d), 1, dev, 0, None, None) == -9          # no header block
    open(p, "wb").write(b"\0" * 8192)
    assert lib.nnv_cache_read(p, ctypes.byref(d), 1, dev, 0, None, None) == -9          # wrong magic


def test_cold_stack_argument_errors_need_no_gpu():
    lib = nnv.load()
    assert lib.nnv_cold_stack(-1, None, None, None, None, None, None, None, 0, 1, None, None) == -7
    assert lib.nnv_cold_stack(0, None, None, None, None, None, None, None, 0, 1, None, None) == 0
    assert lib.nnv_cold_stack(1, None, None, None, None, None, None, None, 0, 1, None, None) == -1


def test_filter_size_limits_of_the_gemm_kind():
    """An 11x11 filter (121 taps) packs in float32; float16 fragments span 32 channels and stop at 64 taps."""
    assert nnv.nnv_kind_supported(D(c=3, h=224, w=224, k=64, r=11, s=11, stride_h=4, stride_w=4, pad_h=2, pad_w=2), 1)
    assert not nnv.nnv_kind_supported(D(c=3, h=224, w=224, k=64, r=11, s=11, stride_h=4, stride_w=4, pad_h=2, pad_w=2, dtype=1), 1)
    assert nnv.nnv_kind_supported(D(r=8, s=8, pad_h=4, pad_w=4, dtype=1), 1)
    assert not nnv.nnv_kind_supported(D(c=4, h=40, w=40, r=12, s=12), 1)
