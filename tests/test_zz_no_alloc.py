"""nnv_conv_forward_static, the entry point for callers that cannot allocate: its kernels take
the library's static device array as their workspace.  Its output must equal, bit for bit,
what nnv_conv_forward writes with a caller-supplied workspace (same kernels, same launch
shapes), on calls in a row that share the array, the later ones with smaller inputs; the
results are also held against the float64 oracle."""
import numpy as np
import pytest

from nnv_workloads import ConvLayer, layer_tensors
from nnv_testlib import conv_tolerance, oracle_forward, KIND_NAMES

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2206_07446_amd as nnv
    assert torch.cuda.is_available(), "GPU tests need the HIP device"
    nnv.load()
    return nnv, torch


def Ly(name, c, h, w, k, r=3, stride=1, pad=1):
    return ConvLayer(name, c, h, w, k, r, r, stride, pad, 1, 1)


def run_both(nnv, torch, layer, kind, half, seed):
    dev = torch.device("cuda:0")
    print(f"case {layer} kind={KIND_NAMES[kind]} half={half}", flush=True)
    w, x = layer_tensors(layer, seed)
    desc = nnv.make_desc(layer, nnv.F16 if half else nnv.F32)
    wd = torch.from_numpy(w).to(dev)
    xd = torch.from_numpy(x).to(dev)
    if half:
        xd = xd.half()
    wt = torch.empty(max(16, nnv.nnv_transformed_bytes(desc, kind)), dtype=torch.uint8, device=dev)
    nnv.nnv_transform_weights(desc, kind, wd, wt)
    need = nnv.nnv_workspace_bytes(desc, kind)
    ws = torch.full((max(need, 16),), 0x5A, dtype=torch.uint8, device=dev)
    dt = torch.float16 if half else torch.float32
    y_ws = torch.full((layer.n, layer.k, layer.p, layer.q), float("nan"), dtype=dt, device=dev)
    y_st = torch.full_like(y_ws, float("nan"))
    nnv.nnv_conv_forward(desc, kind, xd, wt, None, y_ws, ws)
    nnv.nnv_conv_forward_static(desc, kind, xd, wt, None, y_st)
    torch.cuda.synchronize()
    assert torch.equal(y_ws.view(torch.uint8), y_st.view(torch.uint8)), "static-scratch output differs from the workspace route"
    ref = oracle_forward(layer, half, w, x)
    got = y_st.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    err = np.abs(got - ref).max() / np.abs(ref).max()
    assert err <= conv_tolerance(kind, half), f"rel err {err:.3e}"
    return need


def test_two_calls_in_a_row_second_smaller(env):
    nnv, torch = env
    big = Ly("static_big", 64, 56, 56, 64)
    small = Ly("static_small", 37, 13, 19, 20)
    for kind in (nnv.WINO_F4, nnv.WINO_F2, nnv.WINO_F6):
        assert run_both(nnv, torch, big, kind, False, seed=61) > 0          # uses the scratch array (V and M)
        assert run_both(nnv, torch, small, kind, False, seed=62) > 0        # smaller: stale contents beyond it
    # float16: Winograd, and the channel-last copy of the implicit GEMM
    for kind in (nnv.WINO_F4, nnv.IM2COL_GEMM):
        assert run_both(nnv, torch, big, kind, True, seed=63) > 0
        assert run_both(nnv, torch, small, kind, True, seed=64) > 0
    # kinds without scratch go through the same entry point
    for kind in (nnv.DIRECT, nnv.IM2COL_GEMM):
        assert run_both(nnv, torch, small, kind, False, seed=65) == 0


def test_sizes_beyond_the_static_array_are_refused(env):
    nnv, torch = env
    dev = torch.device("cuda:0")
    layer = Ly("static_too_big", 64, 224, 224, 64)
    desc = nnv.make_desc(layer, nnv.F16)          # float16 F(2x2): V and M take 77 MB, the array holds 64 MiB
    assert nnv.nnv_workspace_bytes(desc, nnv.WINO_F2) > nnv.STATIC_SCRATCH_BYTES
    x = torch.zeros(layer.c * layer.h * layer.w, dtype=torch.float16, device=dev)
    wt = torch.zeros(nnv.nnv_transformed_bytes(desc, nnv.WINO_F2), dtype=torch.uint8, device=dev)
    y = torch.full((layer.k * layer.p * layer.q,), 7.0, dtype=torch.float16, device=dev)
    with pytest.raises(nnv.NnvError) as e:
        nnv.nnv_conv_forward_static(desc, nnv.WINO_F2, x, wt, None, y)
    assert e.value.status == -4
    torch.cuda.synchronize()
    assert (y == 7.0).all()                                                 # nothing was launched
    with pytest.raises(nnv.NnvError) as e:
        nnv.nnv_conv_forward_static(desc, nnv.DEPTHWISE, x, wt, None, y)
    assert e.value.status == -3
