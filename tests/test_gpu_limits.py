"""Largest buffers the library accepts: activations just below 2 GiB (the kernels address every
buffer with 32-bit byte offsets) for the kinds without a workspace, and just below 1 GiB for the
fused Winograd route.  Outputs are compared with the float64 definition on sampled positions
(corners, borders, the last rows and random interior points); one step beyond the limit is refused."""
import numpy as np
import pytest

from nnv_workloads import ConvLayer
from nnv_testlib import conv_tolerance, KIND_NAMES
from oracle.direct import conv2d_at

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2206_07446_amd as nnv
    assert torch.cuda.is_available(), "GPU tests need the HIP device"
    nnv.load()
    return nnv, torch


def sample_positions(layer, rng, n_random=1500):
    P, Q, K = layer.p, layer.q, layer.k
    ps = [0, 1, P // 2, P - 2, P - 1]
    qs = [0, 1, Q // 2, Q - 2, Q - 1]
    pos = [(k, p, q) for k in (0, K - 1) for p in ps for q in qs]
    pos += [(int(rng.integers(K)), int(rng.integers(P)), int(rng.integers(Q))) for _ in range(n_random)]
    return pos


def run_and_check(nnv, torch, layer, kinds, seed):
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(seed)
    x = rng.random((layer.n, layer.c, layer.h, layer.w), dtype=np.float32) * 2 - 1
    w = (rng.standard_normal((layer.k, layer.c // layer.groups, layer.r, layer.s)) *
         np.sqrt(2.0 / (layer.c // layer.groups * layer.r * layer.s))).astype(np.float32)
    pos = sample_positions(layer, rng)
    ref = conv2d_at(x, w, [(0, k, p, q) for k, p, q in pos], layer.stride, layer.pad, layer.groups)
    scale = np.abs(ref).max()
    xd, wd = torch.from_numpy(x).to(dev), torch.from_numpy(w).to(dev)
    desc = nnv.make_desc(layer, nnv.F32)
    idx = tuple(np.array(v) for v in zip(*pos))
    for kind in kinds:
        print(f"case {layer} kind={KIND_NAMES[kind]}", flush=True)
        assert nnv.nnv_kind_supported(desc, kind) == 1
        wt = wd if kind == nnv.DIRECT else torch.empty(nnv.nnv_transformed_bytes(desc, kind), dtype=torch.uint8, device=dev)
        ws_bytes = nnv.nnv_workspace_bytes(desc, kind)
        ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
        y = torch.full((layer.k, layer.p, layer.q), float("nan"), dtype=torch.float32, device=dev)
        nnv.nnv_transform_weights(desc, kind, wd, wt)
        nnv.nnv_conv_forward(desc, kind, xd, wt, None, y, ws)
        torch.cuda.synchronize()
        got = y.cpu().numpy()
        assert np.isfinite(got).all()
        err = np.abs(got[idx].astype(np.float64) - ref).max() / scale
        assert err <= conv_tolerance(kind, False), f"{KIND_NAMES[kind]}: rel err {err:.3e}"
        del y, ws, got


def test_activations_just_below_2_gib(env):
    nnv, torch = env
    # x and y: 32 x 4095 x 4095 float32 = 2 146 435 200 bytes (limit 2 147 483 648)
    layer = ConvLayer("limit2g", 32, 4095, 4095, 32, 3, 3, 1, 1)
    assert 2 ** 31 - 2 ** 21 < layer.c * layer.h * layer.w * 4 < 2 ** 31
    run_and_check(nnv, torch, layer, (nnv.DIRECT, nnv.IM2COL_GEMM), seed=91)
    # Winograd would need V and M beyond 2 GiB here and x is too large for the fused route
    desc = nnv.make_desc(layer, nnv.F32)
    assert nnv.nnv_kind_supported(desc, nnv.WINO_F2) == 0 and nnv.nnv_kind_supported(desc, nnv.WINO_F4) == 0
    # one more row and column: exactly 2^31 bytes, refused by every kind
    over = ConvLayer("over2g", 32, 4096, 4096, 32, 3, 3, 1, 1)
    od = nnv.make_desc(over, nnv.F32)
    assert all(nnv.nnv_kind_supported(od, k) <= 0 for k in (nnv.DIRECT, nnv.IM2COL_GEMM, nnv.WINO_F2))


def test_depthwise_just_below_2_gib(env):
    nnv, torch = env
    layer = ConvLayer("limit2g_dw", 32, 4095, 4095, 32, 3, 3, 1, 1, 32)
    run_and_check(nnv, torch, layer, (nnv.DEPTHWISE, nnv.DIRECT), seed=92)


def test_fused_winograd_just_below_1_gib(env):
    nnv, torch = env
    # x and y: 16 x 4095 x 4095 float32 = 1 073 217 600 bytes (the fused route takes x below 2^30)
    layer = ConvLayer("limit1g", 16, 4095, 4095, 16, 3, 3, 1, 1)
    desc = nnv.make_desc(layer, nnv.F32)
    assert 2 ** 30 - 2 ** 20 < layer.c * layer.h * layer.w * 4 < 2 ** 30
    for kind in (nnv.WINO_F2, nnv.WINO_F4):
        assert nnv.nnv_workspace_bytes(desc, kind) == 0
    run_and_check(nnv, torch, layer, (nnv.WINO_F2, nnv.WINO_F4), seed=93)


def test_winograd_workspace_just_below_2_gib(env):
    nnv, torch = env
    # three-kernel F(4x4) (144 output channels: not the fused route): V + M = 2 143 641 600 bytes
    layer = ConvLayer("ws2g", 16, 1220, 1220, 144, 3, 3, 1, 1)
    desc = nnv.make_desc(layer, nnv.F32)
    assert 2 ** 31 - 2 ** 23 < nnv.nnv_workspace_bytes(desc, nnv.WINO_F4) < 2 ** 31
    # F(2x2) has four times the tiles and would need more than 2 GiB of V and M; F(6x6) needs 1.7 GB
    assert nnv.nnv_kind_supported(desc, nnv.WINO_F2) == 0
    run_and_check(nnv, torch, layer, (nnv.WINO_F4, nnv.WINO_F6), seed=94)
