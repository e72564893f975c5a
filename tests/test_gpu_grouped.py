"""nnv_conv_forward_grouped: many independent layers in one call.  Every output is compared with
the float64 oracle element by element; canaries around every output and around the workspace
catch writes outside them."""
import numpy as np
import pytest

from nnv_workloads import ConvLayer, stack, layer_tensors
from nnv_testlib import conv_tolerance, oracle_forward, applicable_kinds, KIND_NAMES
from oracle import cdirect

pytestmark = pytest.mark.gpu
PAD = 256


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2206_07446_amd as nnv
    assert torch.cuda.is_available(), "GPU tests need the HIP device"
    nnv.load()
    return nnv, torch


def Ly(name, c, h, w, k, r, stride, pad, groups=1, n=1):
    return ConvLayer(name, c, h, w, k, r, r, stride, pad, groups, n)


class Case:
    def __init__(self, nnv, torch, layer, kind, half, seed, bias=False):
        dev = torch.device("cuda:0")
        self.layer, self.kind, self.half = layer, kind, half
        self.w, self.x = layer_tensors(layer, seed)
        self.b = np.random.default_rng(seed + 7).standard_normal(layer.k) if bias else None
        self.desc = nnv.make_desc(layer, nnv.F16 if half else nnv.F32)
        wd = torch.from_numpy(self.w).to(dev)
        self.wt = wd if kind == nnv.DIRECT else torch.empty(nnv.nnv_transformed_bytes(self.desc, kind), dtype=torch.uint8, device=dev)
        nnv.nnv_transform_weights(self.desc, kind, wd, self.wt)
        self.xd = torch.from_numpy(self.x).to(dev)
        if half:
            self.xd = self.xd.half()
        self.bd = None if self.b is None else torch.from_numpy(self.b.astype(np.float32)).to(dev)
        self.numel = layer.n * layer.k * layer.p * layer.q
        self.esz = 2 if half else 4
        self.ybuf = torch.full((self.numel * self.esz + 2 * PAD,), 0x7F, dtype=torch.uint8, device=dev)
        self.y = self.ybuf[PAD:PAD + self.numel * self.esz]

    def result(self):
        yh = self.ybuf.cpu().numpy()
        assert (yh[:PAD] == 0x7F).all() and (yh[PAD + self.numel * self.esz:] == 0x7F).all(), f"{self.layer.name}: write outside y"
        out = yh[PAD:PAD + self.numel * self.esz].view(np.float16 if self.half else np.float32)
        l = self.layer
        return out.astype(np.float64).reshape(l.n, l.k, l.p, l.q)

    def reference(self, big=False):
        l = self.layer
        if big and not self.half:
            ref = cdirect.conv2d_direct_c(self.x, self.w, l.stride, l.pad, l.groups)
            return ref if self.b is None else ref + self.b.reshape(1, -1, 1, 1)
        return oracle_forward(l, self.half, self.w, self.x, self.b)


def run_grouped(nnv, torch, cases, relu=False, big=False):
    dev = torch.device("cuda:0")
    descs, kinds = [c.desc for c in cases], [c.kind for c in cases]
    need = nnv.nnv_conv_forward_grouped_workspace_bytes(descs, kinds)
    wsbuf = torch.full((need + 2 * PAD,), 0x5A, dtype=torch.uint8, device=dev)
    ws = wsbuf[PAD:PAD + need] if need else None
    bias = [c.bd for c in cases] if any(c.bd is not None for c in cases) else None
    print("grouped call:", [(c.layer.name, KIND_NAMES[c.kind], c.half) for c in cases], flush=True)
    nnv.nnv_conv_forward_grouped(descs, kinds, [c.xd for c in cases], [c.wt for c in cases], bias, [c.y for c in cases],
                                 ws, need, nnv.FORWARD_RELU if relu else 0)
    torch.cuda.synchronize()
    wh = wsbuf.cpu().numpy()
    assert (wh[:PAD] == 0x5A).all() and (wh[PAD + need:] == 0x5A).all(), "write outside the workspace"
    worst = 0.0
    for c in cases:
        got, ref = c.result(), c.reference(big)
        assert np.isfinite(got).all(), c.layer.name
        scale = np.abs(ref).max()
        if relu:
            ref = np.maximum(ref, 0.0)
            assert (got >= 0).all()
        err = np.abs(got - ref).max() / scale
        assert err <= conv_tolerance(c.kind, c.half), f"{c.layer.name} {KIND_NAMES[c.kind]} half={c.half}: rel err {err:.3e}"
        worst = max(worst, err)
    return worst


SMALL = [
    Ly("cfg1", 16, 32, 32, 16, 3, 1, 1),
    Ly("ragged", 37, 13, 19, 20, 3, 1, 1),
    Ly("batch2", 8, 9, 10, 24, 3, 1, 1, n=2),
    Ly("pad0", 12, 10, 10, 16, 3, 1, 0),
    Ly("tiny", 1, 3, 3, 1, 3, 1, 1),
    Ly("s2", 16, 15, 15, 32, 3, 2, 1),
    Ly("stem", 3, 32, 32, 64, 7, 2, 3),
    Ly("pw", 96, 14, 14, 24, 1, 1, 0),
    Ly("pw_s2", 64, 14, 14, 128, 1, 2, 0),
    Ly("pw_wide", 40, 7, 7, 1280, 1, 1, 0),
    Ly("pw_c1100", 1100, 5, 5, 40, 1, 1, 0),
    Ly("deep", 512, 7, 7, 64, 3, 1, 1),
    Ly("deep_k80", 300, 7, 7, 80, 3, 1, 1),                  # five panels: two per tile, last tile half empty
    Ly("k5", 6, 11, 9, 7, 5, 1, 2),
    Ly("k11", 3, 35, 35, 24, 11, 4, 2),
    Ly("k4x4", 20, 12, 12, 16, 4, 1, 2),
    Ly("batch3", 20, 11, 13, 40, 3, 1, 1, n=3),
    Ly("batch5_deep", 128, 7, 7, 64, 3, 1, 1, n=5),
    Ly("g3_pw", 240, 14, 14, 240, 1, 1, 0, groups=3),
    Ly("g3_pw_in", 24, 14, 14, 60, 1, 1, 0, groups=3),
    Ly("g32_3x3", 128, 14, 14, 128, 3, 1, 1, groups=32),
    Ly("g2_5x5", 96, 13, 13, 64, 5, 1, 2, groups=2),
    Ly("g4_s2_n2", 32, 11, 11, 48, 3, 2, 1, groups=4, n=2),
]


@pytest.mark.parametrize("half", [False, True], ids=["f32", "f16"])
def test_small_gemm_layers_in_one_call(env, half):
    """23 layers (more than one launch carries): every filter mode, ragged tiles, batches, groups, split reductions."""
    nnv, torch = env
    cases = [Case(nnv, torch, l, nnv.IM2COL_GEMM, half, 700 + i) for i, l in enumerate(SMALL + SMALL[:6])
             if nnv.IM2COL_GEMM in applicable_kinds(l, half)]
    assert len(cases) > 21
    run_grouped(nnv, torch, cases)


def test_bias_and_relu(env):
    nnv, torch = env
    for half in (False, True):
        cases = [Case(nnv, torch, l, nnv.IM2COL_GEMM, half, 800 + i, bias=(i % 3 != 0)) for i, l in enumerate(SMALL[:12])]
        run_grouped(nnv, torch, cases)
        run_grouped(nnv, torch, cases, relu=True)


def test_grouped_matches_layer_by_layer(env):
    """Same launches or not, the grouped call computes the same convolutions: against single calls
    the difference is float32 summation order only."""
    nnv, torch = env
    dev = torch.device("cuda:0")
    cases = [Case(nnv, torch, l, nnv.IM2COL_GEMM, False, 900 + i) for i, l in enumerate(SMALL)]
    run_grouped(nnv, torch, cases)
    for c in cases:
        y1 = torch.empty(c.numel, device=dev)
        nnv.nnv_conv_forward(c.desc, c.kind, c.xd, c.wt, None, y1, None)
        torch.cuda.synchronize()
        a, b = c.result().ravel(), y1.cpu().numpy().astype(np.float64)
        assert np.abs(a - b).max() <= 2e-5 * np.abs(b).max(), c.layer.name


def test_mixed_kinds_in_one_call(env):
    nnv, torch = env
    layers = [SMALL[0], SMALL[1], SMALL[5], SMALL[7], Ly("dw", 48, 15, 15, 48, 3, 2, 1, groups=48), SMALL[11]]
    kinds = [nnv.WINO_F4, nnv.IM2COL_GEMM, nnv.DIRECT, nnv.IM2COL_GEMM, nnv.DEPTHWISE, nnv.WINO_F2]
    cases = [Case(nnv, torch, l, k, False, 1000 + i) for i, (l, k) in enumerate(zip(layers, kinds))]
    run_grouped(nnv, torch, cases)
    # every kind of one layer, as the decision stage profiles them
    cases = [Case(nnv, torch, SMALL[1], k, False, 1100) for k in (0, 1, 2, 3, 5)]
    run_grouped(nnv, torch, cases)


@pytest.mark.parametrize("name,half", [("resnet18", False), ("mobilenetv2", False), ("resnet50", False), ("resnet50", True),
                                       ("resnet18", True), ("vgg16", True)])
def test_full_stacks_gemm_kind(env, name, half):
    """Whole stacks at full size, every layer the implicit GEMM can run, one grouped call.  In float16 the
    small stacks run items a quarter as long as the VGG-16-shaped one; all channels-last copies are one launch."""
    nnv, torch = env
    cases = [Case(nnv, torch, l, nnv.IM2COL_GEMM, half, 220607446 + 3000 + i)
             for i, l in enumerate(stack(name)) if l.groups == 1]
    worst = run_grouped(nnv, torch, cases, big=True)
    print(name, half, f"worst rel err {worst:.2e}")


WINO_SMALL = [
    Ly("cfg1", 16, 32, 32, 16, 3, 1, 1),
    Ly("ragged", 37, 13, 19, 20, 3, 1, 1),
    Ly("batch2", 8, 9, 10, 24, 3, 1, 1, n=2),
    Ly("pad0", 12, 10, 10, 16, 3, 1, 0),
    Ly("pad2", 4, 6, 7, 5, 3, 1, 2),
    Ly("tiny", 1, 3, 3, 1, 3, 1, 1),
    Ly("deep", 512, 7, 7, 64, 3, 1, 1),
    Ly("batch3", 20, 11, 13, 40, 3, 1, 1, n=3),
    Ly("batch5_deep", 128, 7, 7, 64, 3, 1, 1, n=5),
    Ly("wide_k", 24, 20, 18, 200, 3, 1, 1),
    Ly("one_k16", 40, 30, 30, 16, 3, 1, 1),              # a single 16-row panel: 16 x 16 GEMM tiles
    Ly("fz_ragged", 6, 90, 90, 24, 3, 1, 1),             # float32 F(2x2)/F(4x4): the fused single-kernel route, run on its own
]


@pytest.mark.parametrize("kind", [2, 3, 5], ids=["f2", "f4", "f6"])
@pytest.mark.parametrize("half", [False, True], ids=["f32", "f16"])
def test_winograd_layers_in_one_call(env, kind, half):
    nnv, torch = env
    layers = [l for l in WINO_SMALL + WINO_SMALL[:10] if kind in applicable_kinds(l, half)]
    if not layers:
        pytest.skip("F(6x6) exists in float32 only")
    cases = [Case(nnv, torch, l, kind, half, 1400 + i, bias=(i % 2 == 1)) for i, l in enumerate(layers)]
    assert half or len(cases) > 20          # more than one launch group carries
    run_grouped(nnv, torch, cases)
    run_grouped(nnv, torch, cases, relu=True)
    if not half:                            # against the single calls: float32 summation order only
        dev = torch.device("cuda:0")
        run_grouped(nnv, torch, cases)
        for c in cases:
            need = nnv.nnv_workspace_bytes(c.desc, kind)
            ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
            y1 = torch.empty(c.numel, device=dev)
            nnv.nnv_conv_forward(c.desc, kind, c.xd, c.wt, c.bd, y1, ws)
            torch.cuda.synchronize()
            a, b = c.result().ravel(), y1.cpu().numpy().astype(np.float64)
            assert np.abs(a - b).max() <= 0.1 * conv_tolerance(kind, False) * np.abs(b).max(), c.layer.name


@pytest.mark.parametrize("name,kind,half", [("resnet18", 2, False), ("resnet18", 3, False), ("resnet18", 5, False),
                                            ("vgg16", 3, False), ("resnet50", 3, True), ("resnet50", 2, True)])
def test_full_stacks_winograd(env, name, kind, half):
    nnv, torch = env
    cases = [Case(nnv, torch, l, kind, half, 220607446 + 4000 + i) for i, l in enumerate(stack(name)) if l.winograd_ok
             and kind in applicable_kinds(l, half)]
    worst = run_grouped(nnv, torch, cases, big=True)
    print(name, KIND_NAMES[kind], half, f"worst rel err {worst:.2e}")


DIRECT_DW = [
    Ly("cfg1", 16, 32, 32, 16, 3, 1, 1),
    Ly("ragged", 37, 13, 19, 20, 3, 1, 1),
    Ly("batch2", 8, 9, 10, 24, 3, 1, 1, n=2),
    Ly("tiny", 1, 3, 3, 4, 3, 1, 1),
    Ly("s2", 16, 15, 15, 32, 3, 2, 1),
    Ly("stem", 3, 32, 32, 64, 7, 2, 3),
    Ly("pw", 96, 14, 14, 24, 1, 1, 0),
    Ly("pw_s2", 64, 14, 14, 128, 1, 2, 0),
    Ly("pw_odd_c", 41, 7, 7, 16, 1, 1, 0),
    Ly("deep", 512, 7, 7, 64, 3, 1, 1),                      # 7x7 plane: the lane-grid variant
    Ly("plane5", 9, 5, 7, 8, 3, 1, 1),
    Ly("plane7_pad0", 9, 7, 7, 12, 3, 1, 0),
    Ly("k5", 6, 11, 9, 8, 5, 1, 2),
    Ly("batch3", 20, 11, 13, 40, 3, 1, 1, n=3),
    Ly("k_odd", 10, 9, 9, 7, 3, 1, 1),                       # K not a multiple of 4: runs on its own
    Ly("grp2", 8, 9, 9, 12, 3, 1, 1, groups=2),              # grouped: runs on its own
    Ly("dw_s1", 32, 14, 14, 32, 3, 1, 1, groups=32),
    Ly("dw_s2", 48, 15, 15, 48, 3, 2, 1, groups=48),
    Ly("dw_n2", 5, 7, 7, 5, 3, 1, 1, groups=5, n=2),
    Ly("dw5_s1", 40, 14, 14, 40, 5, 1, 2, groups=40),
    Ly("dw5_s2", 72, 15, 13, 72, 5, 2, 2, groups=72, n=2),
    Ly("dw_big", 96, 40, 40, 96, 3, 1, 1, groups=96),
]


@pytest.mark.parametrize("half", [False, True], ids=["f32", "f16"])
def test_direct_and_depthwise_layers_in_one_call(env, half):
    nnv, torch = env
    cases = [Case(nnv, torch, l, nnv.DIRECT, half, 1500 + i, bias=(i % 2 == 0)) for i, l in enumerate(DIRECT_DW + DIRECT_DW[:14])]
    cases += [Case(nnv, torch, l, nnv.DEPTHWISE, half, 1600 + i, bias=(i % 2 == 1)) for i, l in enumerate(DIRECT_DW) if l.is_depthwise]
    run_grouped(nnv, torch, cases)
    run_grouped(nnv, torch, cases, relu=True)
    dev = torch.device("cuda:0")
    run_grouped(nnv, torch, cases)
    for c in cases:                       # the same block code as the single launches; only the channel split differs
        y1 = torch.empty(c.numel, dtype=torch.float16 if half else torch.float32, device=dev)
        nnv.nnv_conv_forward(c.desc, c.kind, c.xd, c.wt, c.bd, y1, None)
        torch.cuda.synchronize()
        a, b = c.result().ravel(), y1.cpu().numpy().astype(np.float64)
        assert np.abs(a - b).max() <= (2e-3 if half else 2e-5) * np.abs(b).max(), c.layer.name


# float32 layers with K a multiple of 64 that run with the lanes along the output channels: 3x3 at stride 1
# (tiles of 2 rows x 7 or 14 columns) or 2 (one row), C a multiple of 4, taps of two channels at a time through
# LDS; 1x1 at stride 1 or 2, C a multiple of 16, taps of sixteen channels at a time; 7x7 (stride 2) with at
# most 4 channels, whole filters staged in LDS.  Pixels through LDS.
KLANE = [
    Ly("kl_w7", 8, 7, 7, 64, 3, 1, 1),                       # 7-wide tiles, last row pair half empty
    Ly("kl_w14", 12, 14, 14, 64, 3, 1, 1),                   # one tile per row pair: both edges in it
    Ly("kl_w28", 16, 6, 28, 128, 3, 1, 1),                   # two tiles per row pair, two blocks of output channels
    Ly("kl_w42", 4, 5, 42, 64, 3, 1, 1),                     # three tiles; one pair of channel pairs, odd H
    Ly("kl_deep", 256, 7, 7, 64, 3, 1, 1),                   # eight wavefronts per tile (one per 32 channels)
    Ly("kl_c128", 128, 4, 14, 64, 3, 1, 1),                  # four wavefronts per tile
    Ly("kl_c132", 132, 3, 14, 64, 3, 1, 1),                  # 33 channel groups: one wavefront per tile
    Ly("kl_h1", 4, 1, 14, 64, 3, 1, 1),
    Ly("kl_n2", 8, 7, 14, 128, 3, 1, 1, n=2),
    Ly("kl_w56", 64, 4, 56, 64, 3, 1, 1),                    # two wavefronts per tile
    Ly("kl_w15", 8, 9, 15, 64, 3, 1, 1),                     # Q = 15: a full tile and one column of a ragged one
    Ly("kl_p0", 8, 9, 16, 64, 3, 1, 0),                      # no padding: Q = 14, P = 7
    Ly("kl_p2", 4, 5, 10, 64, 3, 1, 2),                      # padding 2: Q = 12, P = 7
    Ly("other_c3", 3, 10, 28, 64, 3, 1, 1),                  # three channels: not covered
    Ly("ks_stem28", 3, 28, 28, 64, 7, 2, 3),                 # 7x7: filters staged in LDS; Q = 14
    Ly("ks_stem42", 3, 12, 42, 128, 7, 2, 3, n=2),           # Q = 21: a full and a ragged tile, two blocks of output channels
    Ly("ks_stem_c4", 4, 9, 30, 64, 7, 2, 2),                 # four channels (even filter length, odd LDS stride), pad 2, Q = 14
    Ly("ks_stem_c1", 1, 20, 20, 64, 7, 2, 0),                # one channel, no padding, Q = 7
    Ly("ks_w28", 16, 10, 28, 128, 3, 2, 1),                  # Q = 14
    Ly("ks_c128", 128, 6, 28, 64, 3, 2, 1),                  # four wavefronts per tile
    Ly("ks_deep", 256, 14, 14, 64, 3, 2, 1),                 # Q = 7: 7-wide tiles, eight wavefronts per tile
    Ly("ks_w56", 64, 6, 56, 64, 3, 2, 1),                    # Q = 28: two tiles per row, two wavefronts per tile
    Ly("ks_q13", 8, 7, 26, 64, 3, 2, 1, n=2),                # Q = 13: ragged tile
    Ly("ks_q21", 4, 5, 42, 64, 3, 2, 1),                     # Q = 21: three 7-wide tiles
    Ly("ks_q17_p0", 12, 9, 35, 64, 3, 2, 0),                 # no padding, Q = 17: a full and a ragged tile
    Ly("other_s2", 16, 15, 15, 32, 3, 2, 1),                 # not covered (K = 32): the pixel-lane kernel in the same call
    Ly("other_s2_c6", 6, 14, 14, 64, 3, 2, 1),               # not covered (C = 6)
    Ly("other_c6", 6, 14, 14, 64, 3, 1, 1),
    Ly("k1_s2", 64, 14, 14, 128, 1, 2, 0),                   # 1x1 (C a multiple of 16): Q = 7, 7-wide one-row tiles
    Ly("k1_s2_w28", 48, 9, 55, 64, 1, 2, 0),                 # Q = 28, P = 5; three groups of 16 channels
    Ly("k1_w7", 256, 7, 7, 64, 1, 1, 0),                     # stride 1: two-row tiles, two wavefronts per tile
    Ly("k1_w28", 32, 5, 28, 128, 1, 1, 0, n=2),              # two tiles per row pair, odd P
    Ly("k1_w15", 16, 4, 15, 64, 1, 1, 0),                    # ragged tile
    Ly("k1_deep", 1024, 7, 7, 64, 1, 1, 0),                  # eight wavefronts per tile
    Ly("other_1x1_c24", 24, 14, 14, 64, 1, 1, 0),            # not covered (C = 24)
    Ly("other_5x5", 4, 12, 12, 64, 5, 1, 2),
]


@pytest.mark.parametrize("half", [False, True], ids=["f32", "f16"])
def test_direct_output_channel_lanes(env, half):
    nnv, torch = env
    cases = [Case(nnv, torch, l, nnv.DIRECT, half, 1700 + i, bias=(i % 2 == 0)) for i, l in enumerate(KLANE)]
    run_grouped(nnv, torch, cases)
    run_grouped(nnv, torch, cases, relu=True)


@pytest.mark.parametrize("name,kind", [("resnet18", 0), ("mobilenetv2", 0), ("mobilenetv2", 4), ("efficientnet_b0", 4)])
def test_full_stacks_direct_and_depthwise(env, name, kind):
    nnv, torch = env
    cases = [Case(nnv, torch, l, kind, False, 220607446 + 5000 + i) for i, l in enumerate(stack(name))
             if kind in applicable_kinds(l, False)]
    worst = run_grouped(nnv, torch, cases, big=True)
    print(name, KIND_NAMES[kind], f"worst rel err {worst:.2e}")


def test_graph_replay(env):
    """The grouped call captured into a HIP graph and replayed, outputs and workspace scrambled in between."""
    nnv, torch = env
    dev = torch.device("cuda:0")
    cases = [Case(nnv, torch, l, nnv.IM2COL_GEMM, False, 1200 + i) for i, l in enumerate(SMALL[:16])]
    cases += [Case(nnv, torch, l, nnv.WINO_F4, False, 1250 + i) for i, l in enumerate(WINO_SMALL[:8])]
    # direct layers of all three launch classes
    cases += [Case(nnv, torch, l, nnv.DIRECT, False, 1270 + i) for i, l in enumerate(DIRECT_DW[:12] + KLANE[:6])]
    cases += [Case(nnv, torch, l, nnv.DEPTHWISE, False, 1290 + i) for i, l in enumerate(DIRECT_DW) if l.is_depthwise]
    descs, kinds = [c.desc for c in cases], [c.kind for c in cases]
    need = nnv.nnv_conv_forward_grouped_workspace_bytes(descs, kinds)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    args = (descs, kinds, [c.xd for c in cases], [c.wt for c in cases], None, [c.y for c in cases], ws, need)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        nnv.nnv_conv_forward_grouped(*args)
    torch.cuda.synchronize()
    expect = [c.y.clone() for c in cases]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        nnv.nnv_conv_forward_grouped(*args)
    for rep in range(3):
        for c in cases:
            c.y.fill_(0x33)
        ws.fill_(0xFF)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for c, e in zip(cases, expect):
            assert torch.equal(c.y, e), (rep, c.layer.name)
    for c in cases:
        ref = c.reference()
        assert np.abs(c.result() - ref).max() <= conv_tolerance(c.kind, False) * np.abs(ref).max()


def test_argument_errors(env):
    nnv, torch = env
    dev = torch.device("cuda:0")
    # four layers: enough for the work-item launch (fewer would run by themselves, without a workspace)
    cases = [Case(nnv, torch, l, nnv.IM2COL_GEMM, False, 1300 + i) for i, l in enumerate((SMALL[11], SMALL[1], SMALL[2], SMALL[3]))]
    descs, kinds = [c.desc for c in cases], [c.kind for c in cases]
    xs, wts, ys = [c.xd for c in cases], [c.wt for c in cases], [c.y for c in cases]
    need = nnv.nnv_conv_forward_grouped_workspace_bytes(descs, kinds)
    assert need > 0                                     # the 512-channel layer is split
    small = torch.empty(need - 256, dtype=torch.uint8, device=dev)
    with pytest.raises(nnv.NnvError) as e:
        nnv.nnv_conv_forward_grouped(descs, kinds, xs, wts, None, ys, small)
    assert e.value.status == -4
    with pytest.raises(nnv.NnvError) as e:
        nnv.nnv_conv_forward_grouped(descs, kinds, xs, wts, None, ys, None, 0)
    assert e.value.status == -1
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    with pytest.raises(nnv.NnvError) as e:
        nnv.nnv_conv_forward_grouped(descs, [nnv.DEPTHWISE, 1, 1, 1], xs, wts, None, ys, ws)
    assert e.value.status == -3
    with pytest.raises(nnv.NnvError) as e:
        nnv.nnv_conv_forward_grouped(descs, kinds, xs, wts, None, ys, ws, flags=2)
    assert e.value.status == -7
    with pytest.raises(nnv.NnvError) as e:
        nnv.nnv_conv_forward_grouped(descs, kinds, [xs[0], None, xs[2], xs[3]], wts, None, ys, ws)
    assert e.value.status == -1
    torch.cuda.synchronize()
    for c in cases:                                     # nothing was launched by the refused calls
        assert (c.ybuf == 0x7F).all()
    nnv.nnv_conv_forward_grouped([], [], [], [], None, [], None)
