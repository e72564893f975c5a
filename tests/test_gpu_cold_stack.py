"""GPU tests of the pipelined cold pass (Section 3.1.3): transforming stage s + 1 on one stream
while stage s executes on another gives, bit for bit, what the same launches give one after
the other; also when the pass is captured into a HIP graph and replayed."""
import numpy as np
import pytest

from nnv_workloads import stack, layer_tensors
from nnv_testlib import conv_tolerance, KIND_NAMES
from oracle import cdirect

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2206_07446_amd as nnv
    assert torch.cuda.is_available(), "GPU tests need the HIP device"
    nnv.load()
    return nnv, torch


def build_stack(nnv, torch, name, pick):
    dev = torch.device("cuda:0")
    descs, kinds, ws, xs, raw = [], [], 16, [], []
    for i, layer in enumerate(stack(name)):
        d = nnv.make_desc(layer)
        k = pick(i, layer)
        assert nnv.nnv_kind_supported(d, k)
        w, x = layer_tensors(layer, 4000 + i)
        descs.append(d); kinds.append(k)
        raw.append(torch.from_numpy(w).to(dev)); xs.append(torch.from_numpy(x).to(dev))
        ws = max(ws, nnv.nnv_workspace_bytes(d, k))
    def outputs():
        wt = [torch.zeros(max(16, nnv.nnv_transformed_bytes(d, k)), dtype=torch.uint8, device=dev) for d, k in zip(descs, kinds)]
        ys = [torch.zeros(l.n * l.k * l.p * l.q, device=dev) for l in stack(name)]
        return wt, ys
    return descs, kinds, raw, xs, torch.empty(ws, dtype=torch.uint8, device=dev), outputs


def mixed(i, layer):
    if layer.is_depthwise:
        return 4
    if layer.winograd_ok:
        return (1, 2, 3, 5)[i % 4]
    return 1 if i % 3 else 0


def reference(nnv, torch, descs, kinds, raw, xs, ws, outputs):
    wt, ys = outputs()
    for d, k, w, t, x, y in zip(descs, kinds, raw, wt, xs, ys):
        nnv.nnv_transform_weights(d, k, w, t)
        nnv.nnv_conv_forward(d, k, x, t, None, y, ws)
    torch.cuda.synchronize()
    return wt, ys


@pytest.mark.parametrize("name", ["resnet18", "mobilenetv2"])
@pytest.mark.parametrize("stage", [1, 3, 0])
def test_pipelined_equals_layer_by_layer(env, name, stage):
    nnv, torch = env
    descs, kinds, raw, xs, ws, outputs = build_stack(nnv, torch, name, mixed)
    wt0, ys0 = reference(nnv, torch, descs, kinds, raw, xs, ws, outputs)
    s_exec, s_tx = torch.cuda.Stream(), torch.cuda.Stream()
    for tx_stream in (None, s_tx):
        wt, ys = outputs()
        torch.cuda.synchronize()
        nnv.nnv_cold_stack(descs, kinds, raw, wt, xs, ys, ws, stage, s_exec, tx_stream)
        s_exec.synchronize()          # stream_exec alone orders the whole pass
        for a, b in zip(wt + ys, wt0 + ys0):
            assert torch.equal(a, b)


def test_captured_pass_replays(env):
    nnv, torch = env
    descs, kinds, raw, xs, ws, outputs = build_stack(nnv, torch, "resnet18", mixed)
    wt0, ys0 = reference(nnv, torch, descs, kinds, raw, xs, ws, outputs)
    wt, ys = outputs()
    s_exec, s_tx = torch.cuda.Stream(), torch.cuda.Stream()
    nnv.nnv_cold_stack(descs, kinds, raw, wt, xs, ys, ws, 2, s_exec, s_tx)      # warm-up outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s_exec):
        nnv.nnv_cold_stack(descs, kinds, raw, wt, xs, ys, ws, 2, s_exec, s_tx)
    for rep in range(3):
        for t in wt + ys:
            t.zero_()                  # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for a, b in zip(wt + ys, wt0 + ys0):
            assert torch.equal(a, b), rep
    # the outputs of the last replay (two streams, graph replay) against the float64 definition
    for i, (layer, kind, y) in enumerate(zip(stack("resnet18"), kinds, ys)):
        w, x = layer_tensors(layer, 4000 + i)
        ref = cdirect.conv2d_direct_c(x, w, layer.stride, layer.pad, layer.groups)
        got = y.cpu().numpy().astype(np.float64).reshape(ref.shape)
        err = np.abs(got - ref).max() / np.abs(ref).max()
        assert err <= conv_tolerance(kind, False), f"{layer.name} {KIND_NAMES[kind]}: rel err {err:.3e}"


def test_pipelined_mobilenetv2_against_the_oracle(env):
    """Two-stream pass over the MobileNetV2-shaped stack (depthwise, pointwise GEMM, direct stem),
    stage size 3, every output against the float64 definition."""
    nnv, torch = env
    descs, kinds, raw, xs, ws, outputs = build_stack(nnv, torch, "mobilenetv2", mixed)
    wt, ys = outputs()
    s_exec, s_tx = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    nnv.nnv_cold_stack(descs, kinds, raw, wt, xs, ys, ws, 3, s_exec, s_tx)
    s_exec.synchronize()
    for i, (layer, kind, y) in enumerate(zip(stack("mobilenetv2"), kinds, ys)):
        w, x = layer_tensors(layer, 4000 + i)
        ref = cdirect.conv2d_direct_c(x, w, layer.stride, layer.pad, layer.groups)
        got = y.cpu().numpy().astype(np.float64).reshape(ref.shape)
        err = np.abs(got - ref).max() / np.abs(ref).max()
        assert err <= conv_tolerance(kind, False), f"{layer.name} {KIND_NAMES[kind]}: rel err {err:.3e}"


def test_argument_errors(env):
    nnv, torch = env
    descs, kinds, raw, xs, ws, outputs = build_stack(nnv, torch, "resnet18", lambda i, l: 3 if l.winograd_ok else 1)
    wt, ys = outputs()
    small = torch.empty(16, dtype=torch.uint8, device=ws.device)
    with pytest.raises(nnv.NnvError) as e:
        nnv.nnv_cold_stack(descs, kinds, raw, wt, xs, ys, small, 1)
    assert e.value.status == -4
    bad = list(kinds); bad[0] = 3      # the stem is not a Winograd layer
    with pytest.raises(nnv.NnvError) as e:
        nnv.nnv_cold_stack(descs, bad, raw, wt, xs, ys, ws, 1)
    assert e.value.status == -3
    nnv.nnv_cold_stack([], [], [], [], [], [], None, 1)       # empty list: nothing to do
