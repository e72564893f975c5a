"""Parity in the launch configuration that bench.py times: the ResNet-18-shaped stack at full
size, every (layer, kind) pair of the step, the whole transformation as ONE grouped launch, the
forward pass of each kind as ONE grouped call (nnv_conv_forward_grouped) with one shared
workspace, issued eagerly call after call as bench.py does.  Before that the five phases are also
captured into HIP graphs and replayed twice.  All destinations are overwritten before every pass,
so a pass that did no work cannot pass; every transformed buffer and every output of the last
(eager) pass is compared with the oracle."""
import numpy as np
import pytest

import bench
from nnv_workloads import stack, layer_tensors
from nnv_testlib import oracle_transformed, conv_tolerance, KIND_NAMES
from oracle import cdirect
from test_gpu_transform import check_wino_u

pytestmark = pytest.mark.gpu


def test_step_as_timed_matches_oracle():
    import torch
    import paper_2206_07446_amd as nnv
    assert torch.cuda.is_available(), "GPU tests need the HIP device"
    nnv.load()
    dev = torch.device("cuda:0")
    layers = stack("resnet18")
    pairs, host = [], {}
    for i, layer in enumerate(layers):
        w, x = layer_tensors(layer, 220607446 + 2000 + i)            # the seeds bench.py uses
        host[layer.name] = (w, x)
        wd, xd = torch.from_numpy(w).to(dev), torch.from_numpy(x).to(dev)
        for kind in bench.applicable_kinds(nnv, layer):
            pairs.append(bench.Pair(nnv, torch, layer, kind, wd, xd, dev))
    assert len(pairs) == 66
    descs, kinds = [p.desc for p in pairs], [p.kind for p in pairs]
    srcs, dsts = [p.w_raw for p in pairs], [p.w_tx for p in pairs]
    step_kinds = (nnv.DIRECT, nnv.IM2COL_GEMM, nnv.WINO_F2, nnv.WINO_F4)
    by_kind = {k: [p for p in pairs if p.kind == k] for k in step_kinds}
    need = max(nnv.nnv_conv_forward_grouped_workspace_bytes([p.desc for p in sel], [p.kind for p in sel])
               for sel in by_kind.values())
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)

    def transform_all():
        nnv.nnv_transform_weights_grouped(descs, kinds, srcs, dsts)

    def forward_kind(kind):
        bench.grouped_forward(nnv, by_kind[kind], ws)

    def scramble():
        for p in pairs:
            if p.kind != nnv.DIRECT:
                p.w_tx.fill_(0x7F)
            p.y.fill_(float("nan"))
        ws.fill_(0xFF)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        transform_all()
        for kind in step_kinds:
            forward_kind(kind)
    torch.cuda.synchronize()
    graphs = []
    for fn in [transform_all] + [(lambda k=k: forward_kind(k)) for k in step_kinds]:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            fn()
        graphs.append(g)
    for _ in range(2):
        scramble()
        torch.cuda.synchronize()
        for g in graphs:
            g.replay()
        torch.cuda.synchronize()
    assert all(torch.isfinite(p.y).all() for p in pairs), "a replayed phase left outputs unwritten"
    scramble()
    torch.cuda.synchronize()
    transform_all()                      # the step as bench.py issues it
    for kind in step_kinds:
        forward_kind(kind)
    torch.cuda.synchronize()

    refs = {}
    for p in pairs:
        w, x = host[p.layer.name]
        tag = f"{p.layer.name} {KIND_NAMES[p.kind]}"
        print("check", tag, flush=True)
        # transformed weights
        if p.kind == nnv.IM2COL_GEMM:
            exp, _ = oracle_transformed(w, p.kind, False, p.layer.groups)
            got = p.w_tx.cpu().numpy().view(np.float32)
            assert np.array_equal(got.view(np.uint32), exp.reshape(-1).view(np.uint32)), tag
        elif p.kind in (nnv.WINO_F2, nnv.WINO_F4):
            exp64, bound = oracle_transformed(w, p.kind, False)
            got = p.w_tx.cpu().numpy().view(np.float32).reshape(exp64.shape)
            check_wino_u(got, exp64, bound, False)
        # outputs
        if p.layer.name not in refs:
            refs[p.layer.name] = cdirect.conv2d_direct_c(x, w, p.layer.stride, p.layer.pad, p.layer.groups)
        ref = refs[p.layer.name]
        y = p.y.cpu().numpy().astype(np.float64).reshape(ref.shape)
        assert np.isfinite(y).all(), tag
        err = np.abs(y - ref).max() / np.abs(ref).max()
        assert err <= conv_tolerance(p.kind, False), f"{tag}: rel err {err:.3e}"
