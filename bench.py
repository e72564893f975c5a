#!/usr/bin/env python3
"""Benchmark of the conv hot path: cold weight transformation + convolution of a whole
ResNet-18-shaped conv stack (batch 1, float32, 224x224 input) on one MI355X.

One step = every layer of the stack through every kernel alternative that can run it
(direct, im2col GEMM, Winograd F(2x2) and F(4x4)): first the weight transformations of all
(layer, kind) pairs from raw OIHW weights (one grouped launch), then, per kind, the
convolutions of all layers of the stack from their transformed weights (one grouped call per
kind: the layers of a stack are independent here, each has its own input).  Inputs and raw
weights are synthetic (seeded) and resident in HBM before the timed region.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X HBM3E
MFMA_F32_PEAK_TFLOPS = 157.3  # dense float32 matrix-core peak
MFMA_F16_PEAK_TFLOPS = 2500.0
VALU_F32_PEAK_TFLOPS = 157.3  # float32 vector peak (packed FMA; plain FMA, as compiled here, tops out at 78.6)

# HBM bytes per step and phase, (read MB, written MB), from the two `rocprofv3 --pmc` runs of
# `bench.py --counter-pass` summarised in profiles/bench_resnet18_hbm_traffic.md (counter values scaled
# by what the same counters read for the plain copy kernel).  They describe the kernel sources with
# the digest below; once a source file changes, `traffic` is reported as null until the counters
# are taken again.
MEASURED_TRAFFIC = {
    "csrc_sha256_16": "9eb774670b804f0b",
    "MB_per_step": {
        "transform": (44.9, 262.9),
        "direct": (77.7, 10.2),
        "im2col_gemm": (97.4, 23.0),
        "wino_f2": (137.8, 50.7),
        "wino_f4": (198.3, 38.4),
    },
}

KIND_LABEL = {0: "direct", 1: "im2col_gemm", 2: "wino_f2", 3: "wino_f4", 4: "depthwise", 5: "wino_f6"}
# kernels a grouped forward call of one kind launches for a stack (one launch group)
PHASE_KERNELS = {
    "transform": "transform_kernel (grouped weight transformation, all kinds)",
    "direct": "direct_conv_many_klane_kernel<float> (direct convolution of all layers in one launch, lanes along the output channels, vector ALU)",
    "im2col_gemm": "gemm_items_kernel + gemm_reduce_kernel (implicit GEMM work items of all layers, float32 MFMA)",
    "wino_f2": "wino_f2: wino_input_many + wino_gemm_many (float32 MFMA) + wino_output_many",
    "wino_f4": "wino_f4: wino_input_many + wino_gemm_many (float32 MFMA) + wino_output_many",
}
PHASE_LAUNCHES = {"transform": 1, "direct": 1, "im2col_gemm": 2, "wino_f2": 3, "wino_f4": 3}


def csrc_digest():
    import glob
    import hashlib
    h = hashlib.sha256()
    files = [f for pat in ("*.hip", "*.h") for f in glob.glob(os.path.join(ROOT, "paper_2206_07446_amd", "csrc", pat))]
    for f in sorted(files):      # kernels, their launch heuristics and shared headers; not the host-only .cpp files
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def applicable_kinds(nnv, layer):
    """The kinds of the timed step (F(6x6) and float16 are measured beside it)."""
    kinds = [nnv.DIRECT]
    if layer.groups == 1:
        kinds.append(nnv.IM2COL_GEMM)
        if layer.winograd_ok:
            kinds += [nnv.WINO_F2, nnv.WINO_F4]
    if layer.is_depthwise:
        kinds.append(nnv.DEPTHWISE)
    return kinds


class Pair:
    """One (layer, kind): device buffers and the algorithmic traffic/work it stands for."""

    def __init__(self, nnv, torch, layer, kind, w_raw, x, dev, dtype=0):
        self.layer, self.kind = layer, kind
        self.desc = nnv.make_desc(layer, dtype)
        self.w_raw, self.x = w_raw, x
        self.tx_bytes = nnv.nnv_transformed_bytes(self.desc, kind)
        # DIRECT executes from the raw layout: its transformed weights alias the raw ones (no work)
        self.w_tx = w_raw if kind == nnv.DIRECT else torch.empty(self.tx_bytes, dtype=torch.uint8, device=dev)
        self.ws_bytes = nnv.nnv_workspace_bytes(self.desc, kind)
        esz = 2 if dtype == nnv.F16 else 4
        self.y = torch.empty(layer.n * layer.k * layer.p * layer.q, dtype=torch.float16 if esz == 2 else torch.float32,
                             device=dev)
        self.raw_bytes = layer.params * 4
        self.transform_bytes = 0 if kind == nnv.DIRECT else self.raw_bytes + self.tx_bytes
        if kind in (nnv.WINO_F2, nnv.WINO_F4, nnv.WINO_F6):
            m = {nnv.WINO_F2: 2, nnv.WINO_F4: 4, nnv.WINO_F6: 6}[kind]
            tiles = layer.n * -(-layer.p // m) * -(-layer.q // m)
            self.flops = 2.0 * (m + 2) ** 2 * layer.k * layer.c * tiles
        else:
            self.flops = 2.0 * layer.macs
        self.direct_flops = 2.0 * layer.macs
        self.forward_bytes = esz * (layer.n * layer.c * layer.h * layer.w + layer.n * layer.k * layer.p * layer.q) \
            + self.tx_bytes


def cpu_baseline(layers, nnv, budget_s=12.0):
    """The oracle as it stands (float64 C direct convolution on all host cores; numpy weight
    transforms and numpy reference Winograd) timed over whole passes of the same step, every
    (layer, kind) pair, until about budget_s seconds of CPU work are done."""
    from nnv_workloads import layer_tensors
    from oracle import cdirect, layouts as OL, winograd as OW
    data = [layer_tensors(layer, 220607446 + 2000 + i) for i, layer in enumerate(layers)]
    passes, t_total, pairs_done = 0, 0.0, 0
    n_pairs = sum(len(applicable_kinds(nnv, l)) for l in layers)
    while t_total < budget_s and passes < 3:
        for layer, (w, x) in zip(layers, data):
            for kind in applicable_kinds(nnv, layer):
                t0 = time.perf_counter()
                if kind == nnv.IM2COL_GEMM:
                    OL.pack_gemm(w, False)
                elif kind in (nnv.WINO_F2, nnv.WINO_F4):
                    var = "F2" if kind == nnv.WINO_F2 else "F4"
                    OL.pack_wino(OW.transform_weights(w, var), False)
                if kind in (nnv.WINO_F2, nnv.WINO_F4):
                    OW.conv2d_winograd(x, w, var, layer.pad)
                else:
                    cdirect.conv2d_direct_c(x, w, layer.stride, layer.pad, layer.groups)
                t_total += time.perf_counter() - t0
                pairs_done += 1
        passes += 1
    return {"value": round(t_total * 1e3 / passes, 1), "unit": "ms", "cores": cdirect.threads(), "kind": "oracle",
            "sample": f"{passes} whole pass(es) of the same step ({n_pairs} layer-kind pairs of the ResNet-18-shaped "
                      f"stack: oracle weight transform + float64 forward), {t_total:.1f} s of CPU work; the C direct "
                      f"convolution uses all cores, the numpy transforms and reference Winograd one"}


def graph_ms(torch, np, side, fn, reps=10, before=None, calls=1):
    """Median time of fn's launches, captured on `side` into a HIP graph and replayed; `before`
    (if given) runs ahead of every timed replay, outside the event pair.  With calls > 1 the graph
    holds that many calls of fn back to back and the time is per call: a replay has a fixed cost
    of 20-25 us between its two events, which would otherwise be most of a small workload's time."""
    with torch.cuda.stream(side):
        fn()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        for _ in range(calls):
            fn()
    g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ts = []
    for _ in range(reps):
        if before is not None:
            before()
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1))
    return float(np.median(ts)) / calls


def grouped_forward(nnv, sel, ws):
    nnv.nnv_conv_forward_grouped([p.desc for p in sel], [p.kind for p in sel], [p.x for p in sel], [p.w_tx for p in sel],
                                 None, [p.y for p in sel], ws, ws.numel())


CONFIG_CALLS = 5     # calls per replayed graph for the other configurations (time reported per call)


def stack_report(nnv, torch, np, side, name, dtype, kinds, per_layer=False):
    """One of the other workload configurations, measured beside the step by graph replay
    (CONFIG_CALLS calls per graph, time per call): the grouped transformation of every (layer, kind)
    pair, the grouped forward pass per kind, and the sum over layers of each layer's fastest kind
    (per-layer times from nnv_time_layer)."""
    from nnv_workloads import stack, layer_tensors, STACK_NAMES
    dev = torch.device("cuda:0")
    half = dtype == nnv.F16
    layers = stack(name)
    base = 220607446 + 1000 * (STACK_NAMES.index(name) + 1)
    pairs, inputs = [], []
    for i, layer in enumerate(layers):
        w, x = layer_tensors(layer, base + i)
        wd, xd = torch.from_numpy(w).to(dev), torch.from_numpy(x).to(dev)
        if half:
            xd = xd.half()
        inputs.append((wd, xd))
        d = nnv.make_desc(layer, dtype)
        for kind in kinds:
            if nnv.nnv_kind_supported(d, kind):
                pairs.append(Pair(nnv, torch, layer, kind, wd, xd, dev, dtype))
    out = {"stack": name, "dtype": "f16" if half else "f32", "layers": len(layers),
           "GMAC": round(sum(l.macs for l in layers) / 1e9, 3)}
    tx = [p for p in pairs if p.kind != nnv.DIRECT]
    if tx:
        t = graph_ms(torch, np, side, lambda: nnv.nnv_transform_weights_grouped(
            [p.desc for p in tx], [p.kind for p in tx], [p.w_raw for p in tx], [p.w_tx for p in tx]), calls=CONFIG_CALLS)
        by_kind = {}
        for kind in kinds:
            sel = [p for p in tx if p.kind == kind]
            if sel:
                tk = graph_ms(torch, np, side, lambda sel=sel: nnv.nnv_transform_weights_grouped(
                    [p.desc for p in sel], [p.kind for p in sel], [p.w_raw for p in sel], [p.w_tx for p in sel]), calls=CONFIG_CALLS)
                by_kind[KIND_LABEL[kind]] = {"layers": len(sel), "ms": round(tk, 4), "MB": round(sum(p.transform_bytes for p in sel) / 1e6, 1),
                                             "GBps": round(sum(p.transform_bytes for p in sel) / (tk * 1e-3) / 1e9, 1)}
        unique = sum({id(p.w_raw): p.raw_bytes for p in tx}.values()) + sum(p.tx_bytes for p in tx)
        out["transform"] = {"jobs": len(tx), "ms": round(t, 4), "MB_per_job_sum": round(sum(p.transform_bytes for p in tx) / 1e6, 1),
                            "MB_unique": round(unique / 1e6, 1), "GBps_unique": round(unique / (t * 1e-3) / 1e9, 1),
                            "by_kind": by_kind}
    fw = {}
    for kind in kinds:
        sel = [p for p in pairs if p.kind == kind]
        if not sel:
            continue
        need = nnv.nnv_conv_forward_grouped_workspace_bytes([p.desc for p in sel], [p.kind for p in sel])
        ws = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
        t = graph_ms(torch, np, side, lambda sel=sel, ws=ws: grouped_forward(nnv, sel, ws), calls=CONFIG_CALLS)
        fw[KIND_LABEL[kind]] = {"layers": len(sel), "ms": round(t, 4),
                                "TFLOPs_executed": round(sum(p.flops for p in sel) / (t * 1e-3) / 1e12, 2),
                                "TFLOPs_direct_equivalent": round(sum(p.direct_flops for p in sel) / (t * 1e-3) / 1e12, 2),
                                "GBps_algorithmic": round(sum(p.forward_bytes for p in sel) / (t * 1e-3) / 1e9, 1)}
        del ws
    out["forward_grouped_by_kind"] = fw
    if per_layer:
        # per-layer warm timings (queue of launches between events): each layer's fastest kind, and the
        # best single-layer rates of the GEMM kinds
        best, rates = {}, {}
        wsmax = torch.empty(max(max(p.ws_bytes for p in pairs), 256), dtype=torch.uint8, device=dev)
        for p in pairs:
            t = nnv.nnv_time_layer(p.desc, p.kind, p.w_raw, p.w_tx, p.x, p.y, wsmax, warmup=1, reps=3)
            best[p.layer.name] = min(best.get(p.layer.name, float("inf")), t.forward_ms)
            r = rates.setdefault(KIND_LABEL[p.kind], {"best_layer": None, "best_TFLOPs_executed": 0.0})
            tf = t.forward_flops / (t.forward_ms * 1e-3) / 1e12
            if tf > r["best_TFLOPs_executed"]:
                r["best_layer"], r["best_TFLOPs_executed"] = p.layer.name, round(tf, 2)
        out["layer_by_layer_best_kind_ms"] = round(sum(best.values()), 4)
        out["single_layer_best_rates"] = rates
    return out


def beyond_the_step(nnv, torch, np, layers, pairs, side, quick=False):
    """Measurements outside the timed step, same method (graph replay): the transformation with the
    caches flushed before every replay; the F(6x6) Winograd kind; the layer-by-layer forward pass
    of the step's stack (one launch group per layer, as nnv_conv_forward runs it); the whole cold
    pass of one kernel plan through nnv_cold_stack; the file-to-device rate of the
    transformed-weight cache; and the other workload configurations (single layer,
    MobileNetV2-, VGG-16- and ResNet-50-shaped stacks, the last also in float16)."""
    import tempfile
    dev = torch.device("cuda:0")
    out = {}
    # the step's transformation, cold: 512 MiB (twice the last-level cache) overwritten before each replay
    tx = [p for p in pairs if p.kind != nnv.DIRECT]
    flush = torch.empty(512 << 20, dtype=torch.uint8, device=dev)
    t_cold = graph_ms(torch, np, side, lambda: nnv.nnv_transform_weights_grouped(
        [p.desc for p in tx], [p.kind for p in tx], [p.w_raw for p in tx], [p.w_tx for p in tx]),
        before=lambda: flush.fill_(1))
    unique = sum({id(p.w_raw): p.raw_bytes for p in tx}.values()) + sum(p.tx_bytes for p in tx)
    out["transform_after_cache_flush"] = {"ms": round(t_cold, 4), "GBps_unique_bytes": round(unique / (t_cold * 1e-3) / 1e9, 1),
                                          "frac_of_hbm_peak": round(unique / (t_cold * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
    del flush
    # layer by layer (what nnv_conv_forward does: one launch group per layer)
    lbl = {}
    wsmax = torch.empty(max(max(p.ws_bytes for p in pairs), 256), dtype=torch.uint8, device=dev)
    for kind in (nnv.DIRECT, nnv.IM2COL_GEMM, nnv.WINO_F2, nnv.WINO_F4):
        sel = [p for p in pairs if p.kind == kind]

        def one_by_one(sel=sel):
            for p in sel:
                nnv.nnv_conv_forward(p.desc, p.kind, p.x, p.w_tx, None, p.y, wsmax, wsmax.numel())
        lbl[KIND_LABEL[kind]] = round(graph_ms(torch, np, side, one_by_one), 4)
    out["forward_layer_by_layer_ms"] = lbl
    # F(6x6,3x3) on the 13 eligible layers
    f6 = [Pair(nnv, torch, p.layer, nnv.WINO_F6, p.w_raw, p.x, dev) for p in pairs if p.kind == nnv.WINO_F4]
    need = nnv.nnv_conv_forward_grouped_workspace_bytes([q.desc for q in f6], [q.kind for q in f6])
    ws6 = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    t_tx = graph_ms(torch, np, side, lambda: nnv.nnv_transform_weights_grouped(
        [q.desc for q in f6], [q.kind for q in f6], [q.w_raw for q in f6], [q.w_tx for q in f6]))
    t_fw = graph_ms(torch, np, side, lambda: grouped_forward(nnv, f6, ws6))
    out["wino_f6"] = {"layers": len(f6), "transform_ms": round(t_tx, 4), "forward_ms": round(t_fw, 4),
                      "transform_GBps": round(sum(q.transform_bytes for q in f6) / (t_tx * 1e-3) / 1e9, 1),
                      "TFLOPs_direct_equivalent": round(sum(q.direct_flops for q in f6) / (t_fw * 1e-3) / 1e12, 3)}
    del ws6, f6
    # cold pass of the im2col-GEMM plan (every layer) through nnv_cold_stack
    plan = [p for p in pairs if p.kind == nnv.IM2COL_GEMM]
    tx_stream = torch.cuda.Stream()
    args = ([p.desc for p in plan], [p.kind for p in plan], [p.w_raw for p in plan], [p.w_tx for p in plan],
            [p.x for p in plan], [p.y for p in plan], wsmax)
    needg = nnv.nnv_conv_forward_grouped_workspace_bytes([p.desc for p in plan], [p.kind for p in plan])
    wsg = torch.empty(max(needg, 256), dtype=torch.uint8, device=dev)

    def grouped_plan():
        nnv.nnv_transform_weights_grouped([p.desc for p in plan], [p.kind for p in plan], [p.w_raw for p in plan],
                                          [p.w_tx for p in plan])
        grouped_forward(nnv, plan, wsg)
    out["cold_pass_im2col_plan"] = {
        "grouped_transform_then_grouped_forward_ms": round(graph_ms(torch, np, side, grouped_plan), 4),
        "one_grouped_transform_then_execute_ms": round(graph_ms(torch, np, side, lambda: nnv.nnv_cold_stack(
            *args, stage_layers=0, stream_exec=side)), 4),
        "stages_of_2_layers_one_stream_ms": round(graph_ms(torch, np, side, lambda: nnv.nnv_cold_stack(
            *args, stage_layers=2, stream_exec=side)), 4),
        "stages_of_2_layers_pipelined_on_two_streams_ms": round(graph_ms(torch, np, side, lambda: nnv.nnv_cold_stack(
            *args, stage_layers=2, stream_exec=side, stream_tx=tx_stream)), 4)}
    del wsg
    # transformed-weight cache: largest F(4x4) tensor of the stack, file -> device
    big = max((p for p in pairs if p.kind == nnv.WINO_F4), key=lambda p: p.tx_bytes)
    try:
        with tempfile.TemporaryDirectory() as d:
            path = os.path.join(d, "w.nnvc")
            nnv.nnv_cache_write(path, big.desc, big.kind, big.w_tx)
            ios = [nnv.nnv_cache_read(path, big.desc, big.kind, big.w_tx) for _ in range(3)]
        io = sorted(ios, key=lambda r: r.total_ms)[1]
        out["cache_read"] = {"bytes": int(io.bytes), "total_ms": round(io.total_ms, 3), "file_ms": round(io.file_ms, 3),
                             "GBps": round(io.bytes / (io.total_ms * 1e-3) / 1e9, 2), "direct_io": bool(io.direct_io)}
    except (OSError, nnv.NnvError) as e:
        if isinstance(e, nnv.NnvError) and e.status != -8:
            raise
        out["cache_read"] = None      # no writable temporary directory
    del wsmax
    if quick:
        return out
    # the other workload configurations
    K = nnv
    out["configs"] = {
        "1_single3x3_f32": stack_report(nnv, torch, np, side, "single3x3", K.F32,
                                        (K.DIRECT, K.IM2COL_GEMM, K.WINO_F2, K.WINO_F4), per_layer=True),
        "3_mobilenetv2_f32": stack_report(nnv, torch, np, side, "mobilenetv2", K.F32,
                                          (K.DIRECT, K.IM2COL_GEMM, K.DEPTHWISE), per_layer=True),
        "4_vgg16_f32": stack_report(nnv, torch, np, side, "vgg16", K.F32, (K.IM2COL_GEMM, K.WINO_F2, K.WINO_F4), per_layer=True),
        "5_resnet50_f32": stack_report(nnv, torch, np, side, "resnet50", K.F32, (K.IM2COL_GEMM, K.WINO_F4), per_layer=True),
        "5_resnet50_f16": stack_report(nnv, torch, np, side, "resnet50", K.F16, (K.IM2COL_GEMM, K.WINO_F4), per_layer=True),
    }
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--step-only", action="store_true",
                    help="only the timed step: no measurements beside it and no CPU baseline (the command profiled "
                         "under rocprofv3 --kernel-trace --stats)")
    ap.add_argument("--counter-pass", action="store_true",
                    help="run every kernel of the step a few times eagerly plus a plain 256 MiB copy and a read-mostly "
                         "convolution, nothing timed: the program to put under `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE`")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only; use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2206_07446_amd as nnv
    from nnv_workloads import stack, layer_tensors

    nnv.load()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    layers = stack("resnet18")
    pairs = []
    for i, layer in enumerate(layers):
        w, x = layer_tensors(layer, 220607446 + 2000 + i)
        wd, xd = torch.from_numpy(w).to(dev), torch.from_numpy(x).to(dev)
        for kind in applicable_kinds(nnv, layer):
            pairs.append(Pair(nnv, torch, layer, kind, wd, xd, dev))
    step_kinds = (nnv.DIRECT, nnv.IM2COL_GEMM, nnv.WINO_F2, nnv.WINO_F4)
    by_kind = {k: [p for p in pairs if p.kind == k] for k in step_kinds}
    ws_need = max(nnv.nnv_conv_forward_grouped_workspace_bytes([p.desc for p in sel], [p.kind for p in sel])
                  for sel in by_kind.values())
    ws = torch.empty(max(ws_need, 256), dtype=torch.uint8, device=dev)
    descs = [p.desc for p in pairs]
    kinds = [p.kind for p in pairs]
    srcs = [p.w_raw for p in pairs]
    dsts = [p.w_tx for p in pairs]

    def transform_all():     # on torch's current stream
        nnv.nnv_transform_weights_grouped(descs, kinds, srcs, dsts)

    def forward_kind(kind):
        grouped_forward(nnv, by_kind[kind], ws)

    if args.counter_pass:
        # calibration 1: the library's plain copy kernel over 64 Mi floats (256 MiB read, 256 MiB written);
        # calibration 2: a read-mostly kernel, the direct 1x1 convolution of 64 channels of 1024x1024 into 4
        # (256 MiB of x read once, 16 MiB written)
        big = type("L", (), dict(n=1, c=1024, h=256, w=256, k=1024, r=1, s=64, stride=1, pad=0, groups=1))()
        src = torch.zeros(64 << 20, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        cd = nnv.make_desc(big, nnv.F32)
        ro = type("L", (), dict(n=1, c=64, h=1024, w=1024, k=4, r=1, s=1, stride=1, pad=0, groups=1))()
        rd = nnv.make_desc(ro, nnv.F32)
        rw = torch.zeros(4 * 64, dtype=torch.float32, device=dev)
        ry = torch.empty(4 << 20, dtype=torch.float32, device=dev)
        for _ in range(3):
            nnv.nnv_transform_weights(cd, nnv.DIRECT, src, dst)
            nnv.nnv_conv_forward(rd, nnv.DIRECT, src, rw, None, ry, None)
            transform_all()
            for kind in step_kinds:
                forward_kind(kind)
        torch.cuda.synchronize()
        print(json.dumps({"counter_pass": "done", "copy_bytes_each_way": 4 * (64 << 20),
                          "read_mostly_bytes_read_written": [4 * (64 << 20), 4 * (4 << 20)],
                          "transform_bytes_per_step": sum(p.transform_bytes for p in pairs)}))
        return

    # A step is ten kernel launches in five calls (the grouped transformation, then one grouped
    # forward call per kernel kind), issued eagerly on torch's current stream: the GPU needs about
    # 0.35 ms for them, the host far less to enqueue them, so the queue never runs dry and the
    # events recorded between the calls split the step into its phases.
    phases = [("transform", transform_all)] + [(KIND_LABEL[k], (lambda k=k: forward_kind(k))) for k in step_kinds]
    for _ in range(max(args.warmup, 1)):
        for _, fn in phases:
            fn()
    torch.cuda.synchronize()

    stream = torch.cuda.current_stream()
    nph = len(phases)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(nph + 1)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        ev[s][0].record(stream)
        for i, (_, fn) in enumerate(phases):
            fn()
            ev[s][i + 1].record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    phase_ms = {phases[i][0]: float(np.mean([e[i].elapsed_time(e[i + 1]) for e in ev])) for i in range(nph)}
    tx_ms = phase_ms["transform"]
    fw_ms = sum(v for k, v in phase_ms.items() if k != "transform")

    tx_pairs = [p for p in pairs if p.kind != nnv.DIRECT]
    tx_bytes_jobs = sum(p.transform_bytes for p in tx_pairs)            # raw weights counted once per job
    tx_bytes_unique = sum({id(p.w_raw): p.raw_bytes for p in tx_pairs}.values()) + sum(p.tx_bytes for p in tx_pairs)
    fw_flops = sum(p.flops for p in pairs)
    fw_direct_flops = sum(p.direct_flops for p in pairs)

    # Roofline entries per phase, from the event-bracketed phase times of the timed region (phase
    # time / launches of the phase = average launch duration incl. the gap to the next kernel).
    counters_valid = csrc_digest() == MEASURED_TRAFFIC["csrc_sha256_16"]

    def entry(phase, bound, work, unit_scale, peak, unit, ms, extra=None):
        launches = PHASE_LAUNCHES[phase]
        ach = work / (ms * 1e-3) / unit_scale
        mb = MEASURED_TRAFFIC["MB_per_step"].get(phase) if counters_valid else None
        e = {"kernel": PHASE_KERNELS[phase], "bound": bound, "achieved": round(ach, 2), "peak": peak, "unit": unit,
             "frac": round(ach / peak, 4),
             # HBM bytes per launch (read + written), counters scaled as described at MEASURED_TRAFFIC
             "traffic": None if mb is None else round((mb[0] + mb[1]) * 1e6 / launches),
             "traffic_read_written": None if mb is None else [round(mb[0] * 1e6 / launches), round(mb[1] * 1e6 / launches)],
             "launches_per_step": launches, "avg_launch_us": round(ms * 1e3 / launches, 2), "phase_ms": round(ms, 4)}
        if extra:
            e.update(extra)
        return e

    per_kind, roof_all = {}, []
    # transformation: `achieved` counts every byte once (raw weights of a layer are read by up to
    # three jobs of the one launch, but have to come from HBM once); the per-job sum is given beside it
    mbt = MEASURED_TRAFFIC["MB_per_step"].get("transform") if counters_valid else None
    roof_all.append(entry("transform", "hbm", tx_bytes_unique, 1e9, HBM_PEAK_GBPS, "GB/s", tx_ms, {
        "algorithmic_MB": round(tx_bytes_unique / 1e6, 1), "per_job_sum_MB": round(tx_bytes_jobs / 1e6, 1),
        "achieved_per_job_sum": round(tx_bytes_jobs / (tx_ms * 1e-3) / 1e9, 1),
        "achieved_measured_bytes": None if mbt is None else round((mbt[0] + mbt[1]) * 1e6 / (tx_ms * 1e-3) / 1e9, 1)}))
    for kind in step_kinds:
        kname = KIND_LABEL[kind]
        sel = by_kind[kind]
        ms = phase_ms[kname]
        fl = sum(p.flops for p in sel)
        per_kind[kname] = {"layers": len(sel), "forward_ms": round(ms, 4),
                           "TFLOPs_executed": round(fl / (ms * 1e-3) / 1e12, 3),
                           "TFLOPs_direct_equivalent": round(sum(p.direct_flops for p in sel) / (ms * 1e-3) / 1e12, 3)}
        if kind == nnv.DIRECT:
            roof_all.append(entry(kname, "alu", fl, 1e12, VALU_F32_PEAK_TFLOPS, "TFLOP/s", ms))
        else:
            roof_all.append(entry(kname, "mfma", fl, 1e12, MFMA_F32_PEAK_TFLOPS, "TFLOP/s", ms))
    # the dominant kernel of the step = the phase with the largest share of the step time
    roofline = max(roof_all, key=lambda r: r["phase_ms"])

    out = {
        "metric": "cold transform+conv ms per model stack (weight-transform GB/s; conv TFLOP/s alongside)",
        "value": round(ms_per_step, 4), "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "resnet18-shaped conv stack, batch 1, 224x224, every layer x every applicable "
                               "kernel kind (direct, im2col_gemm, wino_f2, wino_f4); one grouped transformation, "
                               "one grouped forward call per kind",
                   "layers": len(layers), "layer_kind_pairs": len(pairs),
                   "launch": "eager, %d kernel launches per step in 5 calls" % sum(PHASE_LAUNCHES.values())},
        "weight_transform_GBps": round(tx_bytes_unique / (tx_ms * 1e-3) / 1e9, 1),
        "conv_TFLOPs_executed": round(fw_flops / (fw_ms * 1e-3) / 1e12, 3),
        "conv_TFLOPs_direct_equivalent": round(fw_direct_flops / (fw_ms * 1e-3) / 1e12, 3),
        "transform_ms": round(tx_ms, 4), "forward_ms": round(fw_ms, 4),
        "forward_by_kind": per_kind,
        "roofline": roofline,
        "roofline_all": roof_all,
    }
    if not args.step_only:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        out["beyond_the_step"] = beyond_the_step(nnv, torch, np, layers, pairs, side)
    if not (args.no_cpu_baseline or args.step_only):
        out["cpu_baseline"] = cpu_baseline(layers, nnv)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
