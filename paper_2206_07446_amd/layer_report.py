"""Per-layer roofline table of a workload: for every layer and every kernel kind that can run it,
the forward time, the algorithmic bytes and executed flops, the roofline bound
max(bytes / HBM peak, flops / compute peak), which side sets it, and bound / time.

Times come from HIP graph replays of repeated launches of one layer (kernel time plus the
gap between two kernels of a graph), the weight transformation from `nnv_time_layer`.
`python -m paper_2206_07446_amd.layer_report --stack resnet18 > table.md`
"""
from __future__ import annotations

import argparse

HBM_PEAK = 8.0e12            # bytes/s
MFMA_F32_PEAK = 157.3e12     # flop/s, float32 matrix cores
MFMA_F16_PEAK = 2.5e15       # flop/s, float16 matrix cores
VALU_F32_PEAK = 157.3e12     # flop/s, float32 vector ALU

KIND_NAMES = {0: "direct", 1: "im2col_gemm", 2: "wino_f2", 3: "wino_f4", 4: "depthwise", 5: "wino_f6"}


def forward_us(nnv, torch, desc, kind, x, w_tx, y, ws, reps=20):
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        for _ in range(3):
            nnv.nnv_conv_forward(desc, kind, x, w_tx, None, y, ws)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        for _ in range(reps):
            nnv.nnv_conv_forward(desc, kind, x, w_tx, None, y, ws)
    g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    best = float("inf")
    for _ in range(5):
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1) * 1e3 / reps)
    return best


def rows(stack_name: str, half: bool):
    import torch
    from nnv_workloads import stack, layer_tensors
    from . import binding as nnv
    dev = torch.device("cuda:0")
    dtype = nnv.F16 if half else nnv.F32
    for i, layer in enumerate(stack(stack_name)):
        desc = nnv.make_desc(layer, dtype)
        w, x = layer_tensors(layer, 220607446 + i)
        wd, xd = torch.from_numpy(w).to(dev), torch.from_numpy(x).to(dev)
        if half:
            xd = xd.half()
        y = torch.empty(layer.n * layer.k * layer.p * layer.q, dtype=xd.dtype, device=dev)
        for kind in range(6):
            if not nnv.nnv_kind_supported(desc, kind):
                continue
            nb = nnv.nnv_transformed_bytes(desc, kind)
            wt = wd if kind == nnv.DIRECT else torch.empty(nb, dtype=torch.uint8, device=dev)
            ws = torch.empty(max(16, nnv.nnv_workspace_bytes(desc, kind)), dtype=torch.uint8, device=dev)
            t = nnv.nnv_time_layer(desc, kind, wd, wt, xd, y, ws, warmup=1, reps=5)
            us = forward_us(nnv, torch, desc, kind, xd, wt, y, ws)
            peak = VALU_F32_PEAK if kind in (nnv.DIRECT, nnv.DEPTHWISE) else (MFMA_F16_PEAK if half else MFMA_F32_PEAK)
            t_mem, t_cmp = t.forward_bytes / HBM_PEAK * 1e6, t.forward_flops / peak * 1e6
            bound = max(t_mem, t_cmp)
            yield {"layer": f"{i:02d} {layer.name}", "kind": KIND_NAMES[kind], "us": us,
                   "GBps": t.forward_bytes / us / 1e3, "TFLOPs": t.forward_flops / us / 1e6,
                   "TFLOPs_direct_equiv": t.direct_equiv_flops / us / 1e6, "bound_us": bound,
                   "side": "hbm" if t_mem >= t_cmp else ("alu" if kind in (nnv.DIRECT, nnv.DEPTHWISE) else "mfma"),
                   "frac": bound / us, "transform_us": t.transform_ms * 1e3,
                   "transform_GBps": (t.transform_bytes / (t.transform_ms * 1e-3) / 1e9) if t.transform_ms > 0 else 0.0}


def counter_pass(stack_name: str, half: bool):
    """Every (layer, kind) of the stack, transformed once and run three times eagerly, nothing
    timed: the program to put under `rocprofv3 --pmc <counter> --kernel-trace`.  Dispatches
    appear in the order of the printed lines, three forward passes per line."""
    import torch
    from nnv_workloads import stack, layer_tensors
    from . import binding as nnv
    dev = torch.device("cuda:0")
    dtype = nnv.F16 if half else nnv.F32
    for i, layer in enumerate(stack(stack_name)):
        desc = nnv.make_desc(layer, dtype)
        w, x = layer_tensors(layer, 220607446 + i)
        wd, xd = torch.from_numpy(w).to(dev), torch.from_numpy(x).to(dev)
        if half:
            xd = xd.half()
        y = torch.empty(layer.n * layer.k * layer.p * layer.q, dtype=xd.dtype, device=dev)
        for kind in range(6):
            if not nnv.nnv_kind_supported(desc, kind):
                continue
            wt = wd if kind == nnv.DIRECT else torch.empty(nnv.nnv_transformed_bytes(desc, kind), dtype=torch.uint8, device=dev)
            ws = torch.empty(max(16, nnv.nnv_workspace_bytes(desc, kind)), dtype=torch.uint8, device=dev)
            nnv.nnv_transform_weights(desc, kind, wd, wt)
            for _ in range(3):
                nnv.nnv_conv_forward(desc, kind, xd, wt, None, y, ws)
            torch.cuda.synchronize()
            print(f"{i:02d} {layer.name} {KIND_NAMES[kind]}", flush=True)


def grouped_pass(stack_name: str, half: bool):
    """The whole stack through nnv_conv_forward_grouped, one call per kind that runs any of its
    layers, three times eagerly, nothing timed: the program to put under
    `rocprofv3 --kernel-trace --stats` or `--pmc <counter> --kernel-trace` when the kernels of
    the grouped launches are wanted (work items of all layers in one launch)."""
    import torch
    from nnv_workloads import stack, layer_tensors
    from . import binding as nnv
    dev = torch.device("cuda:0")
    dtype = nnv.F16 if half else nnv.F32
    per_kind = {}
    for i, layer in enumerate(stack(stack_name)):
        desc = nnv.make_desc(layer, dtype)
        w, x = layer_tensors(layer, 220607446 + i)
        wd, xd = torch.from_numpy(w).to(dev), torch.from_numpy(x).to(dev)
        if half:
            xd = xd.half()
        for kind in range(6):
            if not nnv.nnv_kind_supported(desc, kind):
                continue
            wt = wd if kind == nnv.DIRECT else torch.empty(nnv.nnv_transformed_bytes(desc, kind), dtype=torch.uint8, device=dev)
            y = torch.empty(layer.n * layer.k * layer.p * layer.q, dtype=xd.dtype, device=dev)
            per_kind.setdefault(kind, []).append((layer, desc, wd, wt, xd, y))
    for kind, sel in per_kind.items():
        descs, kinds = [s[1] for s in sel], [kind] * len(sel)
        nnv.nnv_transform_weights_grouped(descs, kinds, [s[2] for s in sel], [s[3] for s in sel])
        need = nnv.nnv_conv_forward_grouped_workspace_bytes(descs, kinds)
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
        for _ in range(3):
            nnv.nnv_conv_forward_grouped(descs, kinds, [s[4] for s in sel], [s[3] for s in sel], None, [s[5] for s in sel], ws, need)
        torch.cuda.synchronize()
        esz = 2 if half else 4
        act = sum(esz * (l.n * l.c * l.h * l.w + l.n * l.k * l.p * l.q) for l, *_ in sel)
        wbytes = sum(nnv.nnv_transformed_bytes(d, kind) for _, d, *_ in sel)
        print(f"{KIND_NAMES[kind]}: {len(sel)} layers, {sum(2.0 * l.macs for l, *_ in sel) / 1e9:.3f} GFLOP direct-equivalent, "
              f"activations {act / 1e6:.1f} MB + weights {wbytes / 1e6:.1f} MB", flush=True)


def grouped_summary(half: bool):
    """One line per workload: per kind the time of one nnv_conv_forward_grouped call over the layers
    that kind can run (and how many).  Timed as the median of 10 replays of a HIP graph holding
    5 calls back to back (the host side of a call with dozens of layers takes longer than the GPU)."""
    import torch
    from nnv_workloads import STACK_NAMES, stack, layer_tensors
    from . import binding as nnv
    dev = torch.device("cuda:0")
    dtype = nnv.F16 if half else nnv.F32
    kinds = [KIND_NAMES[k] for k in sorted(KIND_NAMES)]
    print("| stack | layers | GMAC | " + " | ".join(f"{k} us (layers)" for k in kinds) + " |")
    print("|---|---:|---:|" + "---:|" * len(kinds))
    for name in STACK_NAMES:
        per_kind = {}
        layers = stack(name)
        for i, layer in enumerate(layers):
            desc = nnv.make_desc(layer, dtype)
            w, x = layer_tensors(layer, 220607446 + i)
            wd, xd = torch.from_numpy(w).to(dev), torch.from_numpy(x).to(dev)
            if half:
                xd = xd.half()
            for kind in range(6):
                if not nnv.nnv_kind_supported(desc, kind):
                    continue
                wt = wd if kind == nnv.DIRECT else torch.empty(nnv.nnv_transformed_bytes(desc, kind), dtype=torch.uint8, device=dev)
                y = torch.empty(layer.n * layer.k * layer.p * layer.q, dtype=xd.dtype, device=dev)
                per_kind.setdefault(kind, []).append((layer, desc, wd, wt, xd, y))
        cells = {}
        for kind, sel in per_kind.items():
            descs, ks = [s[1] for s in sel], [kind] * len(sel)
            nnv.nnv_transform_weights_grouped(descs, ks, [s[2] for s in sel], [s[3] for s in sel])
            need = nnv.nnv_conv_forward_grouped_workspace_bytes(descs, ks)
            ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
            args = (descs, ks, [s[4] for s in sel], [s[3] for s in sel], None, [s[5] for s in sel], ws, need)
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                for _ in range(2):
                    nnv.nnv_conv_forward_grouped(*args)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                for _ in range(5):
                    nnv.nnv_conv_forward_grouped(*args)
            g.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ts = []
            for _ in range(10):
                e0.record()
                g.replay()
                e1.record()
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1) * 1e3 / 5)
            del g
            cells[KIND_NAMES[kind]] = f"{sorted(ts)[len(ts) // 2]:.1f} ({len(sel)})"
            del ws
        print(f"| {name} | {len(layers)} | {sum(l.macs for l in layers) / 1e9:.3f} | " +
              " | ".join(cells.get(k, "-") for k in kinds) + " |", flush=True)


def summary(half: bool):
    """One line per workload: layers, GMAC, and per kind the summed forward time of the layers it
    can run (and how many), then the sum over layers of the fastest kind of each."""
    from nnv_workloads import STACK_NAMES, stack
    kinds = [KIND_NAMES[k] for k in sorted(KIND_NAMES)]
    print("| stack | layers | GMAC | " + " | ".join(f"{k} us (layers)" for k in kinds) + " | best kind per layer, us |")
    print("|---|---:|---:|" + "---:|" * (len(kinds) + 1))
    for name in STACK_NAMES:
        per_kind, best = {}, {}
        for r in rows(name, half):
            a = per_kind.setdefault(r["kind"], [0.0, 0])
            a[0] += r["us"]; a[1] += 1
            best[r["layer"]] = min(best.get(r["layer"], float("inf")), r["us"])
        layers = stack(name)
        cells = [f"{per_kind[k][0]:.1f} ({per_kind[k][1]})" if k in per_kind else "-" for k in kinds]
        print(f"| {name} | {len(layers)} | {sum(l.macs for l in layers) / 1e9:.3f} | " + " | ".join(cells) +
              f" | {sum(best.values()):.1f} |", flush=True)


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--stack", default="resnet18")
    ap.add_argument("--half", action="store_true")
    ap.add_argument("--summary", action="store_true", help="totals of every workload instead of one per-layer table")
    ap.add_argument("--grouped-summary", action="store_true",
                    help="per workload and kind the time of one nnv_conv_forward_grouped call")
    ap.add_argument("--grouped-pass", action="store_true",
                    help="run the stack through nnv_conv_forward_grouped, one call per kind, three times (for rocprofv3)")
    ap.add_argument("--counter-pass", action="store_true",
                    help="run every (layer, kind) three times eagerly, nothing timed (for rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.grouped_summary:
        grouped_summary(args.half)
        return
    if args.grouped_pass:
        grouped_pass(args.stack, args.half)
        return
    if args.counter_pass:
        counter_pass(args.stack, args.half)
        return
    if args.summary:
        summary(args.half)
        return
    print(f"| layer | kind | forward us | GB/s | TFLOP/s executed | TFLOP/s direct-equivalent | bound us | bound by | "
          f"bound/time | transform us | transform GB/s |")
    print("|---|---|---:|---:|---:|---:|---:|---|---:|---:|---:|")
    tot = {}
    for r in rows(args.stack, args.half):
        print(f"| {r['layer']} | {r['kind']} | {r['us']:.2f} | {r['GBps']:.0f} | {r['TFLOPs']:.2f} | "
              f"{r['TFLOPs_direct_equiv']:.2f} | {r['bound_us']:.2f} | {r['side']} | {r['frac']:.3f} | "
              f"{r['transform_us']:.2f} | {r['transform_GBps']:.0f} |", flush=True)
        a = tot.setdefault(r["kind"], [0.0, 0.0, 0])
        a[0] += r["us"]; a[1] += r["bound_us"]; a[2] += 1
    print()
    print("| kind | layers | sum forward us | sum of bounds us | bound/time |")
    print("|---|---:|---:|---:|---:|")
    for k, (us, b, n) in tot.items():
        print(f"| {k} | {n} | {us:.1f} | {b:.1f} | {b / us:.3f} |")


if __name__ == "__main__":
    main()
