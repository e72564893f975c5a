"""Kernel-selection report from per-operation timings (host side, no GPU arithmetic).

The paper's scheduler first profiles, per conv layer, the weight transformation and the
execution of every kernel candidate, drops the candidates that are no faster than another one
in either operation (Algorithm 1, first step; Section 3.3), and then chooses per layer a kernel
and whether to read raw weights and transform them or to read cached post-transformed weights
(Sections 3.1.1, 3.1.2, Table 2).  This module does that much from `nnv_time_layer` results and
`nnv_transformed_bytes`: the Pareto filter and, without the paper's multi-core pipelining
(out of scope), the per-layer minimum of
    read(raw bytes) + transform + execute      versus      read(transformed bytes) + execute
for a given weight-read bandwidth, or, with --cache-dir, for read times measured by writing
every candidate's weights to that directory with `nnv_cache_write` and reading them back cold
with `nnv_cache_read` (the "Read Raw" / "Read Cache" columns of Table 2).
`python -m paper_2206_07446_amd.planner --stack resnet18`.
"""
from __future__ import annotations

import argparse
import json
from dataclasses import dataclass, asdict
from typing import Dict, List, Optional

KIND_NAMES = {0: "direct", 1: "im2col_gemm", 2: "wino_f2", 3: "wino_f4", 4: "depthwise", 5: "wino_f6"}


@dataclass
class Candidate:
    """One kernel alternative of one layer: measured operations and weight sizes."""
    kind: str
    transform_ms: float
    execute_ms: float
    raw_bytes: int
    transformed_bytes: int
    read_raw_ms: Optional[float] = None     # measured file -> device time of the raw weights
    read_cache_ms: Optional[float] = None   # measured file -> device time of the transformed weights

    def read_ms(self, cached: bool, read_gbps: float) -> float:
        """Measured read time if there is one, else bytes over the given bandwidth."""
        measured = self.read_cache_ms if cached else self.read_raw_ms
        if measured is not None:
            return measured
        return (self.transformed_bytes if cached else self.raw_bytes) / (read_gbps * 1e6)


@dataclass
class Choice:
    layer: str
    kind: str
    cached: bool            # True: read post-transformed weights, False: read raw + transform
    cold_ms: float
    read_ms: float
    transform_ms: float
    execute_ms: float


def pareto_filter(cands: List[Candidate]) -> List[Candidate]:
    """Keep a candidate unless another one is at least as fast in both operations and faster in
    one (Algorithm 1, candidate filtering)."""
    kept = []
    for a in cands:
        dominated = any(
            b is not a and b.transform_ms <= a.transform_ms and b.execute_ms <= a.execute_ms and
            (b.transform_ms < a.transform_ms or b.execute_ms < a.execute_ms) for b in cands)
        if not dominated:
            kept.append(a)
    return kept


def choose(layer: str, cands: List[Candidate], read_gbps: float, allow_cache: bool = True) -> Choice:
    """Per-layer minimum over kernel x {raw + transform, cached} of read + transform + execute."""
    best: Optional[Choice] = None
    for c in cands:
        options = [(False, c.read_ms(False, read_gbps), c.transform_ms)]
        if allow_cache:
            options.append((True, c.read_ms(True, read_gbps), 0.0))
        for cached, read_ms, tx_ms in options:
            total = read_ms + tx_ms + c.execute_ms
            if best is None or total < best.cold_ms:
                best = Choice(layer, c.kind, cached, total, read_ms, tx_ms, c.execute_ms)
    assert best is not None
    return best


def plan(table: Dict[str, List[Candidate]], read_gbps: float, allow_cache: bool = True) -> List[Choice]:
    return [choose(name, pareto_filter(cands), read_gbps, allow_cache) for name, cands in table.items()]


def _median_read_ms(nnv, path, desc, kind, dst, reps=3):
    times = sorted(nnv.nnv_cache_read(path, desc, kind, dst).total_ms for _ in range(reps))
    return times[len(times) // 2]


COLD_FLUSH_MB = 512      # twice the 256 MB last-level cache: nothing of a layer survives the overwrite


def profile_stack(stack_name: str, dtype: int = 0, reps: int = 10, flush_mb: int = COLD_FLUSH_MB,
                  cache_dir: Optional[str] = None) -> Dict[str, List[Candidate]]:
    """Time every applicable kind of every layer of a workload on the GPU; with cache_dir also
    write each candidate's weights there and time reading them back.  The kernel selection
    prices the operations of a cold inference (Section 3.1.1, Table 2), so by default a flush
    buffer larger than the last-level cache is overwritten before every timed repetition and a
    repetition is one launch; flush_mb=0 gives warm timings (cache-resident operands, queued
    launches) instead."""
    import os
    import torch
    from nnv_workloads import stack, layer_tensors
    from . import binding as nnv
    dev = torch.device("cuda:0")
    flush = torch.empty(flush_mb << 20, dtype=torch.uint8, device=dev) if flush_mb else None
    table: Dict[str, List[Candidate]] = {}
    for i, layer in enumerate(stack(stack_name)):
        desc = nnv.make_desc(layer, dtype)
        w, x = layer_tensors(layer, 220607446 + i)
        wd = torch.from_numpy(w).to(dev)
        xd = torch.from_numpy(x).to(dev)
        if dtype == nnv.F16:
            xd = xd.half()
        y = torch.empty(layer.n * layer.k * layer.p * layer.q, dtype=xd.dtype, device=dev)
        cands = []
        for kind in range(6):
            if not nnv.nnv_kind_supported(desc, kind):
                continue
            nb = nnv.nnv_transformed_bytes(desc, kind)
            wt = wd if kind == nnv.DIRECT else torch.empty(nb, dtype=torch.uint8, device=dev)
            ws = torch.empty(max(16, nnv.nnv_workspace_bytes(desc, kind)), dtype=torch.uint8, device=dev)
            t = nnv.nnv_time_layer(desc, kind, wd, wt, xd, y, ws, flush=flush, warmup=2, reps=reps)
            cand = Candidate(KIND_NAMES[kind], t.transform_ms, t.forward_ms, layer.params * 4, nb)
            if cache_dir:
                raw_path = os.path.join(cache_dir, f"{i:02d}_raw.nnvc")
                if kind == nnv.DIRECT:
                    nnv.nnv_cache_write(raw_path, desc, nnv.DIRECT, wd)
                    raw_ms = _median_read_ms(nnv, raw_path, desc, nnv.DIRECT, torch.empty_like(wd))
                    cand.read_cache_ms = raw_ms
                else:
                    path = os.path.join(cache_dir, f"{i:02d}_{KIND_NAMES[kind]}.nnvc")
                    nnv.nnv_cache_write(path, desc, kind, wt)
                    cand.read_cache_ms = _median_read_ms(nnv, path, desc, kind, wt)
                    os.remove(path)
                cand.read_raw_ms = raw_ms
            cands.append(cand)
        if cache_dir:
            os.remove(os.path.join(cache_dir, f"{i:02d}_raw.nnvc"))
        table[f"{i:02d}_{layer.name}"] = cands
    return table


def report(table: Dict[str, List[Candidate]], read_gbps: float, timing: str = "cold") -> dict:
    out = {"read_GBps": read_gbps, "timing": timing, "layers": {}, "plans": {}}
    for name, cands in table.items():
        kept = {c.kind for c in pareto_filter(cands)}
        out["layers"][name] = [dict(asdict(c), kept=c.kind in kept) for c in cands]
    for label, cache in (("raw_only", False), ("with_cache", True)):
        choices = plan(table, read_gbps, cache)
        out["plans"][label] = {"cold_ms": sum(c.cold_ms for c in choices), "choices": [asdict(c) for c in choices]}
    # the plan a warm-inference engine would use: fastest execution only, weights transformed cold
    warm = [min(cands, key=lambda c: c.execute_ms) for cands in table.values()]
    out["plans"]["fastest_execution_kernel_cold"] = {
        "cold_ms": sum(c.read_ms(False, read_gbps) + c.transform_ms + c.execute_ms for c in warm),
        "kinds": [c.kind for c in warm]}
    return out


def markdown(rep: dict) -> str:
    """The report as two tables: candidates per layer (Table 2's columns) and the plans."""
    out = [f"Operation timings: {rep.get('timing', 'cold')}.", "",
           "| layer | kind | kept | read raw ms | transform ms | read cache ms | execute ms | raw+transform+execute | cache+execute |",
           "|---|---|---|---:|---:|---:|---:|---:|---:|"]
    gbps = rep["read_GBps"]
    for name, cands in rep["layers"].items():
        for c in cands:
            cand = Candidate(**{k: c[k] for k in ("kind", "transform_ms", "execute_ms", "raw_bytes", "transformed_bytes",
                                                 "read_raw_ms", "read_cache_ms")})
            rr, rc = cand.read_ms(False, gbps), cand.read_ms(True, gbps)
            out.append(f"| {name} | {c['kind']} | {'yes' if c['kept'] else 'no'} | {rr:.3f} | {c['transform_ms']:.3f} | {rc:.3f} | "
                       f"{c['execute_ms']:.3f} | {rr + c['transform_ms'] + c['execute_ms']:.3f} | {rc + c['execute_ms']:.3f} |")
    out += ["", "| plan | cold ms (sum over layers) | choices (layer: kind, * = cached) |", "|---|---:|---|"]
    for label, p in rep["plans"].items():
        if "choices" in p:
            ch = ", ".join(f"{c['layer'].split('_')[0]}: {c['kind']}{'*' if c['cached'] else ''}" for c in p["choices"])
        else:
            ch = ", ".join(p["kinds"])
        out.append(f"| {label} | {p['cold_ms']:.3f} | {ch} |")
    return "\n".join(out)


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--stack", default="resnet18")
    ap.add_argument("--read-gbps", type=float, default=2.0, help="weight read bandwidth (storage), GB/s")
    ap.add_argument("--half", action="store_true")
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--flush-mb", type=int, default=COLD_FLUSH_MB,
                    help="flush buffer overwritten before each timed repetition (cold timing); 0 = warm timing")
    ap.add_argument("--cache-dir", default=None, help="measure weight reads through cache files written here")
    ap.add_argument("--markdown", action="store_true", help="print tables instead of JSON")
    args = ap.parse_args()
    table = profile_stack(args.stack, 1 if args.half else 0, args.reps, args.flush_mb, args.cache_dir)
    rep = report(table, args.read_gbps, "cold" if args.flush_mb else "warm (operands cache-resident)")
    print(markdown(rep) if args.markdown else json.dumps(rep, indent=1))


if __name__ == "__main__":
    main()
