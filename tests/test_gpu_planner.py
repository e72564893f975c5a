"""The kernel-selection report on the device: `profile_stack` runs `nnv_time_layer` for every
candidate (Algorithm 1's profiling input, Section 3.3) and, with a cache directory, writes and
reads every candidate's weights (Table 2's "Read Raw" / "Read Cache").  Timings themselves are
"parity unpinned"; what is checked is that they respect the rooflines, that the sizes equal the
oracle's layout sizes and that the report keeps exactly the non-dominated candidates."""
import pytest

from nnv_workloads import stack
from oracle import layouts as OL

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2206_07446_amd as nnv
    assert torch.cuda.is_available(), "GPU tests need the HIP device"
    nnv.load()
    return nnv, torch


def check_table(nnv, table, name):
    from paper_2206_07446_amd.planner import KIND_NAMES, pareto_filter, report
    layers = stack(name)
    assert len(table) == len(layers)
    for (key, cands), layer in zip(table.items(), layers):
        assert key.endswith(layer.name)
        desc = nnv.make_desc(layer)
        kinds = [c.kind for c in cands]
        assert kinds == [KIND_NAMES[k] for k in range(6) if nnv.nnv_kind_supported(desc, k)]
        macs = layer.n * layer.k * layer.p * layer.q * layer.cg * layer.r * layer.s
        for c in cands:
            assert c.raw_bytes == layer.params * 4
            assert c.transformed_bytes == OL.transformed_bytes(c.kind, layer.k, layer.cg, layer.r, layer.s, False, layer.groups)
            # no faster than the rooflines allow: 8 TB/s for the transformation; 157.3 TFLOP/s for
            # the flops a kind executes (Winograd executes fewer than the plain convolution)
            if c.kind == "direct":
                assert c.transform_ms == 0.0
            else:
                assert c.transform_ms * 1e-3 >= (c.raw_bytes + c.transformed_bytes) / 8e12
            assert c.execute_ms > 0
            if not c.kind.startswith("wino"):
                assert c.execute_ms * 1e-3 >= 2.0 * macs / 157.3e12
    rep = report(table, read_gbps=2.0)
    for key, cands in table.items():
        kept = {c["kind"] for c in rep["layers"][key] if c["kept"]}
        assert kept == {c.kind for c in pareto_filter(cands)}
        for a in cands:                       # the definition, restated: kept <=> nobody dominates
            dom = any(b is not a and b.transform_ms <= a.transform_ms and b.execute_ms <= a.execute_ms and
                      (b.transform_ms < a.transform_ms or b.execute_ms < a.execute_ms) for b in cands)
            assert (a.kind in kept) == (not dom)
    for label in ("raw_only", "with_cache"):
        choices = rep["plans"][label]["choices"]
        assert len(choices) == len(layers)
        for ch, cands in zip(choices, table.values()):
            assert ch["kind"] in {c.kind for c in cands}
            assert abs(ch["cold_ms"] - (ch["read_ms"] + ch["transform_ms"] + ch["execute_ms"])) < 1e-9
        assert abs(rep["plans"][label]["cold_ms"] - sum(c["cold_ms"] for c in choices)) < 1e-9
    assert rep["plans"]["with_cache"]["cold_ms"] <= rep["plans"]["raw_only"]["cold_ms"] + 1e-12
    return rep


def test_profile_single_layer_cold(env):
    nnv, torch = env
    from paper_2206_07446_amd.planner import profile_stack, markdown
    table = profile_stack("single3x3", reps=3, flush_mb=64)
    rep = check_table(nnv, table, "single3x3")
    assert rep["timing"] == "cold" and "wino_f4" in markdown(rep)


def test_profile_with_cache_files(env, tmp_path):
    nnv, torch = env
    from paper_2206_07446_amd.planner import profile_stack
    table = profile_stack("single3x3", reps=2, flush_mb=0, cache_dir=str(tmp_path))
    check_table(nnv, table, "single3x3")
    for cands in table.values():
        for c in cands:
            assert c.read_raw_ms is not None and c.read_raw_ms > 0
            assert c.read_cache_ms is not None and c.read_cache_ms > 0
    assert list(tmp_path.iterdir()) == []          # the files are removed again
