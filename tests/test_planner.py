"""Kernel-selection report logic on hand-made timing tables (no GPU)."""
from paper_2206_07446_amd.planner import Candidate, pareto_filter, choose, plan, report


def table2_like():
    # shaped like the paper's Table 2 (ms): name, transform, execute; raw 0.44 MB, winograd 7.1x larger
    raw = 442368
    return [Candidate("wino_f4", 38.23, 2.98, raw, int(raw * 64 / 9)),
            Candidate("im2col_gemm", 2.21, 8.14, raw, raw),
            Candidate("pack", 2.22, 18.63, raw, raw),
            Candidate("direct", 0.0, 8.01, raw, raw),
            Candidate("general", 0.0, 87.12, raw, raw)]


def test_pareto_filter_drops_dominated_candidates():
    kept = {c.kind for c in pareto_filter(table2_like())}
    # 'pack' and 'general' are slower in both operations than 'direct'; 'im2col_gemm' too
    assert kept == {"wino_f4", "direct"}


def test_equal_candidates_are_both_kept():
    a = Candidate("a", 1.0, 2.0, 10, 10)
    b = Candidate("b", 1.0, 2.0, 10, 10)
    assert len(pareto_filter([a, b])) == 2


def test_choice_depends_on_read_bandwidth_and_cache():
    cands = pareto_filter(table2_like())
    # slow storage (0.63 GB/s as in Table 2): reading the 7x larger cached tensor costs 5 ms
    c = choose("l", cands, read_gbps=0.63, allow_cache=False)
    assert c.kind == "direct" and not c.cached          # 0.70 + 0 + 8.01 beats 0.70 + 38.23 + 2.98
    c = choose("l", cands, read_gbps=0.63, allow_cache=True)
    assert c.kind == "wino_f4" and c.cached             # 4.99 + 2.98 beats 8.71
    assert abs(c.read_ms - 3145728 / 0.63e6) < 1e-9
    # very slow storage: the larger cached tensor no longer pays
    c = choose("l", cands, read_gbps=0.05, allow_cache=True)
    assert c.kind == "direct"


def test_plan_and_report_shapes():
    table = {"l0": table2_like(), "l1": table2_like()[1:]}
    choices = plan(table, 0.63)
    assert [c.layer for c in choices] == ["l0", "l1"]
    rep = report(table, 0.63)
    assert rep["plans"]["with_cache"]["cold_ms"] <= rep["plans"]["raw_only"]["cold_ms"]
    assert rep["plans"]["fastest_execution_kernel_cold"]["kinds"][0] == "wino_f4"
    assert rep["plans"]["fastest_execution_kernel_cold"]["cold_ms"] > rep["plans"]["raw_only"]["cold_ms"]
    assert any(not c["kept"] for c in rep["layers"]["l0"])


def test_measured_read_times_replace_the_bandwidth_model():
    """With Table 2's own read columns (0.70 ms raw, 5.23 ms cached Winograd) the cached Winograd
    kernel wins (5.23 + 2.98) over raw direct (0.70 + 8.01), whatever bandwidth is passed."""
    raw = 442368
    cands = [Candidate("wino_f4", 38.23, 2.98, raw, int(raw * 64 / 9), read_raw_ms=0.70, read_cache_ms=5.23),
             Candidate("direct", 0.0, 8.01, raw, raw, read_raw_ms=0.70, read_cache_ms=0.70)]
    c = choose("l", cands, read_gbps=1e-6, allow_cache=True)
    assert c.kind == "wino_f4" and c.cached and abs(c.cold_ms - 8.21) < 1e-9 and c.read_ms == 5.23
    c = choose("l", cands, read_gbps=1e-6, allow_cache=False)
    assert c.kind == "direct" and abs(c.cold_ms - 8.71) < 1e-9


def test_markdown_has_a_row_per_candidate_and_plan():
    from paper_2206_07446_amd.planner import markdown
    table = {"00_l0": table2_like(), "01_l1": table2_like()[1:]}
    text = markdown(report(table, 0.63))
    rows = [l for l in text.splitlines() if l.startswith("| 0")]
    assert len(rows) == 9
    assert "| with_cache |" in text and "wino_f4*" in text
