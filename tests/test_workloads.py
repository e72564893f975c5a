"""Host checks of the workload shape lists against the sizes the paper's Table 4 quotes
(parameters include the networks' classifier layers, which are not convolutions: the conv
totals must sit below the quoted figure by about that much; FLOPs are quoted at 2 per MAC)."""
import pytest

from nnv_workloads import stack, STACK_NAMES

#            conv params (M)  classifier (M)  Table 4 params (M)  Table 4 GFLOPs
TABLE4 = {"resnet18": (11.17, 0.51, 12.7, 3.9), "resnet50": (23.45, 2.05, 25.7, 7.8),
          "mobilenetv2": (2.19, 1.28, 3.7, 0.6), "mobilenetv1": (3.19, 1.03, 4.4, 1.1),
          "squeezenet": (1.24, 0.0, 1.4, 1.7), "googlenet": (5.97, 1.03, 7.1, 3.2),
          "alexnet": (2.47, 58.63, 61.3, 1.4), "efficientnet_b0": (3.96, 1.28, 5.4, 0.8)}


@pytest.mark.parametrize("name", sorted(TABLE4))
def test_totals_match_table4(name):
    conv_m, fc_m, quoted_m, quoted_gflops = TABLE4[name]
    layers = stack(name)
    params = sum(l.params for l in layers) / 1e6
    gflops = 2 * sum(l.macs for l in layers) / 1e9
    assert abs(params - conv_m) < 0.01
    assert abs(params + fc_m - quoted_m) / quoted_m < 0.12          # batch-norm parameters and rounding aside
    assert abs(gflops - quoted_gflops) / quoted_gflops < 0.12


@pytest.mark.parametrize("name", STACK_NAMES)
def test_layers_are_well_formed(name):
    for l in stack(name):
        assert l.p > 0 and l.q > 0 and l.c % l.groups == 0 and l.k % l.groups == 0, l


def test_inception_branch_widths_chain():
    g = {l.name: l for l in stack("googlenet")}
    order = ["3a", "3b", "4a", "4b", "4c", "4d", "4e", "5a", "5b"]
    for a, b in zip(order, order[1:]):
        out = g[f"i{a}_1x1"].k + g[f"i{a}_3x3"].k + g[f"i{a}_5x5"].k + g[f"i{a}_pool_proj"].k
        assert out == g[f"i{b}_1x1"].c, (a, b)


def test_fire_modules_chain_and_sizes():
    s = stack("squeezenet")
    assert [l.h for l in s if l.name.endswith("squeeze")] == [54, 54, 54, 27, 27, 27, 27, 13]
    for sq, e1, e3 in zip(s[1::3], s[2::3], s[3::3]):
        assert e1.c == sq.k == e3.c and e1.k == e3.k


def test_shufflenet_units():
    """Width 1x, 3 groups: the architecture's own paper quotes 140 M multiply-adds for it (the
    classifier's 0.96 M included); Table 4's figure for "ShuffleNet" (3.6 M parameters, 1.9 GFLOPs)
    matches none of that paper's widths, so it is not asserted."""
    s = stack("shufflenet_g3")
    assert len(s) == 1 + 3 * 16
    assert abs(sum(l.macs for l in s) / 1e6 + 0.96 - 140) < 3
    grouped = [l for l in s if l.groups == 3]
    assert len(grouped) == 31 and all(l.r == 1 and l.c % 3 == 0 and l.k % 3 == 0 for l in grouped)
    assert s[1].groups == 1                                   # the first pointwise conv is not grouped
    assert [l.k for l in s if l.name.endswith("u0_pw2_g3")] == [216, 240, 480]


def test_shufflenetv2_width():
    """Width 1.5x is the published width whose size is closest to Table 4's "ShuffleNetV2" row
    (3.4 M parameters, 0.5 GFLOPs): 2.46 M conv + 1.02 M classifier parameters, 0.295 GMAC (that
    architecture's own paper: 3.5 M, 299 M multiply-adds)."""
    s = stack("shufflenetv2_x1_5")
    params = sum(l.params for l in s) / 1e6
    assert abs(params - 2.455) < 0.01 and abs(params + 1.025 - 3.4) / 3.4 < 0.05
    assert abs(sum(l.macs for l in s) / 1e6 + 1.0 - 299) < 6
    assert sum(l.is_depthwise for l in s) == 3 + 16 and all(l.groups in (1, l.c) for l in s)
