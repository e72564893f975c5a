"""Pins for the Cook-Toom matrices and the reference Winograd convolution (no GPU)."""
import os
from fractions import Fraction as Fr

import numpy as np
import pytest

from oracle import winograd as wg
from oracle.cooktoom import cook_toom
from oracle.direct import conv2d_direct

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _read_matrices():
    out, lines = {}, [l.strip() for l in open(os.path.join(GOLD, "winograd_matrices.txt"))
                      if l.strip() and not l.startswith("#")]
    i = 0
    while i < len(lines):
        name, rows, cols = lines[i].split()
        M = [[Fr(v) for v in lines[i + 1 + r].split()] for r in range(int(rows))]
        assert all(len(r) == int(cols) for r in M)
        out[name] = M
        i += 1 + int(rows)
    return out


def _matmul(A, B):
    return [[sum(A[i][k] * B[k][j] for k in range(len(B))) for j in range(len(B[0]))] for i in range(len(A))]


def _T(A):
    return [list(r) for r in zip(*A)]


@pytest.mark.parametrize("variant", list(wg.VARIANTS))
def test_exact_1d_identity_all_basis_pairs(variant):
    AT, G, BT = wg.matrices_exact(variant)
    m = wg.tile_m(variant)
    n = m + 2
    for gi in range(3):
        for di in range(n):
            Gg = [row[gi] for row in G]
            Bd = [row[di] for row in BT]
            prod = [a * b for a, b in zip(Gg, Bd)]
            y = [sum(AT[o][j] * prod[j] for j in range(n)) for o in range(m)]
            # correlation: y[o] = sum_k d[o+k] g[k] = 1 iff di == o + gi
            assert y == [Fr(1 if di == o + gi else 0) for o in range(m)]


@pytest.mark.parametrize("variant", list(wg.VARIANTS))
def test_exact_2d_identity_random_integers(variant):
    AT, G, BT = wg.matrices_exact(variant)
    m = wg.tile_m(variant)
    n = m + 2
    rng = np.random.default_rng(7)
    g = [[Fr(int(v)) for v in row] for row in rng.integers(-9, 10, (3, 3))]
    d = [[Fr(int(v)) for v in row] for row in rng.integers(-9, 10, (n, n))]
    U = _matmul(_matmul(G, g), _T(G))
    V = _matmul(_matmul(BT, d), _T(BT))
    Mh = [[U[i][j] * V[i][j] for j in range(n)] for i in range(n)]
    Y = _matmul(_matmul(AT, Mh), _T(AT))
    for p in range(m):
        for q in range(m):
            assert Y[p][q] == sum(d[p + r][q + s] * g[r][s] for r in range(3) for s in range(3))


def test_printed_matrices_reproduced():
    gold = _read_matrices()
    for v in ("F2", "F4"):
        AT, G, BT = wg.matrices_exact(v)
        assert AT == gold[f"{v}_AT"]
        assert G == gold[f"{v}_G"]
        assert BT == gold[f"{v}_BT"]


def test_generator_without_rescaling_is_f4_printed_form():
    gold = _read_matrices()
    AT, G, BT = cook_toom(4, (0, 1, -1, 2, -2))
    assert (AT, G, BT) == (gold["F4_AT"], gold["F4_G"], gold["F4_BT"])


def test_half_precision_variant_scaling_is_power_of_two():
    m, pts, gs, bs = wg.VARIANTS["F4H"]
    for v in list(gs) + list(bs):
        assert v > 0 and (int(v) & (int(v) - 1)) == 0


SHAPES = [
    # N, C, H, W, K, pad
    (1, 3, 8, 8, 2, 1),
    (1, 2, 7, 7, 3, 1),      # ragged for m = 2 and m = 4
    (2, 3, 14, 9, 2, 1),     # 14 = 3.5 tiles of 4
    (1, 2, 6, 10, 2, 0),
    (1, 1, 3, 3, 1, 1),      # single ragged tile
    (1, 2, 5, 4, 2, 2),
]


@pytest.mark.parametrize("variant", list(wg.VARIANTS))
@pytest.mark.parametrize("shape", SHAPES)
def test_winograd_equals_direct(variant, shape):
    N, C, H, W, K, pad = shape
    rng = np.random.default_rng(11 + H * W)
    x = rng.uniform(-1, 1, (N, C, H, W))
    w = rng.standard_normal((K, C, 3, 3))
    b = rng.standard_normal(K)
    ref = conv2d_direct(x, w, 1, pad, 1, b)
    got = wg.conv2d_winograd(x, w, variant, pad, b)
    assert got.shape == ref.shape
    assert np.abs(got - ref).max() <= 1e-12 * np.abs(ref).max()


def test_winograd_equals_direct_on_workload_layer():
    from nnv_workloads import stack, layer_tensors
    layer = stack("single3x3")[0]
    w, x = layer_tensors(layer, 1, w_std=0.1)
    ref = conv2d_direct(x, w, 1, 1)
    for v in wg.VARIANTS:
        got = wg.conv2d_winograd(x, w, v, 1)
        assert np.abs(got - ref).max() <= 1e-12 * np.abs(ref).max()


# G times the all-ones vector, typed from the printed matrices
G_ROWSUM = {"F2": [1, 1.5, 0.5, 1], "F4": [1 / 4, -1 / 2, -1 / 6, 7 / 24, 1 / 8, 1],
            # F(6x6): rows (1,0,0), -2/9 (1,1,1), -2/9 (1,-1,1), (1,2,4)/90, (1,-2,4)/90, (32,16,8)/45,
            # (32,-16,8)/45, (0,0,1), worked out by hand from the interpolation points
            "F6": [1, -2 / 3, -2 / 9, 7 / 90, 1 / 30, 56 / 45, 8 / 15, 1]}
# middle column of G, typed from the printed matrices
G_MID = {"F2": [0, 0.5, -0.5, 0], "F4": [0, -1 / 6, 1 / 6, 1 / 12, -1 / 12, 0],
         "F6": [0, -2 / 9, 2 / 9, 1 / 45, -1 / 45, 16 / 45, -16 / 45, 0]}


@pytest.mark.parametrize("variant", ["F2", "F4", "F6"])
def test_weight_transform_closed_forms(variant):
    a = wg.tile_m(variant) + 2
    w = np.zeros((2, 3, 3, 3))
    w[0, :, 1, 1] = 1.0      # centre delta
    w[1] = 1.0               # all ones
    U = wg.transform_weights(w, variant)
    assert U.shape == (a, a, 2, 3)
    mid, ones = np.array(G_MID[variant]), np.array(G_ROWSUM[variant])
    for c in range(3):
        np.testing.assert_allclose(U[:, :, 0, c], np.outer(mid, mid), atol=1e-15)
        np.testing.assert_allclose(U[:, :, 1, c], np.outer(ones, ones), atol=1e-15)


def test_weight_transform_is_not_symmetric_in_r_s():
    """A filter with one off-centre tap: U must be G[:,r] G[:,s]^T, not its transpose."""
    _, G, _ = wg.matrices("F4")
    w = np.zeros((1, 1, 3, 3))
    w[0, 0, 0, 2] = 1.0
    U = wg.transform_weights(w, "F4")[:, :, 0, 0]
    np.testing.assert_allclose(U, np.outer(G[:, 0], G[:, 2]), atol=1e-15)
    assert np.abs(U - U.T).max() > 1e-3


def test_input_transform_tile_geometry():
    """A single 1 at pixel (ih, iw) lands in tile (i, j) at patch position
    (ih + pad - m*i, iw + pad - m*j): V equals the outer product of B^T columns."""
    _, _, BT = wg.matrices("F4")
    x = np.zeros((1, 1, 9, 9))
    x[0, 0, 5, 2] = 1.0
    V = wg.transform_input(x, "F4", pad=1)
    assert V.shape == (6, 6, 1, 1, 3, 3)
    # tile (1, 0): rows 3..8, cols -1..4 -> patch position (5+1-4, 2+1-0) = (2, 3)
    np.testing.assert_allclose(V[:, :, 0, 0, 1, 0], np.outer(BT[:, 2], BT[:, 3]), atol=1e-15)
    # tile (0, 0): rows -1..4 does not contain row 5
    assert np.abs(V[:, :, 0, 0, 0, 0]).max() == 0


def _sim_half(variant, C, K, HW, seed):
    """Winograd with U, V and y stored in float16: error vs direct, share of subnormal U."""
    rng = np.random.default_rng(seed)
    w = (rng.standard_normal((K, C, 3, 3)) * np.sqrt(2 / (C * 9))).astype(np.float32)
    x = rng.uniform(-1, 1, (1, C, HW, HW)).astype(np.float16)
    ref = conv2d_direct(x.astype(np.float64), w.astype(np.float64), 1, 1)
    U = wg.transform_weights(w, variant).astype(np.float32).astype(np.float16)
    sub = np.mean((np.abs(U.astype(np.float32)) < 2.0 ** -14) & (U != 0))
    y = wg.conv2d_winograd_stored(x, w, variant, 1, store=np.float16)
    return np.abs(y - ref).max() / np.abs(ref).max(), sub


@pytest.mark.parametrize("variant", list(wg.VARIANTS))
def test_stored_variant_with_float64_storage_is_the_plain_one(variant):
    rng = np.random.default_rng(21)
    x = rng.uniform(-1, 1, (2, 3, 9, 7))
    w = rng.standard_normal((4, 3, 3, 3))
    b = rng.standard_normal(4)
    a = wg.conv2d_winograd_stored(x, w, variant, 1, b, store=np.float64)
    ref = wg.conv2d_winograd(x, w, variant, 1, b)
    # only the float32 hop of the accumulator separates the two; A^T of the 8x8 tile has
    # entries up to 32, which amplify that rounding
    assert np.abs(a - ref).max() <= (1e-5 if variant == "F6" else 1e-6) * np.abs(ref).max()


def test_f6_is_not_offered_in_half_precision():
    """With U and V rounded to half precision the 8x8-tile variant misses the 5e-3 bound on
    CNN-sized layers (A^T entries up to 32 amplify the rounding of U and V), which is why the
    library refuses that pairing."""
    for C, HW in ((64, 28), (256, 14)):
        e, _ = _sim_half("F6", C, C, HW, 3)
        assert e > 5e-3


def test_half_precision_error_study():
    """Why F(4x4) uses another point set when U and V are stored in half precision:
    the points 0,+-1,+-2 miss the 5e-3 bound, the points 0,1,-1,2,-1/2 meet it and
    their scaled U has almost no half-precision subnormals (only values that are
    accidentally near zero, whose loss is harmless)."""
    for C, HW in ((64, 28), (256, 14)):
        e_canon, _ = _sim_half("F4", C, C, HW, 3)
        e_alt, sub_alt = _sim_half("F4H", C, C, HW, 3)
        e_f2, _ = _sim_half("F2", C, C, HW, 3)
        assert e_canon > 5e-3
        assert e_alt < 4.2e-3 and sub_alt < 1e-3
        assert e_f2 < 1.5e-3
