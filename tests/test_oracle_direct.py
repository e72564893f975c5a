"""Pins for the direct-convolution oracle (no GPU)."""
import itertools
import os

import numpy as np
import pytest
import scipy.signal

from oracle.direct import conv2d_at, conv2d_bruteforce, conv2d_direct, out_size
from oracle.cdirect import conv2d_direct_c

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _read_sobel():
    lines = [l.strip() for l in open(os.path.join(GOLD, "sobel_3x3.txt")) if l.strip() and not l.startswith("#")]
    for i in range(0, len(lines), 4):
        name, stride = lines[i], int(lines[i + 1])
        w = np.array(lines[i + 2].split(), dtype=np.float64).reshape(1, 1, 3, 3)
        y = np.array(lines[i + 3].split(), dtype=np.float64)
        yield name, stride, w, y


@pytest.mark.parametrize("fn", [conv2d_bruteforce, conv2d_direct, conv2d_direct_c])
def test_hand_worked_examples(fn):
    x = np.arange(1, 10, dtype=np.float64).reshape(1, 1, 3, 3)
    for name, stride, w, y in _read_sobel():
        got = fn(x, w, stride=stride, pad=1)
        assert got.ravel().tolist() == y.tolist(), name


CASES = [
    # N, C, H, W, K, R, stride, pad, groups
    (1, 2, 5, 4, 3, 1, 1, 0, 1),
    (1, 2, 5, 4, 3, 3, 1, 1, 1),
    (2, 2, 5, 4, 3, 3, 2, 1, 1),
    (1, 2, 5, 4, 3, 3, 1, 0, 1),
    (1, 3, 9, 8, 2, 7, 2, 3, 1),
    (1, 3, 6, 7, 3, 3, 1, 1, 3),
    (1, 3, 6, 7, 3, 3, 2, 1, 3),
    (1, 4, 5, 5, 6, 3, 1, 1, 2),
    (1, 2, 4, 6, 2, 1, 2, 0, 1),
]


@pytest.mark.parametrize("case", CASES)
def test_direct_matches_bruteforce(case):
    N, C, H, W, K, R, st, pad, g = case
    rng = np.random.default_rng(sum(case))
    x = rng.uniform(-1, 1, (N, C, H, W))
    w = rng.standard_normal((K, C // g, R, R))
    b = rng.standard_normal(K)
    ref = conv2d_bruteforce(x, w, st, pad, g, b)
    assert ref.shape == (N, K, out_size(H, R, st, pad), out_size(W, R, st, pad))
    np.testing.assert_allclose(conv2d_direct(x, w, st, pad, g, b), ref, rtol=0, atol=1e-13)
    x32, w32 = x.astype(np.float32), w.astype(np.float32)
    ref32 = conv2d_bruteforce(x32, w32, st, pad, g, b)
    np.testing.assert_allclose(conv2d_direct_c(x32, w32, st, pad, g, b), ref32, rtol=0, atol=1e-13)


def test_non_square_filter_bruteforce():
    rng = np.random.default_rng(5)
    x = rng.uniform(-1, 1, (1, 2, 6, 7))
    w = rng.standard_normal((3, 2, 1, 3))
    np.testing.assert_allclose(conv2d_direct(x, w, 1, 1), conv2d_bruteforce(x, w, 1, 1), atol=1e-13)


@pytest.mark.parametrize("fn", [conv2d_direct, conv2d_direct_c])
def test_centre_delta_is_identity(fn):
    rng = np.random.default_rng(1)
    C = 3
    x = rng.uniform(-1, 1, (2, C, 6, 5)).astype(np.float32)
    w = np.zeros((C, C, 3, 3), dtype=np.float32)
    for c in range(C):
        w[c, c, 1, 1] = 1.0
    np.testing.assert_array_equal(fn(x, w, 1, 1), x.astype(np.float64))


@pytest.mark.parametrize("fn", [conv2d_direct, conv2d_direct_c])
def test_all_ones_counts_valid_taps(fn):
    C, H, W = 5, 6, 7
    x = np.ones((1, C, H, W), dtype=np.float32)
    w = np.ones((2, C, 3, 3), dtype=np.float32)
    y = fn(x, w, 1, 1)
    exp = np.full((H, W), 9.0 * C)
    exp[0, :] = exp[-1, :] = 6.0 * C
    exp[:, 0] = exp[:, -1] = 6.0 * C
    for p, q in itertools.product((0, H - 1), (0, W - 1)):
        exp[p, q] = 4.0 * C
    for k in range(2):
        np.testing.assert_array_equal(y[0, k], exp)


def test_pointwise_is_matrix_product():
    rng = np.random.default_rng(2)
    x = rng.uniform(-1, 1, (1, 7, 5, 6))
    w = rng.standard_normal((4, 7, 1, 1))
    ref = (w.reshape(4, 7) @ x.reshape(7, 30)).reshape(1, 4, 5, 6)
    np.testing.assert_allclose(conv2d_direct(x, w), ref, atol=1e-13)
    # stride 2 samples every other pixel
    ref2 = (w.reshape(4, 7) @ x[0, :, ::2, ::2].reshape(7, -1)).reshape(1, 4, 3, 3)
    np.testing.assert_allclose(conv2d_direct(x, w, stride=2), ref2, atol=1e-13)


def test_depthwise_matches_scipy_correlate2d():
    rng = np.random.default_rng(3)
    C = 4
    x = rng.uniform(-1, 1, (1, C, 8, 9))
    w = rng.standard_normal((C, 1, 3, 3))
    y = conv2d_direct(x, w, 1, 1, groups=C)
    for c in range(C):
        ref = scipy.signal.correlate2d(x[0, c], w[c, 0], mode="same", boundary="fill", fillvalue=0)
        np.testing.assert_allclose(y[0, c], ref, atol=1e-13)
    y2 = conv2d_direct(x, w, 2, 1, groups=C)
    np.testing.assert_allclose(y2, y[:, :, ::2, ::2], atol=1e-13)


def test_full_conv_matches_scipy_sum_over_channels():
    rng = np.random.default_rng(4)
    x = rng.uniform(-1, 1, (1, 3, 7, 7))
    w = rng.standard_normal((2, 3, 3, 3))
    y = conv2d_direct(x, w, 1, 0)
    for k in range(2):
        ref = sum(scipy.signal.correlate2d(x[0, c], w[k, c], mode="valid") for c in range(3))
        np.testing.assert_allclose(y[0, k], ref, atol=1e-13)


def test_c_oracle_matches_numpy_on_single3x3_workload():
    from nnv_workloads import stack, layer_tensors
    layer = stack("single3x3")[0]
    w, x = layer_tensors(layer, 1, w_std=0.1)
    a = conv2d_direct(x, w, layer.stride, layer.pad)
    b = conv2d_direct_c(x, w, layer.stride, layer.pad)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-13 * np.abs(a).max())


@pytest.mark.parametrize("case", CASES)
def test_single_positions_match_bruteforce(case):
    """conv2d_at at every output position of the tiny layers = the 7-loop definition."""
    N, C, H, W, K, R, st, pad, g = case
    rng = np.random.default_rng(7 + sum(case))
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    w = rng.standard_normal((K, C // g, R, R)).astype(np.float32)
    b = rng.standard_normal(K)
    ref = conv2d_bruteforce(x, w, st, pad, g, b)
    pos = list(itertools.product(*[range(d) for d in ref.shape]))
    got = conv2d_at(x, w, pos, st, pad, g, b)
    np.testing.assert_allclose(got, ref.ravel(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(conv2d_at(x, w, pos[::3], st, pad, g), (ref - b.reshape(1, K, 1, 1)).ravel()[::3],
                               rtol=0, atol=1e-13)


def test_single_positions_hand_worked():
    """The hand-worked 3x3 examples, one position at a time (catches a flip or a transposition
    of the taps and a wrong stride or padding origin)."""
    x = np.arange(1, 10, dtype=np.float64).reshape(1, 1, 3, 3)
    for name, stride, w, y in _read_sobel():
        n = out_size(3, 3, stride, 1)
        pos = [(0, 0, p, q) for p in range(n) for q in range(n)]
        assert conv2d_at(x, w, pos, stride, 1).tolist() == y.tolist(), name
