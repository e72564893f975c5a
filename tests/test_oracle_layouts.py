"""Pins for the packed-layout index maps (no GPU)."""
import os

import numpy as np
import pytest

from oracle import layouts as L

GOLD = os.path.join(os.path.dirname(__file__), "golden", "layout_tables.txt")


def _blocks():
    out = []
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tok = line.split()
        if not tok[0].lstrip("-").isdigit():
            out.append((tok[0], [int(v) for v in tok[1:]], []))
        else:
            out[-1][2].append([int(v) for v in tok])
    return out


def test_hand_written_tables():
    seen = set()
    for name, dims, rows in _blocks():
        seen.add(name)
        if name == "gemm_f32":
            K, C, R, S = dims
            size, off = L.gemm_offsets(K, C, R, S, False)
            assert size == 128
            assert off[:, :, 0, 0].tolist() == rows
        elif name == "gemm_f32_rows":
            K, C, R, S = dims
            size, off = L.gemm_offsets(K, C, R, S, False)
            assert size == 256
            for row in rows:
                assert off[row[0], 0, 0, :].tolist() == row[1:]
        elif name == "gemm_f16":
            K, C, R, S = dims
            size, off = L.gemm_offsets(K, C, R, S, True)
            assert size == 1024
            assert off[0, :, 0, 0].tolist() == rows[0]
        elif name == "depthwise":
            size, off = L.depthwise_offsets(dims[0])
            assert size == 576
            for row in rows:
                c = row[0]
                assert [off[c, 0, 0], off[c, 1, 1], off[c, 2, 2]] == row[1:]
    assert seen == {"gemm_f32", "gemm_f32_rows", "gemm_f16", "depthwise"}


@pytest.mark.parametrize("half", [False, True])
@pytest.mark.parametrize("dims", [(16, 16, 3, 3), (3, 5, 1, 1), (64, 3, 7, 7), (24, 144, 1, 1), (33, 35, 3, 3)])
def test_gemm_map_is_injective_and_round_trips(dims, half):
    K, C, R, S = dims
    size, off = L.gemm_offsets(K, C, R, S, half)
    flat = off.ravel()
    assert flat.min() >= 0 and flat.max() < size
    assert len(np.unique(flat)) == flat.size
    cb = 32 if half else 4
    per = cb * 16
    assert size == -(-K // 16) * -(-C // cb) * R * S * per
    w = np.arange(K * C * R * S, dtype=np.float32).reshape(K, C, R, S)   # index-coded, exact
    if half:
        w = w % 2048        # exactly representable in float16
    buf = L.pack_gemm(w, half)
    assert buf.dtype == (np.float16 if half else np.float32)
    np.testing.assert_array_equal(L.unpack_gemm(buf, K, C, R, S, half), w.astype(buf.dtype))
    mask = np.ones(size, bool)
    mask[flat] = False
    assert not buf[mask].any() and not np.signbit(buf[mask]).any()


@pytest.mark.parametrize("half", [False, True])
@pytest.mark.parametrize("alpha,K,C", [(4, 16, 16), (6, 16, 16), (6, 20, 37), (4, 3, 2)])
def test_wino_map(alpha, K, C, half):
    size, off = L.wino_offsets(alpha, K, C, half)
    flat = off.ravel()
    assert flat.min() >= 0 and flat.max() < size and len(np.unique(flat)) == flat.size
    U = np.arange(alpha * alpha * K * C, dtype=np.float64).reshape(alpha, alpha, K, C) % 2048
    buf = L.pack_wino(U, half)
    np.testing.assert_array_equal(L.unpack_wino(buf, alpha, K, C, half), U.astype(buf.dtype))
    # frequency xi = u*alpha + v is the outermost, contiguous block
    per = size // (alpha * alpha)
    for xi in (0, alpha + 1, alpha * alpha - 1):
        blk = off[xi]
        assert blk.min() >= xi * per and blk.max() < (xi + 1) * per
    # the wino map equals the gemm map of a 1x1 filter, shifted per frequency
    _, g = L.gemm_offsets(K, C, 1, 1, half)
    np.testing.assert_array_equal(off[3], g[:, :, 0, 0] + 3 * per)


@pytest.mark.parametrize("C", [32, 96, 144, 5])
def test_depthwise_map(C):
    size, off = L.depthwise_offsets(C)
    flat = off.ravel()
    assert size == -(-C // 32) * 288
    assert flat.min() >= 0 and flat.max() < size and len(np.unique(flat)) == flat.size
    w = np.arange(C * 9, dtype=np.float32).reshape(C, 1, 3, 3)
    np.testing.assert_array_equal(L.unpack_depthwise(L.pack_depthwise(w, False), C), w)


def test_transformed_size_ratios():
    """Un-padded shapes: Winograd grows 3x3 weights by alpha^2/9 (16/9 and 4), the paper's
    8x8-tile example by 64/9 (Section 2, weights-transformation bullet); GEMM panels keep the size."""
    K = C = 64
    raw = K * C * 9 * 4
    assert L.transformed_bytes("direct", K, C, 3, 3, False) == raw
    assert L.transformed_bytes("im2col_gemm", K, C, 3, 3, False) == raw
    assert L.transformed_bytes("wino_f2", K, C, 3, 3, False) * 9 == raw * 16
    assert L.transformed_bytes("wino_f4", K, C, 3, 3, False) * 9 == raw * 36
    assert L.transformed_bytes("wino_f4", K, C, 3, 3, True) * 9 == raw * 18
    assert L.wino_offsets(8, K, C, False)[0] * 4 * 9 == raw * 64
    assert L.transformed_bytes("depthwise", 64, 1, 3, 3, False) == 64 * 9 * 4


def test_grouped_gemm_map_by_hand_and_by_properties():
    """Two groups of two output channels, one channel each, 1x1, float32: each group is one
    64-float fragment, rows at k % 16 -> offsets 0, 1 | 64, 65 (worked out by hand)."""
    size, off = L.gemm_offsets(4, 1, 1, 1, False, groups=2)
    assert size == 128 and off.ravel().tolist() == [0, 1, 64, 65]
    # float16, 3 groups of 5 output channels, 40 channels per group, 3x3: injective, in range,
    # group g confined to its own block, round trip, padding zero
    K, C, G = 15, 40, 3
    size, off = L.gemm_offsets(K, C, 3, 3, True, groups=G)
    gsize = L.gemm_offsets(K // G, C, 3, 3, True)[0]
    assert size == G * gsize and len(np.unique(off)) == off.size and off.min() >= 0 and off.max() < size
    for g in range(G):
        blk = off[g * 5:(g + 1) * 5]
        assert blk.min() >= g * gsize and blk.max() < (g + 1) * gsize
    w = np.random.default_rng(4).standard_normal((K, C, 3, 3)).astype(np.float32)
    buf = L.pack_gemm(w, True, groups=G)
    np.testing.assert_array_equal(L.unpack_gemm(buf, K, C, 3, 3, True, groups=G), w.astype(np.float16))
    mask = np.ones(size, bool); mask[off.ravel()] = False
    assert (buf[mask] == 0).all()
    assert L.transformed_bytes("im2col_gemm", K, C, 3, 3, True, groups=G) == size * 2


def test_depthwise_5x5_map():
    """5x5 taps: 25 x 32 floats per 32 channels; channel 33, tap (1, 2) of 40 channels sits in the
    second block at tap 7, lane 1: 800 + 7 * 32 + 1 = 1025 (worked out by hand)."""
    size, off = L.depthwise_offsets(40, 5, 5)
    assert size == 2 * 800 and off[33, 1, 2] == 1025 and off[0, 0, 0] == 0 and off[31, 4, 4] == 24 * 32 + 31
    flat = off.ravel()
    assert flat.min() >= 0 and flat.max() < size and len(np.unique(flat)) == flat.size
    w = np.arange(40 * 25, dtype=np.float32).reshape(40, 1, 5, 5)
    buf = L.pack_depthwise(w, False)
    np.testing.assert_array_equal(L.unpack_depthwise(buf, 40, 5, 5), w)
    assert L.transformed_bytes("depthwise", 40, 1, 5, 5, True) == size * 2
