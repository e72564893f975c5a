"""Packed weight layouts (layout version 1) as closed-form index maps.

The weight transformation of a kernel (operation w_i of Section 3.2) ends in a
layout its execution reads directly; Fig. 3 shows the idea for the paper's CPU
kernels (channels interleaved in fours).  Here the blocking follows the
operand fragments of the 16-row matrix instructions the GPU kernels use.  Each
layout is stated as offset(logical index) -> position in a flat,
zero-initialised buffer; padding positions stay +0.

  GEMM panels, float32 (16 output channels x 4 input channels per fragment):
    off(k,c,r,s) = ((k//16 * C4 + c//4) * R*S + r*S + s) * 64 + (c%4)*16 + k%16
    size = ceil(K/16) * C4 * R*S * 64,  C4 = ceil(C/4)
  GEMM panels, float16 (16 x 32 per fragment, 8 consecutive channels per lane):
    off(k,c,r,s) = ((k//16 * C32 + c//32) * R*S + r*S + s) * 512
                   + ((c%32)//8)*128 + (k%16)*8 + c%8
    size = ceil(K/16) * C32 * R*S * 512,  C32 = ceil(C/32)
  Grouped convolution (K output channels in G groups of Kg = K/G, C channels per group):
    one such block per group, concatenated: off = (k // Kg) * size(Kg, C) + off(k % Kg, c, r, s)
  Winograd U[xi,k,c], xi = u*alpha + v: the same two formulas with (r,s) dropped
    and xi as the outermost index:
    float32: off = ((xi*K16 + k//16) * C4  + c//4 ) * 64  + (c%4)*16 + k%16
    float16: off = ((xi*K16 + k//16) * C32 + c//32) * 512 + ((c%32)//8)*128 + (k%16)*8 + c%8
  Depthwise (C,1,R,S), R = S = 3 or 5: off(c,r,s) = (c//32)*R*S*32 + (r*S+s)*32 + c%32,
    size = ceil(C/32)*R*S*32   (3x3: 288 per 32 channels)

Pins (tests/test_oracle_layouts.py): every map is injective and in range, the
unpack of a pack is the identity, sizes follow the formulas, padding is zero,
and a hand-written table for a tiny case in tests/golden/ matches.
"""
from __future__ import annotations

import numpy as np


def _ceil_div(a: int, b: int) -> int:
    return -(-a // b)


def gemm_offsets(K: int, C: int, R: int, S: int, half: bool, groups: int = 1):
    """(size, off) with off an int64 array of shape (K, C, R, S); C = channels per group."""
    if groups > 1:
        assert K % groups == 0
        kg = K // groups
        gsize, goff = gemm_offsets(kg, C, R, S, half)
        off = np.concatenate([goff + g * gsize for g in range(groups)], axis=0)
        return int(groups * gsize), off
    k, c, r, s = np.meshgrid(np.arange(K), np.arange(C), np.arange(R), np.arange(S), indexing="ij")
    if not half:
        cb = _ceil_div(C, 4)
        off = ((k // 16 * cb + c // 4) * (R * S) + r * S + s) * 64 + (c % 4) * 16 + k % 16
        size = _ceil_div(K, 16) * cb * R * S * 64
    else:
        cb = _ceil_div(C, 32)
        off = (((k // 16 * cb + c // 32) * (R * S) + r * S + s) * 512
               + ((c % 32) // 8) * 128 + (k % 16) * 8 + c % 8)
        size = _ceil_div(K, 16) * cb * R * S * 512
    return int(size), off.astype(np.int64)


def wino_offsets(alpha: int, K: int, C: int, half: bool):
    """(size, off) with off of shape (alpha*alpha, K, C)."""
    xi, k, c = np.meshgrid(np.arange(alpha * alpha), np.arange(K), np.arange(C), indexing="ij")
    kb = _ceil_div(K, 16)
    if not half:
        cb = _ceil_div(C, 4)
        off = ((xi * kb + k // 16) * cb + c // 4) * 64 + (c % 4) * 16 + k % 16
        size = alpha * alpha * kb * cb * 64
    else:
        cb = _ceil_div(C, 32)
        off = ((xi * kb + k // 16) * cb + c // 32) * 512 + ((c % 32) // 8) * 128 + (k % 16) * 8 + c % 8
        size = alpha * alpha * kb * cb * 512
    return int(size), off.astype(np.int64)


def depthwise_offsets(C: int, R: int = 3, S: int = 3):
    """(size, off) with off of shape (C, R, S)."""
    c, r, s = np.meshgrid(np.arange(C), np.arange(R), np.arange(S), indexing="ij")
    off = (c // 32) * (R * S * 32) + (r * S + s) * 32 + c % 32
    return int(_ceil_div(C, 32) * R * S * 32), off.astype(np.int64)


def _scatter(values, size, off, dtype):
    out = np.zeros(size, dtype=dtype)
    out[off.ravel()] = np.asarray(values).astype(dtype).ravel()
    return out


def pack_gemm(w, half: bool, groups: int = 1):
    """OIHW weights (K, C/groups, R, S) -> flat GEMM-panel buffer (float32, or float16 rounded to
    nearest even)."""
    K, C, R, S = w.shape
    size, off = gemm_offsets(K, C, R, S, half, groups)
    return _scatter(w, size, off, np.float16 if half else np.float32)


def unpack_gemm(buf, K, C, R, S, half: bool, groups: int = 1):
    _, off = gemm_offsets(K, C, R, S, half, groups)
    return np.asarray(buf)[off]


def pack_wino(U, half: bool, dtype=None):
    """U of shape (alpha, alpha, K, C) -> flat buffer; `dtype` overrides the storage type
    (float64 keeps the oracle's full precision for value comparisons)."""
    a, a2, K, C = U.shape
    assert a == a2
    size, off = wino_offsets(a, K, C, half)
    if dtype is None:
        dtype = np.float16 if half else np.float32
    return _scatter(U.reshape(a * a, K, C), size, off, dtype)


def unpack_wino(buf, alpha, K, C, half: bool):
    _, off = wino_offsets(alpha, K, C, half)
    return np.asarray(buf)[off].reshape(alpha, alpha, K, C)


def pack_depthwise(w, half: bool):
    C, one, R, S = w.shape
    assert one == 1 and R == S and R in (3, 5)
    size, off = depthwise_offsets(C, R, S)
    return _scatter(w.reshape(C, R, S), size, off, np.float16 if half else np.float32)


def unpack_depthwise(buf, C, R: int = 3, S: int = 3):
    _, off = depthwise_offsets(C, R, S)
    return np.asarray(buf)[off].reshape(C, 1, R, S)


def transformed_bytes(kind: str, K: int, Cg: int, R: int, S: int, half: bool, groups: int = 1) -> int:
    """Size of the transformed-weight buffer in bytes, per kernel kind."""
    e = 2 if half else 4
    if kind == "direct":
        return K * Cg * R * S * 4
    if kind == "im2col_gemm":
        return gemm_offsets(K, Cg, R, S, half, groups)[0] * e
    if kind == "wino_f2":
        return wino_offsets(4, K, Cg, half)[0] * e
    if kind == "wino_f4":
        return wino_offsets(6, K, Cg, half)[0] * e
    if kind == "wino_f6":
        return wino_offsets(8, K, Cg, half)[0] * e
    if kind == "depthwise":
        return depthwise_offsets(K, R, S)[0] * e
    raise ValueError(kind)
