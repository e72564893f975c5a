"""Reference Winograd F(m x m, 3 x 3) convolution in float64.

The paper's Winograd kernels (Table 2 "3x3s1-winograd(-pack4)", Fig. 3) turn
each 3x3 filter into an alpha x alpha tile (alpha = m + 2) ahead of execution
-- the weight transformation whose cost Section 3.1 trades against execution
time -- and then run the convolution tile by tile in the transformed domain.
This module states that computation step by step:

  1. U[k,c]   = G g[k,c] G^T                       (weight transformation)
  2. V[c,t]   = B^T d[c,t] B    d = alpha x alpha input patch of tile t,
                                 rows m*i - pad ... m*i - pad + alpha - 1, zero outside
  3. M[k,t]   = sum_c U[k,c] * V[c,t]              (elementwise per frequency)
  4. Y[k,t]   = A^T M[k,t] A                       (m x m outputs of tile t)
  5. rows/cols beyond P, Q are dropped.

The matrices come from oracle.cooktoom with the point sets and row scalings
declared in VARIANTS.  The result equals the direct convolution exactly in
real arithmetic.

conv2d_winograd_stored() is the same five steps with U, V and y rounded to a
storage type where the half-precision kernels round them (U after step 1, V
after step 2, y after step 5; everything between in float32 or wider).  It
states what the float16 Winograd variant computes, rounding included.

Pins (tests/test_oracle_winograd.py): conv2d_winograd_stored with float64
storage equals conv2d_winograd; with float16 storage it stays within the
half-precision bound of the direct convolution on the workload shapes.
conv2d_winograd == oracle.direct to
1e-12 relative on random layers including ragged tile edges; U for the
centre-delta and the all-ones filter against the closed forms
G[:,1] G[:,1]^T and (G 1)(G 1)^T typed from the printed matrices.
"""
from __future__ import annotations

from fractions import Fraction as Fr

import numpy as np

from .cooktoom import cook_toom, rescale

# variant -> (m, finite interpolation points, G row scale, B^T row scale)
#   F2       points 0, 1, -1 with the two sign flips that give the usual printed form.
#   F4       points 0, +-1, +-2: the usual printed F(4x4,3x3) matrices.
#   F4H      points 0, 1, -1, 2, -1/2 with power-of-two G row scaling; used when
#            U and V are stored in half precision (smaller dynamic range of U,
#            smaller entries in A^T; see the error study in the test-suite).
#   F6       points 0, +-1, +-2, +-1/2 (8 x 8 tiles, the tile size of Fig. 3), with the sign
#            of G row 0 and B^T row 0 flipped so that G starts (1, 0, 0).
VARIANTS = {
    "F2": (2, (0, 1, -1), (-1, 1, 1, 1), (-1, 1, 1, -1)),
    "F4": (4, (0, 1, -1, 2, -2), (1, 1, 1, 1, 1, 1), (1, 1, 1, 1, 1, 1)),
    "F4H": (4, (0, 1, -1, 2, Fr(-1, 2)), (4, 4, 4, 16, 4, 1), (1, 1, 1, 1, 1, 1)),
    "F6": (6, (0, 1, -1, 2, -2, Fr(1, 2), Fr(-1, 2)), (-1, 1, 1, 1, 1, 1, 1, 1), (-1, 1, 1, 1, 1, 1, 1, 1)),
}


def matrices_exact(variant: str):
    m, pts, gs, bs = VARIANTS[variant]
    AT, G, BT = cook_toom(m, pts)
    return rescale(AT, G, BT, gs, bs)


def matrices(variant: str):
    """(AT, G, BT) as float64 arrays (each rational rounded once)."""
    return tuple(np.array([[float(v) for v in row] for row in M], dtype=np.float64)
                 for M in matrices_exact(variant))


def tile_m(variant: str) -> int:
    return VARIANTS[variant][0]


def transform_weights(w, variant: str):
    """Step 1. w: (K, C, 3, 3) -> U: (alpha, alpha, K, C), U[u,v,k,c] = (G g[k,c] G^T)[u,v]."""
    w = np.asarray(w, dtype=np.float64)
    _, G, _ = matrices(variant)
    return np.einsum("ur,kcrs,vs->uvkc", G, w, G)


def transform_input(x, variant: str, pad: int = 1):
    """Step 2. x: (N, C, H, W) -> V: (alpha, alpha, N, C, tiles_h, tiles_w)."""
    x = np.asarray(x, dtype=np.float64)
    m = tile_m(variant)
    a = m + 2
    _, _, BT = matrices(variant)
    N, C, H, W = x.shape
    P, Q = H + 2 * pad - 2, W + 2 * pad - 2
    th, tw = -(-P // m), -(-Q // m)
    xp = np.zeros((N, C, th * m + 2, tw * m + 2), dtype=np.float64)
    hh, ww = min(H, xp.shape[2] - pad), min(W, xp.shape[3] - pad)
    xp[:, :, pad:pad + hh, pad:pad + ww] = x[:, :, :hh, :ww]
    V = np.zeros((a, a, N, C, th, tw), dtype=np.float64)
    for i in range(th):
        for j in range(tw):
            d = xp[:, :, i * m:i * m + a, j * m:j * m + a]
            V[:, :, :, :, i, j] = np.einsum("ur,ncrs,vs->uvnc", BT, d, BT)
    return V


def conv2d_winograd(x, w, variant: str, pad: int = 1, bias=None):
    """3x3, stride-1 convolution through steps 1-5 above."""
    x = np.asarray(x, dtype=np.float64)
    m = tile_m(variant)
    AT, _, _ = matrices(variant)
    N, C, H, W = x.shape
    K = w.shape[0]
    P, Q = H + 2 * pad - 2, W + 2 * pad - 2
    U = transform_weights(w, variant)
    V = transform_input(x, variant, pad)
    th, tw = V.shape[4], V.shape[5]
    Mf = np.einsum("uvkc,uvncij->uvnkij", U, V)
    Y = np.einsum("pu,uvnkij,qv->nkipjq", AT, Mf, AT).reshape(N, K, th * m, tw * m)
    y = Y[:, :, :P, :Q]
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64).reshape(1, K, 1, 1)
    return np.ascontiguousarray(y)


def conv2d_winograd_stored(x, w, variant: str, pad: int = 1, bias=None, store=np.float16):
    """Steps 1-5 with U, V and y rounded (to nearest even) to `store`; U and V are
    formed in float32 before that rounding, the contraction accumulates in float32."""
    m = tile_m(variant)
    AT, _, _ = matrices(variant)
    xs = np.asarray(x).astype(store).astype(np.float64)
    N, C, H, W = xs.shape
    K = w.shape[0]
    P, Q = H + 2 * pad - 2, W + 2 * pad - 2
    U = transform_weights(np.asarray(w, dtype=np.float64), variant).astype(np.float32).astype(store).astype(np.float64)
    V = transform_input(xs, variant, pad).astype(np.float32).astype(store).astype(np.float64)
    th, tw = V.shape[4], V.shape[5]
    Mf = np.einsum("uvkc,uvncij->uvnkij", U, V).astype(np.float32).astype(np.float64)
    Y = np.einsum("pu,uvnkij,qv->nkipjq", AT, Mf, AT).reshape(N, K, th * m, tw * m)
    y = Y[:, :, :P, :Q]
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64).reshape(1, K, 1, 1)
    return np.ascontiguousarray(y.astype(np.float32).astype(store).astype(np.float64))
