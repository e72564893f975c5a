"""Winograd F(m, 3) transform matrices by the Cook-Toom construction, in exact rationals.

The paper only names the Winograd kernel (Section 3.1.1, Table 2, Fig. 3; its
reference [36]); it prints no matrices.  They follow from polynomial
interpolation: the m outputs of a 3-tap correlation are the coefficients of a
product of two polynomials taken modulo prod(x - p_j) and "x - infinity",
evaluated at n - 1 = m + 1 finite points p_j and recombined.

Pinned by tests/test_oracle_winograd.py: the exact 1-D identity
A^T[(G g) * (B^T d)] = correlate(d, g) for every pair of basis vectors, an
exact 2-D identity on random integers, and the printed F(2,3)/F(4,3) matrices
of the common literature form for the points {0, 1, -1} and {0, 1, -1, 2, -2}.
"""
from __future__ import annotations

from fractions import Fraction as Fr
from typing import List, Sequence, Tuple

Mat = List[List[Fr]]


def _poly_mul_linear(coef: List[Fr], root: Fr) -> List[Fr]:
    """coef (ascending powers) times (x - root)."""
    out = [Fr(0)] * (len(coef) + 1)
    for i, a in enumerate(coef):
        out[i + 1] += a
        out[i] -= a * root
    return out


def cook_toom(m: int, points: Sequence) -> Tuple[Mat, Mat, Mat]:
    """Return (AT, G, BT) for F(m, 3) built on the finite `points` plus infinity.

    AT is m x n, G is n x 3, BT is n x n with n = m + 2 = len(points) + 1, and
    for a 3-tap filter g and an n-long signal d
        AT @ ((G @ g) * (BT @ d))  ==  [sum_k d[o + k] * g[k] for o in range(m)].
    """
    pts = [Fr(p) for p in points]
    n = m + 2
    if len(pts) != n - 1 or len(set(pts)) != len(pts):
        raise ValueError("need m + 1 distinct finite points")
    AT = [[pts[j] ** i for j in range(n - 1)] + [Fr(1 if i == m - 1 else 0)] for i in range(m)]
    G = []
    for j, pj in enumerate(pts):
        nj = Fr(1)
        for l, pl in enumerate(pts):
            if l != j:
                nj *= pj - pl
        G.append([pj ** k / nj for k in range(3)])
    G.append([Fr(0), Fr(0), Fr(1)])
    BT = []
    for j in range(n - 1):
        coef = [Fr(1)]
        for l, pl in enumerate(pts):
            if l != j:
                coef = _poly_mul_linear(coef, pl)
        BT.append(coef + [Fr(0)])
    coef = [Fr(1)]
    for pl in pts:
        coef = _poly_mul_linear(coef, pl)
    BT.append(coef)
    return AT, G, BT


def rescale(AT: Mat, G: Mat, BT: Mat, g_scale: Sequence, b_scale: Sequence) -> Tuple[Mat, Mat, Mat]:
    """Multiply row j of G by g_scale[j] and row j of BT by b_scale[j]; divide
    column j of AT by their product.  The identity of cook_toom() is unchanged."""
    gs = [Fr(v) for v in g_scale]
    bs = [Fr(v) for v in b_scale]
    G2 = [[gs[j] * v for v in row] for j, row in enumerate(G)]
    B2 = [[bs[j] * v for v in row] for j, row in enumerate(BT)]
    A2 = [[v / (gs[j] * bs[j]) for j, v in enumerate(row)] for row in AT]
    return A2, G2, B2
