"""Direct 2-D convolution (zero-padded cross-correlation) in float64.

Every kernel alternative of a conv operator computes the same operator
(Section 3.1.1: kernels are different implementations of one operator; the
engine has zero accuracy loss, Section 1), so one definition serves all of
them:

    y[n,k,p,q] = b[k] + sum_{c in group(k)} sum_{r<R} sum_{s<S}
                 x[n, c, p*stride - pad + r, q*stride - pad + s] * w[k, c', r, s]

with x = 0 outside the image, no filter flip, dilation 1 and
P = floor((H + 2*pad - R)/stride) + 1 (same for Q).

Pins (tests/test_oracle_direct.py): conv2d_direct against the 7-loop
conv2d_bruteforce on tiny layers; both against closed forms (centre-delta
filter gives y = x; all-ones tensors count the valid taps), against a plain
matrix product for 1x1 filters, against scipy.signal.correlate2d per channel,
and against brute-force values worked by hand in tests/golden/.  conv2d_at
(single output positions of layers too large to evaluate whole) against
conv2d_bruteforce at every position of tiny layers, and against a hand-worked
golden value.
"""
from __future__ import annotations

import numpy as np


def out_size(h: int, r: int, stride: int, pad: int) -> int:
    return (h + 2 * pad - r) // stride + 1


def conv2d_bruteforce(x, w, stride=1, pad=0, groups=1, bias=None):
    """The definition as seven nested Python loops (tiny inputs only)."""
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    N, C, H, W = x.shape
    K, Cg, R, S = w.shape
    assert C == Cg * groups and K % groups == 0
    P, Q = out_size(H, R, stride, pad), out_size(W, S, stride, pad)
    kg = K // groups
    y = np.zeros((N, K, P, Q), dtype=np.float64)
    for n in range(N):
        for k in range(K):
            g = k // kg
            for p in range(P):
                for q in range(Q):
                    acc = 0.0 if bias is None else float(bias[k])
                    for c in range(Cg):
                        for r in range(R):
                            ih = p * stride - pad + r
                            if ih < 0 or ih >= H:
                                continue
                            for s in range(S):
                                iw = q * stride - pad + s
                                if iw < 0 or iw >= W:
                                    continue
                                acc += x[n, g * Cg + c, ih, iw] * w[k, c, r, s]
                    y[n, k, p, q] = acc
    return y


def conv2d_direct(x, w, stride=1, pad=0, groups=1, bias=None):
    """Same definition, one filter tap at a time: for each (r, s) the strided
    window of the zero-padded input is contracted with w[:, :, r, s] over the
    group's channels (a matrix product per group)."""
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    N, C, H, W = x.shape
    K, Cg, R, S = w.shape
    assert C == Cg * groups and K % groups == 0
    P, Q = out_size(H, R, stride, pad), out_size(W, S, stride, pad)
    kg = K // groups
    xp = np.zeros((N, C, H + 2 * pad, W + 2 * pad), dtype=np.float64)
    xp[:, :, pad:pad + H, pad:pad + W] = x
    y = np.zeros((N, groups, kg, P * Q), dtype=np.float64)
    wg = w.reshape(groups, kg, Cg, R, S)
    for r in range(R):
        for s in range(S):
            win = xp[:, :, r:r + (P - 1) * stride + 1:stride, s:s + (Q - 1) * stride + 1:stride]
            win = np.ascontiguousarray(win).reshape(N, groups, Cg, P * Q)
            # (groups, kg, Cg) @ (N, groups, Cg, PQ) -> (N, groups, kg, PQ)
            y += np.matmul(wg[None, :, :, :, r, s], win)
    y = y.reshape(N, K, P, Q)
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64).reshape(1, K, 1, 1)
    return y


def conv2d_at(x, w, positions, stride=1, pad=0, groups=1, bias=None):
    """The same definition evaluated at single output positions (n, k, p, q) only, for
    layers whose whole output the CPU cannot afford: per position, the sum over the filter
    taps that fall inside the image of the dot product over the group's channels."""
    N, C, H, W = x.shape
    K, Cg, R, S = w.shape
    assert C == Cg * groups and K % groups == 0
    kg = K // groups
    out = np.empty(len(positions), dtype=np.float64)
    for i, (n, k, p, q) in enumerate(positions):
        c0 = (k // kg) * Cg
        acc = 0.0 if bias is None else float(bias[k])
        for r in range(R):
            ih = p * stride - pad + r
            if ih < 0 or ih >= H:
                continue
            for s in range(S):
                iw = q * stride - pad + s
                if iw < 0 or iw >= W:
                    continue
                acc += float(np.dot(np.asarray(x[n, c0:c0 + Cg, ih, iw], dtype=np.float64),
                                    np.asarray(w[k, :, r, s], dtype=np.float64)))
        out[i] = acc
    return out
