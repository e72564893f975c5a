"""Helpers shared by the GPU parity tests: run one (layer, kind, dtype) through the C ABI
and build the oracle's expectation for it.  The oracle side lives in oracle/ only."""
from __future__ import annotations

import numpy as np

from oracle import layouts as OL
from oracle import winograd as OW
from oracle.direct import conv2d_direct

KIND_NAMES = {0: "direct", 1: "im2col_gemm", 2: "wino_f2", 3: "wino_f4", 4: "depthwise", 5: "wino_f6"}


def wino_variant(kind: int, half: bool) -> str:
    if kind == 2:
        return "F2"
    if kind == 5:
        return "F6"
    return "F4H" if half else "F4"


def conv_tolerance(kind: int, half: bool) -> float:
    """max|y - y_oracle| <= tol * max|y_oracle|: 1e-4 for the float32 direct, GEMM, depthwise and
    F(2x2) kernels, 2e-3 for float32 F(4x4) and F(6x6), 5e-3 for float16 storage."""
    if half:
        return 5e-3
    return 2e-3 if kind in (3, 5) else 1e-4


def applicable_kinds(layer, half=False):
    """Kernel kinds that can run the layer (F(6x6) exists in float32 only)."""
    kinds = [0]
    taps_ok = layer.r * layer.s <= (64 if half else 128)
    if layer.groups > 1 and taps_ok and layer.groups <= 64 and (not half or layer.r * layer.s == 1 or layer.cg % 32 == 0):
        kinds.append(1)          # grouped convolution on the matrix cores: one panel block per group
    if layer.groups == 1:
        if taps_ok:
            kinds.append(1)
        if layer.winograd_ok:
            # float16 Winograd is offered from 16 input channels up; F(6x6) in float32 only
            kinds += ([2, 3] if layer.c >= 16 else []) if half else [2, 3, 5]
    if layer.is_depthwise and layer.r == layer.s and layer.r in (3, 5) and layer.stride in (1, 2):
        kinds.append(4)
    return kinds


def oracle_transformed(w: np.ndarray, kind: int, half: bool, groups: int = 1):
    """Expected transformed-weight buffer (and, for Winograd, the float64 values + abs bound)."""
    if kind == 0:
        return w.reshape(-1).copy(), None
    if kind == 1:
        return OL.pack_gemm(w, half, groups), None
    if kind == 4:
        return OL.pack_depthwise(w, half), None
    var = wino_variant(kind, half)
    U = OW.transform_weights(w, var)
    _, G, _ = OW.matrices(var)
    bound = np.einsum("ur,kcrs,vs->uvkc", np.abs(G), np.abs(w.astype(np.float64)), np.abs(G))
    return OL.pack_wino(U, half, dtype=np.float64), OL.pack_wino(bound, half, dtype=np.float64)


def gpu_transform(nnv, torch, layer, kind, half, w_np):
    desc = nnv.make_desc(layer, nnv.F16 if half else nnv.F32)
    dev = torch.device("cuda:0")
    wd = torch.from_numpy(np.ascontiguousarray(w_np)).to(dev)
    nbytes = nnv.nnv_transformed_bytes(desc, kind)
    # canaries around the output catch writes outside the buffer
    pad = 256
    buf = torch.full((nbytes + 2 * pad,), 0xA5, dtype=torch.uint8, device=dev)
    wt = buf[pad:pad + nbytes]
    nnv.nnv_transform_weights(desc, kind, wd, wt)
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    assert (host[:pad] == 0xA5).all() and (host[pad + nbytes:] == 0xA5).all(), "write outside w_tx"
    dt = np.float32 if (kind == 0 or not half) else np.float16
    return host[pad:pad + nbytes].view(dt).copy(), wt, wd, desc


def gpu_forward(nnv, torch, layer, kind, half, w_np, x_np, bias_np=None, relu=False):
    """Transform + forward on the GPU; returns y as float64 numpy."""
    dev = torch.device("cuda:0")
    _, wt, _, desc = gpu_transform(nnv, torch, layer, kind, half, w_np)
    xt = torch.from_numpy(np.ascontiguousarray(x_np)).to(dev)
    if half:
        xt = xt.half()
    bias = None if bias_np is None else torch.from_numpy(bias_np.astype(np.float32)).to(dev)
    ws_bytes = nnv.nnv_workspace_bytes(desc, kind)
    pad = 256
    wsbuf = torch.full((ws_bytes + 2 * pad,), 0x5A, dtype=torch.uint8, device=dev)
    ws = wsbuf[pad:pad + ws_bytes] if ws_bytes else None
    numel = layer.n * layer.k * layer.p * layer.q
    esz = 2 if half else 4
    ybuf = torch.full((numel * esz + 2 * pad,), 0x7F, dtype=torch.uint8, device=dev)
    y = ybuf[pad:pad + numel * esz]
    (nnv.nnv_conv_forward_relu if relu else nnv.nnv_conv_forward)(desc, kind, xt, wt, bias, y, ws, ws_bytes)
    torch.cuda.synchronize()
    yh = ybuf.cpu().numpy()
    assert (yh[:pad] == 0x7F).all() and (yh[pad + numel * esz:] == 0x7F).all(), "write outside y"
    if ws_bytes:
        wh = wsbuf.cpu().numpy()
        assert (wh[:pad] == 0x5A).all() and (wh[pad + ws_bytes:] == 0x5A).all(), "write outside workspace"
    out = yh[pad:pad + numel * esz].view(np.float16 if half else np.float32)
    return out.astype(np.float64).reshape(layer.n, layer.k, layer.p, layer.q)


def oracle_forward(layer, half, w_np, x_np, bias_np=None):
    x = x_np.astype(np.float16).astype(np.float64) if half else x_np.astype(np.float64)
    return conv2d_direct(x, w_np.astype(np.float64), layer.stride, layer.pad, layer.groups, bias_np)


def oracle_forward_stored(layer, kind, w_np, x_np, bias_np=None):
    """The float16 Winograd variant with its storage roundings (U, V, y in half precision)."""
    return OW.conv2d_winograd_stored(x_np, w_np, wino_variant(kind, True), layer.pad, bias_np, store=np.float16)
