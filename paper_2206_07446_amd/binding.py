"""ctypes binding of libnnv.so: the same entry points as include/nnv.h, argument
marshalling only.  torch supplies device memory and the stream handle."""
from __future__ import annotations

import ctypes
import os
from ctypes import c_char_p, c_double, c_int, c_int32, c_size_t, c_void_p, POINTER, Structure, byref

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libnnv.so")

DIRECT, IM2COL_GEMM, WINO_F2, WINO_F4, DEPTHWISE, WINO_F6 = range(6)
KINDS = {"direct": DIRECT, "im2col_gemm": IM2COL_GEMM, "wino_f2": WINO_F2, "wino_f4": WINO_F4,
         "depthwise": DEPTHWISE, "wino_f6": WINO_F6}
F32, F16 = 0, 1

EXPORTS = ("nnv_layout_version", "nnv_status_string", "nnv_last_hip_error", "nnv_kind_supported",
           "nnv_transformed_bytes", "nnv_workspace_bytes", "nnv_transform_weights",
           "nnv_transform_weights_grouped", "nnv_conv_forward", "nnv_conv_forward_relu", "nnv_conv_forward_static", "nnv_conv_forward_grouped",
           "nnv_conv_forward_grouped_workspace_bytes", "nnv_time_layer", "nnv_cold_stack", "nnv_cache_write",
           "nnv_cache_read")


class NnvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        text = nnv_status_string(status)
        if status == -6:
            text += ": " + nnv_last_hip_error()
        if status == -8:
            text += ": " + os.strerror(ctypes.get_errno())
        super().__init__(f"{where}: {text} ({status})")


class ConvDesc(Structure):
    _fields_ = [(n, c_int32) for n in ("n", "c", "h", "w", "k", "r", "s", "stride_h", "stride_w",
                                       "pad_h", "pad_w", "groups", "dtype")]


class Timing(Structure):
    _fields_ = [(n, c_double) for n in ("transform_ms", "forward_ms", "transform_bytes", "forward_bytes",
                                        "forward_flops", "direct_equiv_flops")]


class CacheIo(Structure):
    _fields_ = [("total_ms", c_double), ("file_ms", c_double), ("bytes", c_double), ("direct_io", c_int32)]


_lib = None


def load():
    """Load libnnv.so (building it first only if it does not exist).  torch is imported
    before the library so that both share one HIP runtime."""
    global _lib
    if _lib is not None:
        return _lib
    import torch  # noqa: F401  (loads the HIP runtime the library binds to)
    if not os.path.exists(LIB_PATH):
        from .build import build
        build()
    lib = ctypes.CDLL(LIB_PATH, use_errno=True)
    lib.nnv_layout_version.restype = c_int
    lib.nnv_status_string.restype = c_char_p
    lib.nnv_status_string.argtypes = [c_int]
    lib.nnv_last_hip_error.restype = c_char_p
    lib.nnv_kind_supported.restype = c_int
    lib.nnv_kind_supported.argtypes = [POINTER(ConvDesc), c_int]
    lib.nnv_transformed_bytes.restype = c_size_t
    lib.nnv_transformed_bytes.argtypes = [POINTER(ConvDesc), c_int]
    lib.nnv_workspace_bytes.restype = c_size_t
    lib.nnv_workspace_bytes.argtypes = [POINTER(ConvDesc), c_int]
    lib.nnv_transform_weights.restype = c_int
    lib.nnv_transform_weights.argtypes = [POINTER(ConvDesc), c_int, c_void_p, c_void_p, c_void_p]
    lib.nnv_transform_weights_grouped.restype = c_int
    lib.nnv_transform_weights_grouped.argtypes = [c_int, POINTER(ConvDesc), POINTER(c_int), POINTER(c_void_p),
                                                  POINTER(c_void_p), c_void_p]
    lib.nnv_conv_forward.restype = c_int
    lib.nnv_conv_forward.argtypes = [POINTER(ConvDesc), c_int, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                     c_size_t, c_void_p]
    lib.nnv_conv_forward_relu.restype = c_int
    lib.nnv_conv_forward_relu.argtypes = lib.nnv_conv_forward.argtypes
    lib.nnv_conv_forward_grouped_workspace_bytes.restype = c_size_t
    lib.nnv_conv_forward_grouped_workspace_bytes.argtypes = [c_int, POINTER(ConvDesc), POINTER(c_int)]
    lib.nnv_conv_forward_grouped.restype = c_int
    lib.nnv_conv_forward_grouped.argtypes = [c_int, POINTER(ConvDesc), POINTER(c_int), POINTER(c_void_p), POINTER(c_void_p),
                                             POINTER(c_void_p), POINTER(c_void_p), c_void_p, c_size_t, ctypes.c_uint, c_void_p]
    lib.nnv_conv_forward_static.restype = c_int
    lib.nnv_conv_forward_static.argtypes = [POINTER(ConvDesc), c_int, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.nnv_time_layer.restype = c_int
    lib.nnv_time_layer.argtypes = [POINTER(ConvDesc), c_int, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                   c_size_t, c_void_p, c_size_t, c_int, c_int, c_void_p, POINTER(Timing)]
    lib.nnv_cold_stack.restype = c_int
    lib.nnv_cold_stack.argtypes = [c_int, POINTER(ConvDesc), POINTER(c_int), POINTER(c_void_p), POINTER(c_void_p),
                                   POINTER(c_void_p), POINTER(c_void_p), c_void_p, c_size_t, c_int, c_void_p, c_void_p]
    lib.nnv_cache_write.restype = c_int
    lib.nnv_cache_write.argtypes = [c_char_p, POINTER(ConvDesc), c_int, c_void_p, c_void_p]
    lib.nnv_cache_read.restype = c_int
    lib.nnv_cache_read.argtypes = [c_char_p, POINTER(ConvDesc), c_int, c_void_p, c_int, c_void_p, POINTER(CacheIo)]
    _lib = lib
    return lib


def make_desc(layer, dtype: int = F32) -> ConvDesc:
    """ConvDesc from any object with c,h,w,k,r,s,stride,pad,groups,n attributes."""
    return ConvDesc(layer.n, layer.c, layer.h, layer.w, layer.k, layer.r, layer.s, layer.stride, layer.stride,
                    layer.pad, layer.pad, layer.groups, dtype)


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return c_void_p(t)
    return c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    return c_void_p(stream)


def _check(rc: int, where: str):
    if rc < 0:
        raise NnvError(rc, where)
    return rc


def nnv_layout_version() -> int:
    return load().nnv_layout_version()


def nnv_status_string(status: int) -> str:
    return load().nnv_status_string(status).decode()


def nnv_last_hip_error() -> str:
    return load().nnv_last_hip_error().decode()


def nnv_kind_supported(desc: ConvDesc, kind: int) -> bool:
    return bool(_check(load().nnv_kind_supported(byref(desc), kind), "nnv_kind_supported"))


def nnv_transformed_bytes(desc: ConvDesc, kind: int) -> int:
    return int(load().nnv_transformed_bytes(byref(desc), kind))


def nnv_workspace_bytes(desc: ConvDesc, kind: int) -> int:
    return int(load().nnv_workspace_bytes(byref(desc), kind))


def nnv_transform_weights(desc: ConvDesc, kind: int, w_raw, w_tx, stream=None) -> None:
    _check(load().nnv_transform_weights(byref(desc), kind, _ptr(w_raw), _ptr(w_tx), _stream(stream)),
           "nnv_transform_weights")


def nnv_transform_weights_grouped(descs, kinds, w_raw, w_tx, stream=None) -> None:
    n = len(descs)
    d = (ConvDesc * n)(*descs)
    k = (c_int * n)(*kinds)
    src = (c_void_p * n)(*[t if isinstance(t, int) else t.data_ptr() for t in w_raw])
    dst = (c_void_p * n)(*[t if isinstance(t, int) else t.data_ptr() for t in w_tx])
    _check(load().nnv_transform_weights_grouped(n, d, k, src, dst, _stream(stream)), "nnv_transform_weights_grouped")


def nnv_conv_forward(desc: ConvDesc, kind: int, x, w_tx, bias, y, workspace, workspace_bytes=None, stream=None) -> None:
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().nnv_conv_forward(byref(desc), kind, _ptr(x), _ptr(w_tx), _ptr(bias), _ptr(y), _ptr(workspace),
                                   workspace_bytes, _stream(stream)), "nnv_conv_forward")


def nnv_conv_forward_relu(desc: ConvDesc, kind: int, x, w_tx, bias, y, workspace, workspace_bytes=None, stream=None) -> None:
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().nnv_conv_forward_relu(byref(desc), kind, _ptr(x), _ptr(w_tx), _ptr(bias), _ptr(y), _ptr(workspace),
                                        workspace_bytes, _stream(stream)), "nnv_conv_forward_relu")


FORWARD_RELU = 1


def nnv_conv_forward_grouped_workspace_bytes(descs, kinds) -> int:
    n = len(descs)
    return int(load().nnv_conv_forward_grouped_workspace_bytes(n, (ConvDesc * n)(*descs), (c_int * n)(*kinds)))


def nnv_conv_forward_grouped(descs, kinds, x, w_tx, bias, y, workspace, workspace_bytes=None, flags=0, stream=None) -> None:
    """bias: None, or a list with a tensor or None per layer."""
    n = len(descs)
    arr = lambda ts: (c_void_p * n)(*[None if t is None else (t if isinstance(t, int) else t.data_ptr()) for t in ts])
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().nnv_conv_forward_grouped(n, (ConvDesc * n)(*descs), (c_int * n)(*kinds), arr(x), arr(w_tx),
                                           None if bias is None else arr(bias), arr(y), _ptr(workspace), workspace_bytes,
                                           flags, _stream(stream)), "nnv_conv_forward_grouped")


STATIC_SCRATCH_BYTES = 64 << 20


def nnv_conv_forward_static(desc: ConvDesc, kind: int, x, w_tx, bias, y, stream=None) -> None:
    _check(load().nnv_conv_forward_static(byref(desc), kind, _ptr(x), _ptr(w_tx), _ptr(bias), _ptr(y), _stream(stream)),
           "nnv_conv_forward_static")


def nnv_time_layer(desc: ConvDesc, kind: int, w_raw, w_tx, x, y, workspace, flush=None, warmup=2, reps=10,
                   stream=None) -> Timing:
    out = Timing()
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    fl_bytes = 0 if flush is None else flush.numel() * flush.element_size()
    _check(load().nnv_time_layer(byref(desc), kind, _ptr(w_raw), _ptr(w_tx), _ptr(x), _ptr(y), _ptr(workspace),
                                 ws_bytes, _ptr(flush), fl_bytes, warmup, reps, _stream(stream), byref(out)),
           "nnv_time_layer")
    return out


def nnv_cache_write(path: str, desc: ConvDesc, kind: int, w_tx, stream=None) -> None:
    _check(load().nnv_cache_write(os.fsencode(path), byref(desc), kind, _ptr(w_tx), _stream(stream)), "nnv_cache_write")


def nnv_cache_read(path: str, desc: ConvDesc, kind: int, w_tx, verify: bool = False, stream=None) -> CacheIo:
    out = CacheIo()
    _check(load().nnv_cache_read(os.fsencode(path), byref(desc), kind, _ptr(w_tx), int(verify), _stream(stream),
                                 byref(out)), "nnv_cache_read")
    return out


def nnv_cold_stack(descs, kinds, w_raw, w_tx, x, y, workspace, stage_layers=1, stream_exec=None, stream_tx=None) -> None:
    """stream_tx=None runs both operations on stream_exec (the unpipelined order)."""
    n = len(descs)
    arr = lambda ts: (c_void_p * n)(*[t if isinstance(t, int) else t.data_ptr() for t in ts])
    se = _stream(stream_exec)
    stx = se if stream_tx is None else _stream(stream_tx)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().nnv_cold_stack(n, (ConvDesc * n)(*descs), (c_int * n)(*kinds), arr(w_raw), arr(w_tx), arr(x), arr(y),
                                 _ptr(workspace), ws_bytes, stage_layers, se, stx), "nnv_cold_stack")
