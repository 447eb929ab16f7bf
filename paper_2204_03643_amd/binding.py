"""ctypes binding: argument marshalling only.  Function names match include/tvprox.h."""
from __future__ import annotations

import ctypes

from . import build as _build

_i64 = ctypes.c_int64
_vp = ctypes.c_void_p


class tv_rows(ctypes.Structure):
    _fields_ = [("n_outer", _i64), ("outer_stride", _i64), ("n_inner", _i64),
                ("inner_stride", _i64), ("length", _i64), ("elem_stride", _i64)]


class tv_lambda(ctypes.Structure):
    _fields_ = [("lam", _vp), ("count", _i64), ("div", _i64)]


class tv_fwd_extra(ctypes.Structure):
    _fields_ = [("info", _vp), ("seg", _vp), ("ws", _vp), ("ws_bytes", ctypes.c_size_t),
                ("flags", ctypes.c_uint32)]


TV_FWD_ORDER_READY = 1
TV_FWD_PARALLEL_SEARCH = 2


class TVError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__("tvprox: %s (status %d)" % (status_str(status), status))


_lib = None


def lib() -> ctypes.CDLL:
    """Loads libtvprox.so.  A library that is missing, or that was built from other sources than
    the tree now holds, is built first (hipcc); if that fails this raises: an old library is
    never loaded silently, and there is no other path."""
    global _lib
    if _lib is None:
        if _build.is_stale():
            _build.build_library()
        # PyTorch ships a HIP runtime of its own.  Loaded first, it is the one this library binds
        # to as well, and device pointers and streams mean the same thing to both; in the other
        # order the process ends up with the system's runtime underneath PyTorch's libraries,
        # and every kernel launch of this library fails.
        import torch  # noqa: F401
        L = ctypes.CDLL(_build.LIB)
        L.tv_dispatch_name.argtypes = [ctypes.c_int]
        L.tv_dispatch_name.restype = ctypes.c_char_p
        L.tv_dispatch_threshold.argtypes = [ctypes.c_char_p]
        L.tv_dispatch_threshold.restype = _i64
        L.tv_dispatch_override.argtypes = [ctypes.c_char_p, _i64]
        L.tv_dispatch_override.restype = ctypes.c_int
        L.tv_status_str.argtypes = [ctypes.c_int]
        L.tv_status_str.restype = ctypes.c_char_p
        L.tv1d_prox_fwd.argtypes = [_vp, _vp, tv_rows, tv_lambda, _vp]
        L.tv1d_prox_fwd.restype = ctypes.c_int
        L.tv1d_prox_fwd_info.argtypes = [_vp, _vp, _vp, tv_rows, tv_lambda, _vp]
        L.tv1d_prox_fwd_info.restype = ctypes.c_int
        L.tv1d_fwd_steps_floats_per_row.argtypes = [_i64]
        L.tv1d_fwd_steps_floats_per_row.restype = ctypes.c_size_t
        L.tv1d_prox_fwd_steps.argtypes = [_vp, _vp, _vp, _vp, _i64, tv_rows, tv_lambda, _vp]
        L.tv1d_prox_fwd_steps.restype = ctypes.c_int
        L.tv1d_prox_bwd.argtypes = [_vp, _vp, _vp, _vp, tv_rows, tv_lambda, _vp, ctypes.c_size_t, _vp]
        L.tv1d_prox_bwd.restype = ctypes.c_int
        L.tv1d_prox_bwd_noalloc.argtypes = [_vp, _vp, _vp, _vp, tv_rows, tv_lambda, _vp]
        L.tv1d_prox_bwd_noalloc.restype = ctypes.c_int
        L.tv1d_prox_fwd_seg.argtypes = [_vp, _vp, _vp, tv_rows, tv_lambda, _vp]
        L.tv1d_prox_fwd_seg.restype = ctypes.c_int
        L.tv1d_prox_fwd_ex.argtypes = [_vp, _vp, tv_rows, tv_lambda, tv_fwd_extra, _vp]
        L.tv1d_prox_fwd_ex.restype = ctypes.c_int
        L.tv1d_fwd_workspace_bytes.argtypes = [tv_rows, tv_lambda]
        L.tv1d_fwd_workspace_bytes.restype = ctypes.c_size_t
        L.tv1d_prox_bwd_seg.argtypes = [_vp, _vp, _vp, _vp, tv_rows, tv_lambda, _vp, ctypes.c_size_t, _vp]
        L.tv1d_prox_bwd_seg.restype = ctypes.c_int
        L.tv1d_prox_fwd_seg_bf16.argtypes = [_vp, _vp, _vp, tv_rows, tv_lambda, _vp, ctypes.c_size_t, _vp]
        L.tv1d_prox_fwd_seg_bf16.restype = ctypes.c_int
        L.tv1d_prox_bwd_seg_bf16.argtypes = [_vp, _vp, _vp, _vp, tv_rows, tv_lambda, _vp, ctypes.c_size_t, _vp]
        L.tv1d_prox_bwd_seg_bf16.restype = ctypes.c_int
        L.tv1d_bwd_workspace_bytes.argtypes = [tv_rows, tv_lambda]
        L.tv1d_bwd_workspace_bytes.restype = ctypes.c_size_t
        L.tv2d_workspace_bytes.argtypes = [_i64, _i64, _i64, ctypes.c_int]
        L.tv2d_workspace_bytes.restype = ctypes.c_size_t
        L.tv2d_prox_fwd.argtypes = [_vp, _vp, _i64, _i64, _i64, tv_lambda, ctypes.c_int, _vp,
                                    ctypes.c_size_t, _vp]
        L.tv2d_prox_fwd.restype = ctypes.c_int
        L.tv2d_prox_bwd.argtypes = [_vp, _vp, _vp, _i64, _i64, _i64, tv_lambda, ctypes.c_int, _vp,
                                    ctypes.c_size_t, _vp]
        L.tv2d_prox_bwd.restype = ctypes.c_int
        L.tv2d_prox_fwd_bf16.argtypes = L.tv2d_prox_fwd.argtypes
        L.tv2d_prox_fwd_bf16.restype = ctypes.c_int
        L.tv2d_prox_bwd_bf16.argtypes = L.tv2d_prox_bwd.argtypes
        L.tv2d_prox_bwd_bf16.restype = ctypes.c_int
        _lib = L
    return _lib


def status_str(status: int) -> str:
    return lib().tv_status_str(int(status)).decode()


def tv_dispatch_thresholds() -> dict:
    """{name: value} of every dispatch threshold of the library."""
    out, i = {}, 0
    while True:
        name = lib().tv_dispatch_name(i)
        if name is None:
            return out
        out[name.decode()] = int(lib().tv_dispatch_threshold(name))
        i += 1


def tv_dispatch_threshold(name: str) -> int:
    return int(lib().tv_dispatch_threshold(name.encode()))


def tv_dispatch_override(name: str, value: int):
    _check(lib().tv_dispatch_override(name.encode(), int(value)))


def _ptr(t):
    """Device pointer of a torch tensor (or a raw integer address / None)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _check(st: int):
    if st != 0:
        raise TVError(st)


def rows_along(shape, axis: int) -> tv_rows:
    """tv_rows describing the rows of a contiguous tensor of `shape` taken along `axis`;
    row ids run in C order over the remaining axes."""
    nd = len(shape)
    axis %= nd
    n = int(shape[axis])
    es = 1
    for d in shape[axis + 1:]:
        es *= int(d)
    outer = 1
    for d in shape[:axis]:
        outer *= int(d)
    return tv_rows(outer, n * es, es, 1, n, es)


def tv1d_prox_fwd(y, x, rows: tv_rows, lam: tv_lambda, stream=None):
    _check(lib().tv1d_prox_fwd(_ptr(y), _ptr(x), rows, lam, _stream(stream)))


def tv1d_prox_fwd_info(y, x, info, rows: tv_rows, lam: tv_lambda, stream=None):
    _check(lib().tv1d_prox_fwd_info(_ptr(y), _ptr(x), _ptr(info), rows, lam, _stream(stream)))


def tv1d_fwd_steps_floats_per_row(length: int) -> int:
    return int(lib().tv1d_fwd_steps_floats_per_row(int(length)))


def tv1d_prox_fwd_steps(y, x, info, record, record_rows: int, rows: tv_rows, lam: tv_lambda, stream=None):
    _check(lib().tv1d_prox_fwd_steps(_ptr(y), _ptr(x), _ptr(info), _ptr(record), int(record_rows), rows, lam,
                                     _stream(stream)))


def tv1d_bwd_workspace_bytes(rows: tv_rows, lam: tv_lambda) -> int:
    return int(lib().tv1d_bwd_workspace_bytes(rows, lam))


def tv1d_prox_bwd(g_up, x, grad_y, grad_lam, rows: tv_rows, lam: tv_lambda, ws, ws_bytes: int,
                  stream=None):
    _check(lib().tv1d_prox_bwd(_ptr(g_up), _ptr(x), _ptr(grad_y), _ptr(grad_lam), rows, lam,
                               _ptr(ws), int(ws_bytes), _stream(stream)))


def tv1d_prox_bwd_noalloc(g_up, x, grad_y, grad_lam, rows: tv_rows, lam: tv_lambda, stream=None):
    _check(lib().tv1d_prox_bwd_noalloc(_ptr(g_up), _ptr(x), _ptr(grad_y), _ptr(grad_lam), rows, lam,
                                       _stream(stream)))


def tv1d_prox_fwd_seg(y, x, seg, rows: tv_rows, lam: tv_lambda, stream=None):
    _check(lib().tv1d_prox_fwd_seg(_ptr(y), _ptr(x), _ptr(seg), rows, lam, _stream(stream)))


def tv1d_fwd_workspace_bytes(rows: tv_rows, lam: tv_lambda) -> int:
    return int(lib().tv1d_fwd_workspace_bytes(rows, lam))


def tv1d_prox_fwd_ex(y, x, rows: tv_rows, lam: tv_lambda, info=None, seg=None, ws=None,
                     ws_bytes: int = 0, stream=None, flags: int = 0):
    extra = tv_fwd_extra(_ptr(info), _ptr(seg), _ptr(ws), int(ws_bytes), int(flags))
    _check(lib().tv1d_prox_fwd_ex(_ptr(y), _ptr(x), rows, lam, extra, _stream(stream)))


def tv1d_prox_bwd_seg(g_up, seg, grad_y, grad_lam, rows: tv_rows, lam: tv_lambda, ws, ws_bytes: int,
                      stream=None):
    _check(lib().tv1d_prox_bwd_seg(_ptr(g_up), _ptr(seg), _ptr(grad_y), _ptr(grad_lam), rows, lam,
                                   _ptr(ws), int(ws_bytes), _stream(stream)))


def tv1d_prox_fwd_seg_bf16(y, x, seg, rows: tv_rows, lam: tv_lambda, ws=None, ws_bytes: int = 0, stream=None):
    _check(lib().tv1d_prox_fwd_seg_bf16(_ptr(y), _ptr(x), _ptr(seg), rows, lam, _ptr(ws), int(ws_bytes),
                                        _stream(stream)))


def tv1d_prox_bwd_seg_bf16(g_up, seg, grad_y, grad_lam, rows: tv_rows, lam: tv_lambda, ws, ws_bytes: int,
                           stream=None):
    _check(lib().tv1d_prox_bwd_seg_bf16(_ptr(g_up), _ptr(seg), _ptr(grad_y), _ptr(grad_lam), rows, lam,
                                        _ptr(ws), int(ws_bytes), _stream(stream)))


def tv2d_workspace_bytes(planes: int, H: int, W: int, sweeps: int) -> int:
    return int(lib().tv2d_workspace_bytes(planes, H, W, sweeps))


def tv2d_prox_fwd(y, x, planes, H, W, lam: tv_lambda, sweeps, ws, ws_bytes, stream=None):
    _check(lib().tv2d_prox_fwd(_ptr(y), _ptr(x), planes, H, W, lam, int(sweeps), _ptr(ws),
                               int(ws_bytes), _stream(stream)))


def tv2d_prox_bwd(g_up, grad_y, grad_lam, planes, H, W, lam: tv_lambda, sweeps, ws, ws_bytes,
                  stream=None):
    _check(lib().tv2d_prox_bwd(_ptr(g_up), _ptr(grad_y), _ptr(grad_lam), planes, H, W, lam,
                               int(sweeps), _ptr(ws), int(ws_bytes), _stream(stream)))


def tv2d_prox_fwd_bf16(y, x, planes, H, W, lam: tv_lambda, sweeps, ws, ws_bytes, stream=None):
    _check(lib().tv2d_prox_fwd_bf16(_ptr(y), _ptr(x), planes, H, W, lam, int(sweeps), _ptr(ws),
                                    int(ws_bytes), _stream(stream)))


def tv2d_prox_bwd_bf16(g_up, grad_y, grad_lam, planes, H, W, lam: tv_lambda, sweeps, ws, ws_bytes,
                       stream=None):
    _check(lib().tv2d_prox_bwd_bf16(_ptr(g_up), _ptr(grad_y), _ptr(grad_lam), planes, H, W, lam,
                                    int(sweeps), _ptr(ws), int(ws_bytes), _stream(stream)))
