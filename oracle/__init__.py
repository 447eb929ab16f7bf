"""CPU oracle for the TV proximal operator -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``tvprox_oracle.c`` (plain double-precision C).  Only
``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  The product path (the HIP library under
``paper_2204_03643_amd``) shares no code with it and never routes through it.

Operator (paper Eq. 1, with this build's letters: y input, x output):
    x* = argmin_x 1/2 ||x - y||^2 + lam * sum_k |x[k+1] - x[k]|
Backward: paper Eq. 5-6, evaluated as per-segment averaging.
2D: K sweeps of paper Alg. 1 (proximal Dykstra) and its reverse sweep.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tvprox_oracle.c")
_LIB = os.path.join(_HERE, "libtvprox_oracle.so")
_lib = None

_D = ctypes.POINTER(ctypes.c_double)
_L = ctypes.c_long


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over rows; no hand tuning)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.tvo_prox1d.argtypes = [_D, _D, _L, _L, ctypes.c_double]
        lib.tvo_prox1d.restype = ctypes.c_int
        lib.tvo_prox1d_bwd.argtypes = [_D, _D, _D, _L, _L]
        lib.tvo_prox1d_bwd.restype = ctypes.c_double
        lib.tvo_prox1d_batch.argtypes = [_D, _D, _L, _L, _L, _L, _L, _L, _D, _L, _L]
        lib.tvo_prox1d_batch.restype = ctypes.c_int
        lib.tvo_prox1d_bwd_batch.argtypes = [_D, _D, _D, _D, _L, _L, _L, _L, _L, _L, _L, _L]
        lib.tvo_prox1d_bwd_batch.restype = None
        lib.tvo_prox2d_fwd.argtypes = [_D, _D, _L, _L, _L, _D, _L, ctypes.c_int, _D]
        lib.tvo_prox2d_fwd.restype = ctypes.c_int
        lib.tvo_prox2d_bwd.argtypes = [_D, _D, _D, _L, _L, _L, _L, ctypes.c_int, _D]
        lib.tvo_prox2d_bwd.restype = None
        lib.tvo_num_threads.argtypes = []
        lib.tvo_num_threads.restype = ctypes.c_int
        lib.tvo_set_num_threads.argtypes = [ctypes.c_int]
        lib.tvo_set_num_threads.restype = None
        _lib = lib
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(_D)


def _c64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def num_threads() -> int:
    return int(_load().tvo_num_threads())


def set_num_threads(n: int) -> None:
    """Threads the batch functions use from now on (for timing; results do not depend on it)."""
    _load().tvo_set_num_threads(int(n))


def prox1d(y, lam: float) -> np.ndarray:
    """Exact minimiser of paper Eq. 1 for one row (double)."""
    y = _c64(y)
    if y.ndim != 1:
        raise ValueError("prox1d takes one row")
    x = np.empty_like(y)
    if y.size and _load().tvo_prox1d(_p(y), _p(x), y.size, 1, float(lam)):
        raise ValueError("invalid arguments (need n >= 1, finite lam >= 0)")
    return x


def prox1d_bwd(g_up, x):
    """(grad_y, grad_lam) for one row from the forward output x (paper Eq. 5-6)."""
    g = _c64(g_up)
    x = _c64(x)
    gy = np.empty_like(g)
    gl = _load().tvo_prox1d_bwd(_p(g), _p(x), _p(gy), g.size, 1) if g.size else 0.0
    return gy, float(gl)


def _rows_layout(shape, axis):
    """View an array of `shape` (C order) as rows along `axis`:
    returns (n_outer, outer_stride, n_inner, inner_stride, n, es)."""
    nd = len(shape)
    axis %= nd
    n = shape[axis]
    es = int(np.prod(shape[axis + 1:], dtype=np.int64))
    n_outer = int(np.prod(shape[:axis], dtype=np.int64))
    return n_outer, n * es, es, 1, n, es


def _lam_arr(lam) -> np.ndarray:
    lam = _c64(np.atleast_1d(lam)).ravel()
    if not np.all(np.isfinite(lam)) or np.any(lam < 0):
        raise ValueError("lam must be finite and >= 0")
    return lam


def prox1d_batch(y, lam, axis: int = -1, lam_div: int = 1) -> np.ndarray:
    """Rows of `y` along `axis`; row id r (C order over the other axes) uses
    lam[(r // lam_div) % len(lam)]."""
    y = _c64(y)
    lam = _lam_arr(lam)
    x = np.empty_like(y)
    if y.size == 0:
        return x
    no, os_, ni, is_, n, es = _rows_layout(y.shape, axis)
    if _load().tvo_prox1d_batch(_p(y), _p(x), no, os_, ni, is_, n, es, _p(lam), lam.size, lam_div):
        raise ValueError("invalid arguments")
    return x


def prox1d_bwd_batch(g_up, x, lam_count: int = 1, axis: int = -1, lam_div: int = 1):
    """(grad_y, grad_lam[lam_count]) for a batch laid out like prox1d_batch's."""
    g = _c64(g_up)
    x = _c64(x)
    assert g.shape == x.shape
    gy = np.empty_like(g)
    gl = np.zeros(lam_count, dtype=np.float64)
    if g.size:
        no, os_, ni, is_, n, es = _rows_layout(g.shape, axis)
        _load().tvo_prox1d_bwd_batch(_p(g), _p(x), _p(gy), _p(gl), no, os_, ni, is_, n, es,
                                     lam_count, lam_div)
    return gy, gl


def prox2d_fwd(y, lam, sweeps: int):
    """K sweeps of paper Alg. 1 on y[..., H, W]; plane p uses lam[p % len(lam)].
    Returns (x, saved) where saved holds every pass's output for prox2d_bwd."""
    y = _c64(y)
    lam = _lam_arr(lam)
    H, W = y.shape[-2:]
    planes = y.size // (H * W) if H * W else 0
    x = np.empty_like(y)
    saved = np.empty((2 * sweeps,) + y.shape, dtype=np.float64)
    if y.size and _load().tvo_prox2d_fwd(_p(y), _p(x), planes, H, W, _p(lam), lam.size,
                                         int(sweeps), _p(saved)):
        raise ValueError("invalid arguments")
    return x, saved


def prox2d_bwd(g_up, saved, lam_count: int, sweeps: int):
    """Reverse sweep through Alg. 1: (grad_y, grad_lam[lam_count])."""
    g = _c64(g_up)
    H, W = g.shape[-2:]
    planes = g.size // (H * W) if H * W else 0
    gy = np.empty_like(g)
    gl = np.zeros(lam_count, dtype=np.float64)
    if g.size:
        _load().tvo_prox2d_bwd(_p(g), _p(gy), _p(gl), planes, H, W, lam_count, int(sweeps),
                               _p(np.ascontiguousarray(saved)))
    return gy, gl
