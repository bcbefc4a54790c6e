"""CPU oracle for the streaming vector kernels (Table 1: Copy, Mul, Add, Triad, Dot).

TEST INFRASTRUCTURE.  Only tests/, the smoke check and the benchmark's
CPU-baseline leg import this package; the GPU library and its Python binding
never do.  The arithmetic lives in oracle.cpp (plain single-threaded C++
loops); this file only marshals numpy arrays into it through ctypes.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None

_CT = {np.dtype(np.float64): ("f64", ctypes.c_double), np.dtype(np.float32): ("f32", ctypes.c_float)}


def _lib():
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        lib = ctypes.CDLL(path)
        sz = ctypes.c_size_t
        vp = ctypes.c_void_p
        dbl = ctypes.c_double
        for suf in ("f64", "f32"):
            getattr(lib, "oracle_copy_" + suf).argtypes = [vp, vp, sz]
            getattr(lib, "oracle_copy_" + suf).restype = None
            getattr(lib, "oracle_scale_" + suf).argtypes = [vp, vp, dbl, sz]
            getattr(lib, "oracle_scale_" + suf).restype = None
            getattr(lib, "oracle_add_" + suf).argtypes = [vp, vp, vp, sz]
            getattr(lib, "oracle_add_" + suf).restype = None
            getattr(lib, "oracle_triad_" + suf).argtypes = [vp, vp, vp, dbl, sz]
            getattr(lib, "oracle_triad_" + suf).restype = None
            getattr(lib, "oracle_dot_" + suf).argtypes = [vp, vp, sz, vp]
            getattr(lib, "oracle_dot_" + suf).restype = dbl
            getattr(lib, "oracle_dot_plain_" + suf).argtypes = [vp, vp, sz]
            getattr(lib, "oracle_dot_plain_" + suf).restype = dbl
            getattr(lib, "oracle_dot_abs_" + suf).argtypes = [vp, vp, sz]
            getattr(lib, "oracle_dot_abs_" + suf).restype = dbl
            getattr(lib, "oracle_lds_stream_" + suf).argtypes = [vp, vp, dbl, sz, ctypes.c_uint]
            getattr(lib, "oracle_lds_stream_" + suf).restype = ctypes.c_int
        _LIB = lib
    return _LIB


def _chk(*arrs):
    """All arrays: 1-D, C-contiguous, same dtype (f64 or f32), same length."""
    a0 = arrs[0]
    if a0.dtype not in _CT:
        raise TypeError("oracle supports float64 and float32 only, got %s" % a0.dtype)
    for x in arrs:
        if not isinstance(x, np.ndarray) or x.ndim != 1 or not x.flags.c_contiguous:
            raise ValueError("oracle arrays must be 1-D C-contiguous numpy arrays")
        if x.dtype != a0.dtype or x.shape != a0.shape:
            raise ValueError("oracle arrays must share dtype and length")
    return _CT[a0.dtype][0], a0.shape[0]


def _p(x):
    return ctypes.c_void_p(x.ctypes.data)


def copy(a, c):
    """c[i] = a[i]."""
    suf, n = _chk(a, c)
    getattr(_lib(), "oracle_copy_" + suf)(_p(a), _p(c), n)


def scale(b, c, s):
    """b[i] = s * c[i]  (the paper's Mul kernel); s is rounded once to the array type."""
    suf, n = _chk(b, c)
    getattr(_lib(), "oracle_scale_" + suf)(_p(b), _p(c), float(s), n)


def add(a, b, c):
    """c[i] = a[i] + b[i]."""
    suf, n = _chk(a, b, c)
    getattr(_lib(), "oracle_add_" + suf)(_p(a), _p(b), _p(c), n)


def triad(a, b, c, s):
    """a[i] = b[i] + s * c[i], multiply and add rounded separately (no FMA)."""
    suf, n = _chk(a, b, c)
    getattr(_lib(), "oracle_triad_" + suf)(_p(a), _p(b), _p(c), float(s), n)


def dot(a, b):
    """sum_i a[i]*b[i]: compensated long-double sum, rounded once to double."""
    suf, n = _chk(a, b)
    return getattr(_lib(), "oracle_dot_" + suf)(_p(a), _p(b), n, None)


def dot_longdouble(a, b):
    """Same sum, returned as numpy.longdouble (80-bit) without the final rounding."""
    suf, n = _chk(a, b)
    out = np.zeros(1, dtype=np.longdouble)
    getattr(_lib(), "oracle_dot_" + suf)(_p(a), _p(b), n, _p(out))
    return out[0]


def dot_plain(a, b):
    """Uncompensated long-double running sum (brute-force definition), as double."""
    suf, n = _chk(a, b)
    return getattr(_lib(), "oracle_dot_plain_" + suf)(_p(a), _p(b), n)


def dot_abs(a, b):
    """sum_i |a[i]*b[i]| in long double, as double (for condition numbers)."""
    suf, n = _chk(a, b)
    return getattr(_lib(), "oracle_dot_abs_" + suf)(_p(a), _p(b), n)


def lds_stream(inp, out, c, rep):
    """Tile-wise (1024 16-byte vectors per tile): rep rounds of x'[j] = x[(j+1) mod 1024] + c."""
    suf, n = _chk(inp, out)
    if getattr(_lib(), "oracle_lds_stream_" + suf)(_p(inp), _p(out), float(c), n, int(rep)) != 0:
        raise ValueError("n must be a whole number of tiles of 1024 16-byte vectors")
