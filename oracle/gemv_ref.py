"""ctypes front end of ``gemv_ref.c`` (the plain fp64 loops that define the result).

Test infrastructure, not product code.  ``build()`` compiles the C file with gcc;
nothing here falls back to another implementation when the library is missing.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libgemv_ref.so")
_lib = None


def build(force=False):
    """Compile gemv_ref.c -> libgemv_ref.so (plain gcc -O2, single thread)."""
    src = os.path.join(_HERE, "gemv_ref.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-shared", "-fPIC", "-o", _SO, src, "-lm"])
    return _SO


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_SO)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        i64p = ctypes.POINTER(ctypes.c_int64)
        lib.gemv_ref_dense.argtypes = [f32p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                       f32p, ctypes.c_int32, f64p, f64p]
        lib.gemv_ref_dense.restype = None
        lib.gemv_ref_ragged.argtypes = [f32p, i64p, ctypes.c_int32, ctypes.c_int64, f32p, f64p, f64p]
        lib.gemv_ref_ragged.restype = None
        _lib = lib
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def gemv_dense(M, X, ld=None):
    """Y[b][i] = sum_j M[i][j] X[b][j] in fp64.  M: [rows, ld] (first K columns used) fp32,
    X: [B, K] fp32.  Returns (Y, Yabs), both [B, rows] float64; Yabs = sum_j |M X|."""
    M = np.asarray(M)
    X = np.atleast_2d(np.asarray(X))
    rows = M.shape[0]
    B, K = X.shape
    ld = M.shape[1] if ld is None else ld
    assert M.ndim == 2 and M.shape[1] == ld and ld >= K
    Mc, Mp = _f32(M)
    Xc, Xp = _f32(X)
    Y = np.empty((B, rows), dtype=np.float64)
    Ya = np.empty((B, rows), dtype=np.float64)
    f64p = ctypes.POINTER(ctypes.c_double)
    _load().gemv_ref_dense(Mp, rows, K, ld, Xp, B, Y.ctypes.data_as(f64p), Ya.ctypes.data_as(f64p))
    return Y, Ya


def gemv_ragged(M, row_off, X):
    """Segment s = rows row_off[s]..row_off[s+1]-1 of M ([sum rows, K] fp32) times X[s] ([n_seg, K]).
    Returns (Y, Yabs), both [sum rows] float64."""
    M = np.asarray(M)
    X = np.atleast_2d(np.asarray(X))
    row_off = np.ascontiguousarray(row_off, dtype=np.int64)
    n_seg, K = X.shape
    assert row_off.shape == (n_seg + 1,) and row_off[0] == 0 and row_off[-1] == M.shape[0]
    assert np.all(np.diff(row_off) >= 0) and M.shape[1] == K
    Mc, Mp = _f32(M)
    Xc, Xp = _f32(X)
    Y = np.empty(M.shape[0], dtype=np.float64)
    Ya = np.empty(M.shape[0], dtype=np.float64)
    f64p = ctypes.POINTER(ctypes.c_double)
    _load().gemv_ref_ragged(Mp, row_off.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), n_seg, K, Xp,
                            Y.ctypes.data_as(f64p), Ya.ctypes.data_as(f64p))
    return Y, Ya
