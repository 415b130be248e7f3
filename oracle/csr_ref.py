"""ctypes access to the oracle's plain-C CSR products (test / baseline infrastructure only)."""
import ctypes as C
import os

import numpy as np

from . import build_c

_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        if not os.path.exists(build_c.LIB):
            build_c.build()
        lib = C.CDLL(build_c.LIB)
        vp, i64 = C.c_void_p, C.c_int64
        lib.csr_spmm_f64.argtypes = [i64, i64, vp, vp, vp, i64, vp]
        lib.csr_spmm_norm_f64.argtypes = [i64, i64, vp, vp, vp, vp, i64, vp]
        lib.csr_spmm_norm_omp_f32.argtypes = [i64, vp, vp, vp, vp, i64, vp]
        lib.csr_omp_threads.restype = C.c_int
        for f in (lib.csr_spmm_f64, lib.csr_spmm_norm_f64, lib.csr_spmm_norm_omp_f32):
            f.restype = None
        _LIB = lib
    return _LIB


def _prep(rowptr, colidx, X):
    return (np.ascontiguousarray(rowptr, dtype=np.int64), np.ascontiguousarray(colidx, dtype=np.int32),
            np.ascontiguousarray(X, dtype=np.float32))


def spmm_f64(rowptr, colidx, X, row_begin=0, row_end=None):
    rowptr, colidx, X = _prep(rowptr, colidx, X)
    row_end = len(rowptr) - 1 if row_end is None else row_end
    Y = np.empty((row_end - row_begin, X.shape[1]), dtype=np.float64)
    _lib().csr_spmm_f64(row_begin, row_end, rowptr.ctypes.data, colidx.ctypes.data, X.ctypes.data, X.shape[1],
                        Y.ctypes.data)
    return Y


def spmm_norm_f64(rowptr, colidx, d, X, row_begin=0, row_end=None):
    rowptr, colidx, X = _prep(rowptr, colidx, X)
    d = np.ascontiguousarray(d, dtype=np.int64)
    row_end = len(rowptr) - 1 if row_end is None else row_end
    Y = np.empty((row_end - row_begin, X.shape[1]), dtype=np.float64)
    _lib().csr_spmm_norm_f64(row_begin, row_end, rowptr.ctypes.data, colidx.ctypes.data, d.ctypes.data,
                             X.ctypes.data, X.shape[1], Y.ctypes.data)
    return Y


def spmm_norm_omp_f32(rowptr, colidx, s, X, Y=None):
    rowptr, colidx, X = _prep(rowptr, colidx, X)
    s = np.ascontiguousarray(s, dtype=np.float32)
    if Y is None:
        Y = np.empty((len(rowptr) - 1, X.shape[1]), dtype=np.float32)
    _lib().csr_spmm_norm_omp_f32(len(rowptr) - 1, rowptr.ctypes.data, colidx.ctypes.data, s.ctypes.data,
                                 X.ctypes.data, X.shape[1], Y.ctypes.data)
    return Y


def omp_threads() -> int:
    return int(_lib().csr_omp_threads())
