"""ctypes front-end of the CPU oracle (oracle_blas.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the benchmark's cpu-baseline
leg.  The GPU package never imports this module and this module never imports the GPU package.

All arrays are host numpy arrays.  In-place routines modify the array they are given, exactly
like the C routine; reductions return a numpy scalar of the element type.  Each routine takes an
optional ``want_D=True`` to also return the condition denominators (float64) described in
oracle_blas_impl.h.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")

ROW_MAJOR, COL_MAJOR = 101, 102
NO_TRANS, TRANS = 111, 112
UPPER, LOWER = 121, 122
NON_UNIT, UNIT = 131, 132


def build(force: bool = False) -> str:
    """Compile oracle_blas.c with gcc -O2 (no fast-math) into liboracle.so; returns the path."""
    srcs = [os.path.join(_HERE, f) for f in ("oracle_blas.c", "oracle_blas_impl.h")]
    if force or not os.path.exists(_SO) or any(
        os.path.getmtime(s) > os.path.getmtime(_SO) for s in srcs
    ):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", _SO, srcs[0], "-lm"]
        )
    return _SO


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_SO)
        _declare(_lib)
        _declare_mixed(_lib)
    return _lib


_i64 = ctypes.c_int64
_int = ctypes.c_int
_ptr = ctypes.c_void_p


def _declare(lib):
    for p, ct in (("s", ctypes.c_float), ("d", ctypes.c_double)):
        f = getattr(lib, f"oracle_{p}axpy")
        f.argtypes = [_i64, ct, _ptr, _i64, _ptr, _i64, _ptr]
        f.restype = None
        f = getattr(lib, f"oracle_{p}scal")
        f.argtypes = [_i64, ct, _ptr, _i64, _ptr]
        f.restype = None
        f = getattr(lib, f"oracle_{p}dot")
        f.argtypes = [_i64, _ptr, _i64, _ptr, _i64, _ptr]
        f.restype = ct
        for name in ("asum", "nrm2"):
            f = getattr(lib, f"oracle_{p}{name}")
            f.argtypes = [_i64, _ptr, _i64, _ptr]
            f.restype = ct
        f = getattr(lib, f"oracle_{p}copy")
        f.argtypes = [_i64, _ptr, _i64, _ptr, _i64]
        f.restype = None
        f = getattr(lib, f"oracle_{p}swap")
        f.argtypes = [_i64, _ptr, _i64, _ptr, _i64]
        f.restype = None
        f = getattr(lib, f"oracle_{p}rot")
        f.argtypes = [_i64, _ptr, _i64, _ptr, _i64, ct, ct, _ptr]
        f.restype = None
        f = getattr(lib, f"oracle_{p}rotm")
        f.argtypes = [_i64, _ptr, _i64, _ptr, _i64, _ptr, _ptr]
        f.restype = None
        f = getattr(lib, f"oracle_{p}iamax")
        f.argtypes = [_i64, _ptr, _i64]
        f.restype = _i64
        f = getattr(lib, f"oracle_{p}gemv")
        f.argtypes = [_int, _int, _i64, _i64, ct, _ptr, _i64, _ptr, _i64, ct, _ptr, _i64, _ptr]
        f.restype = None
        f = getattr(lib, f"oracle_{p}gemv_batched")
        f.argtypes = [_int, _int, _i64, _i64, ct, _ptr, _i64, _i64, _ptr, _i64, _i64, ct, _ptr, _i64, _i64, _i64, _ptr]
        f.restype = None
        f = getattr(lib, f"oracle_{p}trmv")
        f.argtypes = [_int, _int, _int, _int, _i64, _ptr, _i64, _ptr, _i64, _ptr]
        f.restype = None
        f = getattr(lib, f"oracle_{p}symv")
        f.argtypes = [_int, _int, _i64, ct, _ptr, _i64, _ptr, _i64, ct, _ptr, _i64, _ptr]
        f.restype = None
        f = getattr(lib, f"oracle_{p}ger")
        f.argtypes = [_int, _i64, _i64, ct, _ptr, _i64, _ptr, _i64, _ptr, _i64, _ptr]
        f.restype = None
        f = getattr(lib, f"oracle_{p}syr")
        f.argtypes = [_int, _int, _i64, ct, _ptr, _i64, _ptr, _i64, _ptr]
        f.restype = None
        f = getattr(lib, f"oracle_{p}syr2")
        f.argtypes = [_int, _int, _i64, ct, _ptr, _i64, _ptr, _i64, _ptr, _i64, _ptr]
        f.restype = None
        f = getattr(lib, f"oracle_{p}trsv")
        f.argtypes = [_int, _int, _int, _int, _i64, _ptr, _i64, _ptr, _i64, _ptr]
        f.restype = None


def _declare_mixed(lib):
    lib.oracle_dsdot.argtypes = [_i64, _ptr, _i64, _ptr, _i64, _ptr]
    lib.oracle_dsdot.restype = ctypes.c_double


def _prefix(a: np.ndarray) -> str:
    if a.dtype == np.float32:
        return "s"
    if a.dtype == np.float64:
        return "d"
    raise TypeError(f"oracle supports float32/float64, got {a.dtype}")


def _p(a):
    if a is None:
        return None
    assert isinstance(a, np.ndarray) and a.flags["C_CONTIGUOUS"], "need a C-contiguous numpy array"
    return a.ctypes.data_as(_ptr)


def _same(*arrs):
    p = _prefix(arrs[0])
    for a in arrs[1:]:
        assert _prefix(a) == p, "mixed precisions"
    return p


def _need(a: np.ndarray, n: int, inc: int, what: str):
    need = 0 if n <= 0 else 1 + (n - 1) * abs(inc)
    assert a.size >= need, f"{what}: array of {a.size} elements is too short for n={n}, inc={inc}"


def axpy(n, alpha, x, incx, y, incy, want_D=False):
    p = _same(x, y)
    _need(x, n, incx, "x"); _need(y, n, incy, "y")
    D = np.zeros(max(n, 0), np.float64) if want_D else None
    getattr(_load(), f"oracle_{p}axpy")(n, alpha, _p(x), incx, _p(y), incy, _p(D))
    return D


def scal(n, alpha, x, incx, want_D=False):
    p = _prefix(x)
    if incx > 0:
        _need(x, n, incx, "x")
    D = np.zeros(max(n, 0), np.float64) if want_D else None
    getattr(_load(), f"oracle_{p}scal")(n, alpha, _p(x), incx, _p(D))
    return D


def dot(n, x, incx, y, incy, want_D=False):
    p = _same(x, y)
    _need(x, n, incx, "x"); _need(y, n, incy, "y")
    D = np.zeros(1, np.float64)
    r = x.dtype.type(getattr(_load(), f"oracle_{p}dot")(n, _p(x), incx, _p(y), incy, _p(D)))
    return (r, D[0]) if want_D else r


def _red(name, n, x, incx, want_D):
    p = _prefix(x)
    if incx > 0:
        _need(x, n, incx, "x")
    D = np.zeros(1, np.float64)
    r = x.dtype.type(getattr(_load(), f"oracle_{p}{name}")(n, _p(x), incx, _p(D)))
    return (r, D[0]) if want_D else r


def asum(n, x, incx, want_D=False):
    return _red("asum", n, x, incx, want_D)


def nrm2(n, x, incx, want_D=False):
    return _red("nrm2", n, x, incx, want_D)


def _mat_need(A, layout, rows, cols, lda):
    if rows <= 0 or cols <= 0:
        return
    major, minor = (rows, cols) if layout == ROW_MAJOR else (cols, rows)
    assert lda >= max(1, minor), f"lda={lda} < {minor}"
    assert A.size >= (major - 1) * lda + minor, "matrix buffer too short"


def gemv(layout, trans, m, n, alpha, A, lda, x, incx, beta, y, incy, want_D=False):
    p = _same(A, x, y)
    lenx, leny = (n, m) if trans == NO_TRANS else (m, n)
    _mat_need(A, layout, m, n, lda); _need(x, lenx, incx, "x"); _need(y, leny, incy, "y")
    D = np.zeros(max(leny, 0), np.float64) if want_D else None
    getattr(_load(), f"oracle_{p}gemv")(layout, trans, m, n, alpha, _p(A), lda, _p(x), incx,
                                        beta, _p(y), incy, _p(D))
    return D


def gemv_batched(layout, trans, m, n, alpha, A, lda, strideA, x, incx, stridex, beta, y, incy, stridey, batch, want_D=False):
    """batch independent gemv problems; problem b uses A[b*strideA:], x[b*stridex:], y[b*stridey:]."""
    p = _same(A, x, y)
    lenx, leny = (n, m) if trans == NO_TRANS else (m, n)
    assert min(strideA, stridex, stridey) >= 0 and batch >= 0
    if batch > 0:
        last = batch - 1
        _mat_need(A[last * strideA:], layout, m, n, lda)
        _need(x[last * stridex:], lenx, incx, "x"); _need(y[last * stridey:], leny, incy, "y")
    D = np.zeros(max(leny, 0) * max(batch, 0), np.float64) if want_D else None
    getattr(_load(), f"oracle_{p}gemv_batched")(layout, trans, m, n, alpha, _p(A), lda, strideA, _p(x), incx, stridex,
                                                beta, _p(y), incy, stridey, batch, _p(D))
    return D


def trmv(layout, uplo, trans, diag, n, A, lda, x, incx, want_D=False):
    p = _same(A, x)
    _mat_need(A, layout, n, n, lda); _need(x, n, incx, "x")
    D = np.zeros(max(n, 0), np.float64) if want_D else None
    getattr(_load(), f"oracle_{p}trmv")(layout, uplo, trans, diag, n, _p(A), lda, _p(x), incx,
                                        _p(D))
    return D


def symv(layout, uplo, n, alpha, A, lda, x, incx, beta, y, incy, want_D=False):
    p = _same(A, x, y)
    _mat_need(A, layout, n, n, lda); _need(x, n, incx, "x"); _need(y, n, incy, "y")
    D = np.zeros(max(n, 0), np.float64) if want_D else None
    getattr(_load(), f"oracle_{p}symv")(layout, uplo, n, alpha, _p(A), lda, _p(x), incx,
                                        beta, _p(y), incy, _p(D))
    return D


def ger(layout, m, n, alpha, x, incx, y, incy, A, lda, want_D=False):
    p = _same(A, x, y)
    _mat_need(A, layout, m, n, lda); _need(x, m, incx, "x"); _need(y, n, incy, "y")
    D = np.zeros(max(m * n, 0), np.float64) if want_D else None
    getattr(_load(), f"oracle_{p}ger")(layout, m, n, alpha, _p(x), incx, _p(y), incy, _p(A),
                                       lda, _p(D))
    return D


def syr(layout, uplo, n, alpha, x, incx, A, lda, want_D=False):
    p = _same(A, x)
    _mat_need(A, layout, n, n, lda); _need(x, n, incx, "x")
    D = np.zeros(max(n * n, 0), np.float64) if want_D else None
    getattr(_load(), f"oracle_{p}syr")(layout, uplo, n, alpha, _p(x), incx, _p(A), lda, _p(D))
    return D


def syr2(layout, uplo, n, alpha, x, incx, y, incy, A, lda, want_D=False):
    p = _same(A, x, y)
    _mat_need(A, layout, n, n, lda); _need(x, n, incx, "x"); _need(y, n, incy, "y")
    D = np.zeros(max(n * n, 0), np.float64) if want_D else None
    getattr(_load(), f"oracle_{p}syr2")(layout, uplo, n, alpha, _p(x), incx, _p(y), incy, _p(A),
                                        lda, _p(D))
    return D


def trsv(layout, uplo, trans, diag, n, A, lda, x, incx, want_D=False):
    p = _same(A, x)
    _mat_need(A, layout, n, n, lda); _need(x, n, incx, "x")
    D = np.zeros(max(n, 0), np.float64) if want_D else None
    getattr(_load(), f"oracle_{p}trsv")(layout, uplo, trans, diag, n, _p(A), lda, _p(x), incx,
                                        _p(D))
    return D


def copy(n, x, incx, y, incy):
    p = _same(x, y)
    _need(x, n, incx, "x"); _need(y, n, incy, "y")
    getattr(_load(), f"oracle_{p}copy")(n, _p(x), incx, _p(y), incy)


def swap(n, x, incx, y, incy):
    p = _same(x, y)
    _need(x, n, incx, "x"); _need(y, n, incy, "y")
    getattr(_load(), f"oracle_{p}swap")(n, _p(x), incx, _p(y), incy)


def rot(n, x, incx, y, incy, c, s, want_D=False):
    p = _same(x, y)
    _need(x, n, incx, "x"); _need(y, n, incy, "y")
    D = np.zeros(2 * max(n, 0), np.float64) if want_D else None
    getattr(_load(), f"oracle_{p}rot")(n, _p(x), incx, _p(y), incy, c, s, _p(D))
    return D


def rotm(n, x, incx, y, incy, param, want_D=False):
    p = _same(x, y, param)
    assert param.size >= 5
    _need(x, n, incx, "x"); _need(y, n, incy, "y")
    D = np.zeros(2 * max(n, 0), np.float64) if want_D else None
    getattr(_load(), f"oracle_{p}rotm")(n, _p(x), incx, _p(y), incy, _p(param), _p(D))
    return D


def iamax(n, x, incx):
    p = _prefix(x)
    if incx > 0:
        _need(x, n, incx, "x")
    return int(getattr(_load(), f"oracle_{p}iamax")(n, _p(x), incx))


def dsdot(n, x, incx, y, incy, want_D=False):
    assert x.dtype == np.float32 and y.dtype == np.float32
    _need(x, n, incx, "x"); _need(y, n, incy, "y")
    D = np.zeros(1, np.float64)
    r = np.float64(_load().oracle_dsdot(n, _p(x), incx, _p(y), incy, _p(D)))
    return (r, D[0]) if want_D else r
