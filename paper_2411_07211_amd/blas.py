"""ctypes binding of libmxblas.so: the same names as include/mxblas.h, argument marshalling only.

Every ``mxb_*`` function takes the handle first and accepts, for each device pointer, either a
torch CUDA tensor (its ``data_ptr()`` is passed) or a raw integer address.  Nothing is computed
here and there is no fallback: if the library has not been built, importing this module raises.
For tensors the binding also checks, on the host, that the element type matches the routine and
that the tensor is as large as the call's n / lda / increments require (ValueError / TypeError
otherwise): the C ABI cannot know a buffer's size, and an overrun on the GPU can take the device
down.

:class:`Context` is a small convenience for callers that live in PyTorch: it creates a handle,
points it at torch's current stream and gives it a workspace tensor.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmxblas.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2411_07211_amd.build` "
        "(there is no CPU fallback)"
    )
# PyTorch bundles its own HIP runtime (soname libamdhip64.so.7).  It has to be in the process
# before libmxblas.so is loaded, so that the library's kernels are registered with the same
# runtime that owns torch's device memory and streams; loaded the other way round, the process
# would hold two runtimes and every launch would fail with "no device".
import torch  # noqa: E402,F401  (load order matters)

_lib = ctypes.CDLL(LIB_PATH)

ROW_MAJOR, COL_MAJOR = 101, 102
NO_TRANS, TRANS = 111, 112
UPPER, LOWER = 121, 122
NON_UNIT, UNIT = 131, 132
AXPY, SCAL, DOT, ASUM, NRM2, GEMV, TRMV, SYMV, GER, GEMV_BATCHED, TRSV = range(1, 12)
OK, ERR_HANDLE, ERR_WORKSPACE, ERR_NOT_IMPLEMENTED, ERR_TIMEOUT, ERR_STATIC_LIMIT, ERR_HIP_BASE = 0, 1, 2, 3, 4, 5, 1000
STATIC_SCRATCH_BYTES = 4 << 20
(OPT_L1_BLOCKS_PER_CU, OPT_REDUCE_BLOCKS, OPT_ROWDOT_XCHUNK, OPT_ROWDOT_BLOCKS_PER_CU,
 OPT_COLACC_TARGET_BLOCKS, OPT_COLACC_MIN_ROWS, OPT_SYMV_TARGET_BLOCKS, OPT_GER_ROWS_PER_BLOCK,
 OPT_SYMV_TILE_VECTORS, OPT_TRI_DIAG_WEIGHT, OPT_SYMV_SMALL_MAX, OPT_TRSV_CHAIN_MIN,
 OPT_TRSV_SPIN_LIMIT, OPT_GEMVT_SMALL_MAX, OPT_GEMVN_SMALL_MAX) = range(15)

_i64, _int, _ptr, _sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
_f, _d = ctypes.c_float, ctypes.c_double


def _sig(name, restype, *argtypes):
    fn = getattr(_lib, name)
    fn.restype = restype
    fn.argtypes = list(argtypes)
    return fn


_create = _sig("mxb_create", _int, ctypes.POINTER(_ptr))
_destroy = _sig("mxb_destroy", _int, _ptr)
_set_stream = _sig("mxb_set_stream", _int, _ptr, _ptr)
_set_workspace = _sig("mxb_set_workspace", _int, _ptr, _ptr, _sz)
_workspace_bytes = _sig("mxb_workspace_bytes", _sz, _int, _int, _i64, _i64)
_workspace_bytes_for = _sig("mxb_workspace_bytes_for", _sz, _ptr, _int, _int, _i64, _i64)
_set_option = _sig("mxb_set_option", _int, _ptr, _int, _i64)
_get_option = _sig("mxb_get_option", _i64, _ptr, _int)
_last_status = _sig("mxb_last_status", _int, _ptr)
_probe_copy = _sig("mxb_probe_copy", _int, _ptr, _sz, _ptr, _ptr)
_probe_read = _sig("mxb_probe_read", _int, _ptr, _sz, _ptr)
_fn = {}
for _p, _t in (("s", _f), ("d", _d)):
    _fn[_p + "axpy"] = _sig(f"mxb_{_p}axpy", _int, _ptr, _i64, _t, _ptr, _i64, _ptr, _i64)
    _fn[_p + "scal"] = _sig(f"mxb_{_p}scal", _int, _ptr, _i64, _t, _ptr, _i64)
    _fn[_p + "dot"] = _sig(f"mxb_{_p}dot", _int, _ptr, _i64, _ptr, _i64, _ptr, _i64, _ptr)
    _fn[_p + "asum"] = _sig(f"mxb_{_p}asum", _int, _ptr, _i64, _ptr, _i64, _ptr)
    _fn[_p + "nrm2"] = _sig(f"mxb_{_p}nrm2", _int, _ptr, _i64, _ptr, _i64, _ptr)
    _fn[_p + "copy"] = _sig(f"mxb_{_p}copy", _int, _ptr, _i64, _ptr, _i64, _ptr, _i64)
    _fn[_p + "swap"] = _sig(f"mxb_{_p}swap", _int, _ptr, _i64, _ptr, _i64, _ptr, _i64)
    _fn[_p + "rot"] = _sig(f"mxb_{_p}rot", _int, _ptr, _i64, _ptr, _i64, _ptr, _i64, _t, _t)
    _fn[_p + "rotm"] = _sig(f"mxb_{_p}rotm", _int, _ptr, _i64, _ptr, _i64, _ptr, _i64, _ptr)
    _fn["i" + _p + "amax"] = _sig(f"mxb_i{_p}amax", _int, _ptr, _i64, _ptr, _i64, _ptr)
    _fn[_p + "gemv"] = _sig(f"mxb_{_p}gemv", _int, _ptr, _int, _int, _i64, _i64, _t, _ptr, _i64, _ptr, _i64,
                            _t, _ptr, _i64)
    _fn[_p + "gemv_batched"] = _sig(f"mxb_{_p}gemv_batched", _int, _ptr, _int, _int, _i64, _i64, _t, _ptr, _i64, _i64, _ptr, _i64,
                                    _i64, _t, _ptr, _i64, _i64, _i64)
    _fn[_p + "trmv"] = _sig(f"mxb_{_p}trmv", _int, _ptr, _int, _int, _int, _int, _i64, _ptr, _i64, _ptr, _i64)
    _fn[_p + "trsv"] = _sig(f"mxb_{_p}trsv", _int, _ptr, _int, _int, _int, _int, _i64, _ptr, _i64, _ptr, _i64)
    _fn[_p + "symv"] = _sig(f"mxb_{_p}symv", _int, _ptr, _int, _int, _i64, _t, _ptr, _i64, _ptr, _i64, _t,
                            _ptr, _i64)
    _fn[_p + "ger"] = _sig(f"mxb_{_p}ger", _int, _ptr, _int, _i64, _i64, _t, _ptr, _i64, _ptr, _i64, _ptr, _i64)
    _fn[_p + "syr"] = _sig(f"mxb_{_p}syr", _int, _ptr, _int, _int, _i64, _t, _ptr, _i64, _ptr, _i64)
    _fn[_p + "syr2"] = _sig(f"mxb_{_p}syr2", _int, _ptr, _int, _int, _i64, _t, _ptr, _i64, _ptr, _i64, _ptr, _i64)


_fn["dsdot"] = _sig("mxb_dsdot", _int, _ptr, _i64, _ptr, _i64, _ptr, _i64, _ptr)
_fn["sgemv_static"] = _sig("mxb_sgemv_static", _int, _ptr, _int, _int, _i64, _i64, _f, _ptr, _i64, _ptr, _i64, _f, _ptr, _i64)


def _dp(t):
    """Device address of a torch tensor, or the integer / None given."""
    if t is None:
        return None
    if isinstance(t, int):
        return t or None
    return t.data_ptr() or None


# ---- handle ------------------------------------------------------------------------------------
def mxb_create():
    """Returns (status, handle)."""
    h = _ptr()
    st = _create(ctypes.byref(h))
    return st, h.value


def mxb_destroy(h):
    return _destroy(h)


def mxb_set_stream(h, hip_stream):
    return _set_stream(h, hip_stream)


def mxb_set_workspace(h, dev_ptr, nbytes):
    return _set_workspace(h, _dp(dev_ptr), nbytes)


def mxb_workspace_bytes(routine, elem_size, m, n):
    return _workspace_bytes(routine, elem_size, m, n)


def mxb_workspace_bytes_for(h, routine, elem_size, m, n):
    return _workspace_bytes_for(h, routine, elem_size, m, n)


def mxb_set_option(h, option, value):
    return _set_option(h, option, value)


def mxb_get_option(h, option):
    return _get_option(h, option)


def mxb_last_status(h):
    return _last_status(h)


def _bytes(t):
    return t.numel() * t.element_size() if hasattr(t, "numel") else None


def mxb_probe_copy(h, nbytes, src, dst):
    for t, what in ((src, "src"), (dst, "dst")):
        if _bytes(t) is not None and nbytes > _bytes(t):
            raise ValueError(f"{what}: {nbytes} bytes requested, the tensor holds {_bytes(t)}")
    return _probe_copy(h, nbytes, _dp(src), _dp(dst))


def mxb_probe_read(h, nbytes, src):
    if _bytes(src) is not None and nbytes > _bytes(src):
        raise ValueError(f"src: {nbytes} bytes requested, the tensor holds {_bytes(src)}")
    return _probe_read(h, nbytes, _dp(src))


# ---- operand checks ------------------------------------------------------------------------------
# The C ABI takes bare device pointers and cannot know how large the buffers behind them are.  When a
# torch tensor is passed, the binding knows, and refuses a call whose operands the routine would
# overrun (or whose element type does not match the routine) before anything is launched: an
# out-of-bounds access on the GPU can take the whole device down.  Raw integer addresses pass unchecked.
_DT = {"s": torch.float32, "d": torch.float64}


def _chk(t, need, what, p=None):
    if t is None or t.__class__ is int:
        return
    if p is not None and t.dtype is not _DT[p]:
        raise TypeError(f"{what}: tensor of {t.dtype} passed to a {_DT[p]} routine")
    if need > t.numel():
        raise ValueError(f"{what}: the call reads or writes {need} elements, the tensor holds {t.numel()}")


def _v(t, n, inc, what, p):
    """Device address of a vector operand of n logical elements with increment inc."""
    _chk(t, 0 if n <= 0 else 1 + (n - 1) * abs(inc), what, p)
    return _dp(t)


def _m(t, layout, rows, cols, lda, what, p):
    """Device address of a rows x cols matrix operand with leading dimension lda."""
    major, minor = (rows, cols) if layout == ROW_MAJOR else (cols, rows)
    _chk(t, 0 if major <= 0 or minor <= 0 else (major - 1) * lda + minor, what, p)
    return _dp(t)


# ---- level 1 -----------------------------------------------------------------------------------
def _mk_level1():
    g = globals()
    for p in "sd":
        fn = _fn

        def axpy(h, n, alpha, x, incx, y, incy, p=p):
            return fn[p + "axpy"](h, n, alpha, _v(x, n, incx, "x", p), incx, _v(y, n, incy, "y", p), incy)

        def scal(h, n, alpha, x, incx, p=p):
            return fn[p + "scal"](h, n, alpha, _v(x, n, max(incx, 0), "x", p), incx)

        def dot(h, n, x, incx, y, incy, result, p=p):
            return fn[p + "dot"](h, n, _v(x, n, incx, "x", p), incx, _v(y, n, incy, "y", p), incy, _v(result, 1, 1, "result", p))

        def asum(h, n, x, incx, result, p=p):
            return fn[p + "asum"](h, n, _v(x, n, max(incx, 0), "x", p), incx, _v(result, 1, 1, "result", p))

        def nrm2(h, n, x, incx, result, p=p):
            return fn[p + "nrm2"](h, n, _v(x, n, max(incx, 0), "x", p), incx, _v(result, 1, 1, "result", p))

        def copy(h, n, x, incx, y, incy, p=p):
            return fn[p + "copy"](h, n, _v(x, n, incx, "x", p), incx, _v(y, n, incy, "y", p), incy)

        def swap(h, n, x, incx, y, incy, p=p):
            return fn[p + "swap"](h, n, _v(x, n, incx, "x", p), incx, _v(y, n, incy, "y", p), incy)

        def rot(h, n, x, incx, y, incy, c, s, p=p):
            return fn[p + "rot"](h, n, _v(x, n, incx, "x", p), incx, _v(y, n, incy, "y", p), incy, c, s)

        def rotm(h, n, x, incx, y, incy, param, p=p):
            return fn[p + "rotm"](h, n, _v(x, n, incx, "x", p), incx, _v(y, n, incy, "y", p), incy,
                                  _host5(param, _f if p == "s" else _d))

        def iamax(h, n, x, incx, result, p=p):
            _chk(result, 1, "result")
            return fn["i" + p + "amax"](h, n, _v(x, n, max(incx, 0), "x", p), incx, _dp(result))

        for name, f in (("axpy", axpy), ("scal", scal), ("dot", dot), ("asum", asum), ("nrm2", nrm2), ("copy", copy),
                        ("swap", swap), ("rot", rot), ("rotm", rotm)):
            f.__name__ = f"mxb_{p}{name}"
            g[f.__name__] = f
        iamax.__name__ = f"mxb_i{p}amax"
        g[iamax.__name__] = iamax


def _host5(param, ctype):
    """rotm's parameter block is a HOST array of 5 values."""
    if param is None:
        return None
    return (ctype * 5)(*[float(v) for v in param])


_mk_level1()


def mxb_dsdot(h, n, x, incx, y, incy, result):
    return _fn["dsdot"](h, n, _v(x, n, incx, "x", "s"), incx, _v(y, n, incy, "y", "s"), incy, _v(result, 1, 1, "result", "d"))


# ---- level 2 -----------------------------------------------------------------------------------
def _mk_level2():
    g = globals()
    for p in "sd":
        fn = _fn

        def gemv(h, layout, trans, m, n, alpha, A, lda, x, incx, beta, y, incy, p=p):
            lenx, leny = (n, m) if trans == NO_TRANS else (m, n)
            return fn[p + "gemv"](h, layout, trans, m, n, alpha, _m(A, layout, m, n, lda, "A", p), lda,
                                  _v(x, lenx, incx, "x", p), incx, beta, _v(y, leny, incy, "y", p), incy)

        def gemv_batched(h, layout, trans, m, n, alpha, A, lda, strideA, x, incx, stridex, beta, y, incy, stridey, batch, p=p):
            lenx, leny = (n, m) if trans == NO_TRANS else (m, n)
            major, minor = (m, n) if layout == ROW_MAJOR else (n, m)
            last = max(batch - 1, 0)
            empty = batch <= 0 or m <= 0 or n <= 0
            # the last problem reaches furthest (negative strides are rejected by the library)
            _chk(A, 0 if empty else last * max(strideA, 0) + (major - 1) * lda + minor, "A", p)
            _chk(x, 0 if empty else last * max(stridex, 0) + 1 + (lenx - 1) * abs(incx), "x", p)
            _chk(y, 0 if empty else last * max(stridey, 0) + 1 + (leny - 1) * abs(incy), "y", p)
            return fn[p + "gemv_batched"](h, layout, trans, m, n, alpha, _dp(A), lda, strideA, _dp(x), incx, stridex, beta,
                                          _dp(y), incy, stridey, batch)

        def trmv(h, layout, uplo, trans, diag, n, A, lda, x, incx, p=p):
            return fn[p + "trmv"](h, layout, uplo, trans, diag, n, _m(A, layout, n, n, lda, "A", p), lda, _v(x, n, incx, "x", p), incx)

        def trsv(h, layout, uplo, trans, diag, n, A, lda, x, incx, p=p):
            return fn[p + "trsv"](h, layout, uplo, trans, diag, n, _m(A, layout, n, n, lda, "A", p), lda, _v(x, n, incx, "x", p), incx)

        def symv(h, layout, uplo, n, alpha, A, lda, x, incx, beta, y, incy, p=p):
            return fn[p + "symv"](h, layout, uplo, n, alpha, _m(A, layout, n, n, lda, "A", p), lda, _v(x, n, incx, "x", p), incx,
                                  beta, _v(y, n, incy, "y", p), incy)

        def ger(h, layout, m, n, alpha, x, incx, y, incy, A, lda, p=p):
            return fn[p + "ger"](h, layout, m, n, alpha, _v(x, m, incx, "x", p), incx, _v(y, n, incy, "y", p), incy,
                                 _m(A, layout, m, n, lda, "A", p), lda)

        def syr(h, layout, uplo, n, alpha, x, incx, A, lda, p=p):
            return fn[p + "syr"](h, layout, uplo, n, alpha, _v(x, n, incx, "x", p), incx, _m(A, layout, n, n, lda, "A", p), lda)

        def syr2(h, layout, uplo, n, alpha, x, incx, y, incy, A, lda, p=p):
            return fn[p + "syr2"](h, layout, uplo, n, alpha, _v(x, n, incx, "x", p), incx, _v(y, n, incy, "y", p), incy,
                                  _m(A, layout, n, n, lda, "A", p), lda)

        for name, f in (("gemv", gemv), ("gemv_batched", gemv_batched), ("trmv", trmv), ("trsv", trsv), ("symv", symv), ("ger", ger), ("syr", syr), ("syr2", syr2)):
            f.__name__ = f"mxb_{p}{name}"
            g[f.__name__] = f


_mk_level2()


def mxb_sgemv_static(h, layout, trans, m, n, alpha, A, lda, x, incx, beta, y, incy):
    lenx, leny = (n, m) if trans == NO_TRANS else (m, n)
    return _fn["sgemv_static"](h, layout, trans, m, n, alpha, _m(A, layout, m, n, lda, "A", "s"), lda,
                               _v(x, lenx, incx, "x", "s"), incx, beta, _v(y, leny, incy, "y", "s"), incy)


def routine(prefix: str, name: str):
    """``routine('s', 'gemv')`` -> :func:`mxb_sgemv` (for code that is generic over precision)."""
    return globals()[f"mxb_{prefix}{name}"]


class MxbError(RuntimeError):
    pass


def check(status: int, what: str = "mxblas call"):
    if status != OK:
        raise MxbError(f"{what} failed with status {status}")


class Context:
    """A handle bound to torch's current stream on ``device`` with a workspace tensor."""

    def __init__(self, device="cuda:0", workspace_bytes: int = 64 << 20):
        import torch

        if not torch.cuda.is_available():
            raise MxbError("no GPU: libmxblas has no CPU path")
        self.device = torch.device(device)
        st, self.h = mxb_create()
        check(st, "mxb_create")
        self._ws = torch.empty(workspace_bytes, dtype=torch.uint8, device=self.device)
        check(mxb_set_workspace(self.h, self._ws, workspace_bytes), "mxb_set_workspace")
        self.use_current_stream()

    def use_current_stream(self):
        import torch

        check(mxb_set_stream(self.h, torch.cuda.current_stream(self.device).cuda_stream), "mxb_set_stream")

    def set_option(self, option, value):
        check(mxb_set_option(self.h, option, value), "mxb_set_option")

    def last_status(self):
        return mxb_last_status(self.h)

    def close(self):
        if getattr(self, "h", None):
            mxb_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
