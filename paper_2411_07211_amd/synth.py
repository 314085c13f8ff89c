"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds no BLAS arithmetic: only a counter-based generator, so that the CPU oracle and the GPU
library are always fed bit-identical host arrays (generated here, then uploaded).

Generator: element ``i`` of tensor ``tensor_id`` under ``seed`` is derived from
``mix64(mix64(seed * 0x9E3779B97F4A7C15 + tensor_id) + i)`` where ``mix64`` is the published
splitmix64 output function (Steele, Lea, Flood 2014).  Uniform draws use the top 24 (fp32) or 53
(fp64) bits: ``2 * k / 2**bits - 1`` in [-1, 1), exactly representable.  Normal draws are
Box-Muller in fp64 on two uniform(0,1] / [0,1) draws, then rounded to the element type.

Tensor ids by convention: A = 0, x = 1, y = 2, scalars = 3.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

TENSOR_A, TENSOR_X, TENSOR_Y, TENSOR_SCALARS = 0, 1, 2, 3

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 20
_WORKERS = min(8, os.cpu_count() or 1)


def _for_chunks(n: int, fill) -> None:
    """Calls fill(start, count) for every chunk of [0, n); chunks are independent (the generator
    is counter-based), so large tensors are filled by a few threads."""
    starts = range(0, n, _CHUNK)
    if n <= 4 * _CHUNK:
        for s in starts:
            fill(s, min(_CHUNK, n - s))
        return
    with ThreadPoolExecutor(_WORKERS) as ex:
        list(ex.map(lambda s: fill(s, min(_CHUNK, n - s)), starts))


def _mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function, in place on a fresh uint64 array."""
    t = np.empty_like(z)
    z += _GOLDEN
    np.right_shift(z, np.uint64(30), out=t); z ^= t; z *= _M1
    np.right_shift(z, np.uint64(27), out=t); z ^= t; z *= _M2
    np.right_shift(z, np.uint64(31), out=t); z ^= t
    return z


def _stream_key(seed: int, tensor_id: int) -> np.uint64:
    with np.errstate(over="ignore"):
        k = np.array([seed & 0xFFFFFFFFFFFFFFFF], np.uint64) * _GOLDEN + np.uint64(tensor_id)
        return _mix64(k)[0]


def raw_u64(seed: int, tensor_id: int, start: int, count: int) -> np.ndarray:
    """``count`` raw 64-bit draws for indices start .. start+count-1."""
    key = _stream_key(seed, tensor_id)
    with np.errstate(over="ignore"):
        idx = np.arange(start, start + count, dtype=np.uint64)
        idx += key
        return _mix64(idx)


def uniform(seed: int, tensor_id: int, n: int, dtype=np.float32) -> np.ndarray:
    """n i.i.d. draws, uniform on [-1, 1)."""
    dtype = np.dtype(dtype)
    bits = 24 if dtype == np.float32 else 53
    out = np.empty(n, dtype)

    def fill(s, c):
        k = raw_u64(seed, tensor_id, s, c) >> np.uint64(64 - bits)
        out[s:s + c] = (k.astype(np.float64) * (2.0 / float(1 << bits)) - 1.0).astype(dtype)

    _for_chunks(n, fill)
    return out


def normal(seed: int, tensor_id: int, n: int, std: float = 1.0, dtype=np.float64) -> np.ndarray:
    """n i.i.d. draws from N(0, std**2) (std is the standard deviation)."""
    dtype = np.dtype(dtype)
    out = np.empty(n, dtype)
    two53 = float(1 << 53)

    def fill(s, c):
        r = raw_u64(seed, tensor_id, 2 * s, 2 * c) >> np.uint64(11)
        u1 = (r[0::2].astype(np.float64) + 1.0) / two53          # (0, 1]
        u2 = r[1::2].astype(np.float64) / two53                  # [0, 1)
        z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
        out[s:s + c] = (std * z).astype(dtype)

    _for_chunks(n, fill)
    return out


def small_ints(seed: int, tensor_id: int, n: int, lo: int = -2, hi: int = 2,
               dtype=np.float32) -> np.ndarray:
    """n i.i.d. integers in [lo, hi] stored as floating point (for bit-exact tests)."""
    dtype = np.dtype(dtype)
    span = np.uint64(hi - lo + 1)
    out = np.empty(n, dtype)

    def fill(s, c):
        k = (raw_u64(seed, tensor_id, s, c) >> np.uint64(33)) % span
        out[s:s + c] = (k.astype(np.int64) + lo).astype(dtype)

    _for_chunks(n, fill)
    return out


def scalar(seed: int, index: int, dtype=np.float32):
    """Scalar number ``index`` of a seed's scalar stream (uniform [-1,1)); draws within 1e-3 of 0
    or of +-1 are skipped so that no special-case path is hit by accident."""
    dtype = np.dtype(dtype)
    i = 0
    taken = -1
    while True:
        v = uniform(seed, TENSOR_SCALARS, i + 1, dtype)[i]
        i += 1
        if abs(v) < 1e-3 or abs(abs(v) - 1.0) < 1e-3:
            continue
        taken += 1
        if taken == index:
            return dtype.type(v)


def strided(dense: np.ndarray, inc: int, fill=np.nan) -> np.ndarray:
    """Spread a dense logical vector over a buffer with BLAS increment ``inc`` (negative: stored
    backwards); the gaps are filled with ``fill`` (NaN canaries by default)."""
    n = dense.size
    a = abs(inc)
    buf = np.full(max(1 + (n - 1) * a, 0) if n > 0 else 0, fill, dense.dtype)
    if n > 0:
        if inc > 0:
            buf[::a] = dense
        else:
            buf[::a] = dense[::-1]
    return buf


def gather(buf: np.ndarray, n: int, inc: int) -> np.ndarray:
    """Inverse of :func:`strided`: the dense logical vector held in ``buf``."""
    a = abs(inc)
    v = buf[: 1 + (n - 1) * a : a] if n > 0 else buf[:0]
    return v.copy() if inc > 0 else v[::-1].copy()
