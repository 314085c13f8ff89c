"""Randomised shapes, increments, pitches, base offsets and scalars for every level-2 routine
(fixed seeds): the parity cases of test_gpu_level2 at sizes and combinations nobody picked by hand."""
import numpy as np
import pytest

import oracle as O
import test_gpu_level2 as L2

pytestmark = pytest.mark.gpu

DT = [np.float32, np.float64]


def draws(seed, count):
    """count tuples of (size a, size b, pad, incx, incy, alpha, beta, base offset, layout, flags)."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        a, b = (int(np.exp(rng.uniform(0, np.log(3000)))) for _ in range(2))
        out.append((max(a, 1), max(b, 1), int(rng.integers(0, 6)), int(rng.choice([1, 1, 1, 2, -1, 3, -2])),
                    int(rng.choice([1, 1, 1, 2, -1, 3, -2])), float(rng.choice([1.0, -1.0, 1.5, 0.25])),
                    float(rng.choice([0.0, 1.0, 0.5, -2.0])), int(rng.integers(0, 4)),
                    int(rng.choice([O.ROW_MAJOR, O.COL_MAJOR])), int(rng.integers(0, 8))))
    return out


@pytest.mark.parametrize("dt", DT)
def test_random_gemv_ger(blas, ctx, dt):
    for (m, n, pad, incx, incy, alpha, beta, off, layout, flags) in draws(101, 200):
        L2.A_OFFSET[0] = off
        try:
            trans = O.TRANS if flags & 1 else O.NO_TRANS
            L2.gemv_case(blas, ctx, dt, layout, trans, m, n, alpha, beta, pad, incx, incy)
            L2.ger_case(blas, ctx, dt, layout, m, n, alpha, pad, incx, incy)
        finally:
            L2.A_OFFSET[0] = 0


@pytest.mark.parametrize("dt", DT)
def test_random_gemv_batched(blas, ctx, dt):
    for (m, n, pad, incx, incy, alpha, beta, off, layout, flags) in draws(102, 120):
        m, n = min(m, 600), min(n, 600)
        trans = O.TRANS if flags & 1 else O.NO_TRANS
        batch = 1 + (flags >> 1) * 3
        L2.gemv_batched_case(blas, ctx, dt, layout, trans, m, n, batch, alpha, beta, pad, incx, incy, gaps=(off, off, pad),
                             share=(bool(flags & 2) and off == 0, bool(flags & 4) and off == 0))


@pytest.mark.parametrize("dt", DT)
def test_random_triangular_and_symmetric(blas, ctx, dt):
    for (n, _, pad, incx, incy, alpha, beta, off, layout, flags) in draws(103, 200):
        L2.A_OFFSET[0] = off
        try:
            uplo = O.UPPER if flags & 1 else O.LOWER
            trans = O.TRANS if flags & 2 else O.NO_TRANS
            diag = O.UNIT if flags & 4 else O.NON_UNIT
            L2.trmv_case(blas, ctx, dt, layout, uplo, trans, diag, n, pad, incx)
            L2.symv_case(blas, ctx, dt, layout, uplo, n, alpha, beta, pad, incx, incy)
            L2.syr_case(blas, ctx, dt, layout, uplo, n, alpha, pad, incx, incy, bool(flags & 2))
            L2.trsv_case(blas, ctx, dt, layout, uplo, trans, diag, n, pad, incx)
        finally:
            L2.A_OFFSET[0] = 0


@pytest.mark.parametrize("dt", DT)
def test_random_trsv_many_workgroups(blas, ctx, dt):
    """Triangular solves of a few thousand unknowns (tens of workgroups of the chained kernel, tiles streamed
    with 128-bit loads) at any base offset, pitch and increment."""
    rng = np.random.default_rng(104)
    for _ in range(10):
        n = int(rng.integers(3000, 9000 if dt == np.float32 else 6500))
        L2.A_OFFSET[0] = int(rng.integers(0, 4))
        try:
            L2.trsv_case(blas, ctx, dt, int(rng.choice([O.ROW_MAJOR, O.COL_MAJOR])), int(rng.choice([O.UPPER, O.LOWER])),
                         int(rng.choice([O.NO_TRANS, O.TRANS])), int(rng.choice([O.NON_UNIT, O.UNIT])), n,
                         int(rng.integers(0, 6)), int(rng.choice([1, 1, 2, -1, 3])), seed=int(rng.integers(1, 1000)))
        finally:
            L2.A_OFFSET[0] = 0
