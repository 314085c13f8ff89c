"""Pins for the CPU oracle: closed forms, invariants, int64 brute force, hand-worked cases and an
independent fp64 library routine.  None of these re-types the oracle's own formula in the same
shape: each would fail on a dropped term, a wrong sign or index, or a transposed operand."""
import itertools
import os

import numpy as np
import pytest

import oracle as O
from paper_2411_07211_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
DT = [np.float32, np.float64]


def ints(seed, tid, n, dtype, lo=-2, hi=2):
    return synth.small_ints(seed, tid, n, lo, hi, dtype)


# ----------------------------------------------------------------------------- level 1
@pytest.mark.parametrize("dt", DT)
def test_dot_closed_forms(dt):
    n = 1 << 20
    one = np.ones(n, dt)
    assert O.dot(n, one, 1, one, 1) == n                       # dot of ones = n
    x = synth.uniform(7, 1, 1000, dt)
    e = np.zeros(1000, dt); e[337] = 1
    assert O.dot(1000, x, 1, e, 1) == x[337]                    # x . e_k = x_k
    assert O.dot(0, x, 1, e, 1) == 0
    # dot(x,x) == nrm2(x)^2 up to the two roundings
    r = float(O.nrm2(1000, x, 1)) ** 2
    assert abs(float(O.dot(1000, x, 1, x, 1)) - r) <= 4 * np.finfo(dt).eps * r


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("incx,incy", [(1, 1), (2, 3), (-1, 2), (3, -2), (-2, -1)])
def test_dot_int64_brute_force_and_strides(dt, incx, incy):
    n = 777
    xd, yd = ints(1, 1, n, dt, -9, 9), ints(1, 2, n, dt, -9, 9)
    exact = int(np.dot(xd.astype(np.int64), yd.astype(np.int64)))
    xb, yb = synth.strided(xd, incx), synth.strided(yd, incy)
    r, D = O.dot(n, xb, incx, yb, incy, want_D=True)
    assert float(r) == exact
    assert D == float(np.sum(np.abs(xd.astype(np.int64) * yd.astype(np.int64))))


@pytest.mark.parametrize("dt", DT)
def test_dot_is_not_symmetric_in_direction(dt):
    # negative increment means "reversed vector": x = (1,2,3), y = (1,10,100)
    x = np.array([1, 2, 3], dt); y = np.array([1, 10, 100], dt)
    assert O.dot(3, x, 1, y, 1) == 321
    assert O.dot(3, x, -1, y, 1) == 123
    assert O.dot(3, x, -1, y, -1) == 321


@pytest.mark.parametrize("dt", DT)
def test_asum(dt):
    n = 4097
    s = np.where(np.arange(n) % 3 == 0, -1, 1).astype(dt)
    assert O.asum(n, s, 1) == n
    x = ints(2, 1, n, dt, -7, 7)
    assert float(O.asum(n, x, 1)) == int(np.abs(x.astype(np.int64)).sum())
    # asum(x) = dot(sign(x), x)
    assert O.asum(n, x, 1) == O.dot(n, np.sign(x).astype(dt), 1, x, 1)
    xb = synth.strided(x, 3)
    assert O.asum(n, xb, 3) == O.asum(n, x, 1)                 # NaN gaps never read
    assert O.asum(n, x, 0) == 0 and O.asum(n, x, -1) == 0 and O.asum(0, x, 1) == 0


@pytest.mark.parametrize("dt", DT)
def test_nrm2(dt):
    k = 4 ** 5
    x = np.concatenate([np.full(k, 3, dt), np.full(k, 4, dt)])
    assert O.nrm2(2 * k, x, 1) == 5 * 2 ** 5                   # sqrt(25 k) = 5 sqrt(k)
    z = np.zeros(100, dt); z[41] = -7.5
    assert O.nrm2(100, z, 1) == 7.5
    u = synth.uniform(3, 1, 5000, dt)
    assert O.nrm2(5000, (2 * u).astype(dt), 1) == 2 * O.nrm2(5000, u, 1)
    assert O.nrm2(5000, u, 0) == 0 and O.nrm2(0, u, 1) == 0
    # overflow / underflow safety of the oracle itself
    big = np.full(4, np.finfo(dt).max / 4, dt)
    assert O.nrm2(4, big, 1) == np.finfo(dt).max / 2
    tiny = np.full(4, np.finfo(dt).tiny, dt)
    assert O.nrm2(4, tiny, 1) == 2 * np.finfo(dt).tiny


@pytest.mark.parametrize("dt", DT)
def test_axpy_scal(dt):
    n = 1000
    x = synth.uniform(4, 1, n, dt); y = synth.uniform(4, 2, n, dt)
    y0 = y.copy(); O.axpy(n, dt(0), x, 1, y, 1)
    assert y.tobytes() == y0.tobytes()                          # alpha = 0: y untouched
    z = np.zeros(n, dt); O.axpy(n, dt(1), x, 1, z, 1)
    assert z.tobytes() == x.tobytes()                           # alpha = 1, y = 0: y = x
    xi, yi = ints(5, 1, n, dt, -50, 50), ints(5, 2, n, dt, -50, 50)
    w = yi.copy(); O.axpy(n, dt(3), xi, 1, w, 1)
    assert np.array_equal(w.astype(np.int64), 3 * xi.astype(np.int64) + yi.astype(np.int64))
    O.axpy(n, dt(-3), xi, 1, w, 1)
    assert np.array_equal(w, yi)                                # axpy then axpy(-alpha)
    # hand-worked, not symmetric in x and y
    yy = np.array([10, 20], dt); O.axpy(2, dt(2), np.array([1, 3], dt), 1, yy, 1)
    assert list(yy) == [12, 26]
    s = x.copy(); O.scal(n, dt(1), s, 1); assert s.tobytes() == x.tobytes()
    s = x.copy(); O.scal(n, dt(-1), s, 1); assert np.array_equal(s, -x)
    s = x.copy(); O.scal(n, dt(2), s, 1); assert np.array_equal(s, x * dt(2))
    s = x.copy(); O.scal(n, dt(2), s, 0); assert s.tobytes() == x.tobytes()
    s = x.copy(); O.scal(n, dt(2), s, -1); assert s.tobytes() == x.tobytes()


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("incx,incy", [(2, 3), (-1, 1), (1, -2), (-3, -2)])
def test_axpy_scal_strided_equals_gathered(dt, incx, incy):
    n = 333
    xd, yd = synth.uniform(6, 1, n, dt), synth.uniform(6, 2, n, dt)
    ref = yd.copy(); O.axpy(n, dt(-0.75), xd, 1, ref, 1)
    xb, yb = synth.strided(xd, incx), synth.strided(yd, incy)
    O.axpy(n, dt(-0.75), xb, incx, yb, incy)
    assert np.array_equal(synth.gather(yb, n, incy), ref)
    gaps = np.ones(yb.size, bool); gaps[::abs(incy)] = False
    assert np.isnan(yb[gaps]).all()                             # gap elements unchanged
    if incx > 0:
        r2 = xd.copy(); O.scal(n, dt(1.25), r2, 1)
        O.scal(n, dt(1.25), xb, incx)
        assert np.array_equal(synth.gather(xb, n, incx), r2)


def test_axpy_single_rounding():
    # alpha*x + y is rounded once: (1+2^-12)^2 - 1 = 2^-11 + 2^-24 exactly, whereas rounding the
    # product to fp32 first loses the 2^-24 (a tie that rounds to even) and gives 2^-11.
    x = np.array([1 + 2.0 ** -12], np.float32); a = np.float32(1 + 2.0 ** -12)
    y = np.array([-1.0], np.float32)
    O.axpy(1, a, x, 1, y, 1)
    assert y[0] == np.float32(2.0 ** -11 + 2.0 ** -24)
    assert np.float32(np.float32(a * x[0]) - np.float32(1)) == np.float32(2.0 ** -11)


# ----------------------------------------------------------------------------- gemv
def brute_gemv(trans, m, n, alpha, A, x, beta, y):
    Ai = A.astype(np.int64); xi = x.astype(np.int64); yi = y.astype(np.int64)
    out = []
    leny, lenx = (m, n) if trans == O.NO_TRANS else (n, m)
    for o in range(leny):
        s = 0
        for k in range(lenx):
            s += (Ai[o, k] if trans == O.NO_TRANS else Ai[k, o]) * xi[k]
        out.append(alpha * s + beta * yi[o])
    return np.array(out, np.int64)


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("layout", [O.ROW_MAJOR, O.COL_MAJOR])
@pytest.mark.parametrize("trans", [O.NO_TRANS, O.TRANS])
@pytest.mark.parametrize("m,n", [(1, 1), (3, 5), (8, 8), (7, 2)])
def test_gemv_int64_brute_force(dt, layout, trans, m, n):
    A = ints(8, 0, m * n, dt, -4, 4).reshape(m, n)
    lenx, leny = (n, m) if trans == O.NO_TRANS else (m, n)
    x, y = ints(8, 1, lenx, dt, -4, 4), ints(8, 2, leny, dt, -4, 4)
    exact = brute_gemv(trans, m, n, 3, A, x, -2, y)
    for pad in (0, 3):
        if layout == O.ROW_MAJOR:
            lda = n + pad; buf = np.full((m, lda), np.nan, dt); buf[:, :n] = A
        else:
            lda = m + pad; buf = np.full((n, lda), np.nan, dt); buf[:, :m] = A.T
        for incx, incy in [(1, 1), (2, -3), (-1, 2)]:
            xb, yb = synth.strided(x, incx), synth.strided(y, incy)
            O.gemv(layout, trans, m, n, dt(3), buf.ravel(), lda, xb, incx, dt(-2), yb, incy)
            assert np.array_equal(synth.gather(yb, leny, incy).astype(np.int64), exact)


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("trans", [O.NO_TRANS, O.TRANS])
def test_gemv_batched_int64_brute_force_and_shared_operands(dt, trans):
    # every problem of a batch against exact integer arithmetic on its own slice; gaps between
    # the problems hold NaN (operands) or a marker (y) and must be neither read nor written
    m, n, batch = 5, 7, 4
    lenx, leny = (n, m) if trans == O.NO_TRANS else (m, n)
    for lda, incx, incy, gapA, gapx, gapy in [(n, 1, 1, 0, 0, 0), (n + 2, 2, -3, 5, 3, 4)]:
        sA = m * lda + gapA
        sx, sy = 1 + (lenx - 1) * abs(incx) + gapx, 1 + (leny - 1) * abs(incy) + gapy
        Ab = np.full(batch * sA, np.nan, dt); xb = np.full(batch * sx, np.nan, dt); yb = np.full(batch * sy, 77, dt)
        want = []
        for b in range(batch):
            A = ints(21, 3 * b, m * n, dt, -4, 4).reshape(m, n)
            x, y = ints(21, 3 * b + 1, lenx, dt, -4, 4), ints(21, 3 * b + 2, leny, dt, -4, 4)
            Ab[b * sA:b * sA + m * lda].reshape(m, lda)[:, :n] = A
            xb[b * sx:b * sx + 1 + (lenx - 1) * abs(incx)] = synth.strided(x, incx)
            ys = synth.strided(y, incy); ys[np.isnan(ys)] = 77
            yb[b * sy:b * sy + ys.size] = ys
            want.append(brute_gemv(trans, m, n, 3, A, x, -2, y))
        before = yb.copy()
        O.gemv_batched(O.ROW_MAJOR, trans, m, n, dt(3), Ab, lda, sA, xb, incx, sx, dt(-2), yb, incy, sy, batch)
        touched = np.zeros(yb.size, bool)
        for b in range(batch):
            got = synth.gather(yb[b * sy:], leny, incy)
            assert np.array_equal(got.astype(np.int64), want[b]), (b, lda, incx, incy)
            idx = b * sy + np.arange(leny) * abs(incy)
            touched[idx] = True
        assert np.array_equal(yb[~touched], before[~touched])       # nothing between or after the vectors
    # stride 0 shares an operand: one matrix, `batch` vectors = the columns of a matrix product
    A = ints(22, 0, m * n, dt, -3, 3).reshape(m, n)
    X = ints(22, 1, batch * lenx, dt, -3, 3).reshape(batch, lenx)
    Y = np.zeros((batch, leny), dt)
    O.gemv_batched(O.ROW_MAJOR, trans, m, n, dt(1), A.ravel(), n, 0, X.ravel(), 1, lenx, dt(0), Y.ravel(), 1, leny, batch)
    op = A.astype(np.int64) if trans == O.NO_TRANS else A.astype(np.int64).T
    assert np.array_equal(Y.astype(np.int64), (op @ X.astype(np.int64).T).T)
    # an empty batch touches nothing
    Y0 = Y.copy()
    O.gemv_batched(O.ROW_MAJOR, trans, m, n, dt(1), A.ravel(), n, 0, X.ravel(), 1, lenx, dt(0), Y.ravel(), 1, leny, 0)
    assert Y.tobytes() == Y0.tobytes()


@pytest.mark.parametrize("dt", DT)
def test_gemv_closed_forms(dt):
    n = 64
    x, y = synth.uniform(9, 1, n, dt), synth.uniform(9, 2, n, dt)
    I = np.eye(n, dtype=dt)
    for trans in (O.NO_TRANS, O.TRANS):
        out = y.copy()
        O.gemv(O.ROW_MAJOR, trans, n, n, dt(1), I.ravel(), n, x, 1, dt(0), out, 1)
        assert out.tobytes() == x.tobytes()                    # identity returns x
        out = y.copy()
        O.gemv(O.ROW_MAJOR, trans, n, n, dt(0), I.ravel(), n, x, 1, dt(1), out, 1)
        assert out.tobytes() == y.tobytes()                    # alpha=0, beta=1: untouched
        out = y.copy()                                         # alpha*x + beta*y, exact scalars
        O.gemv(O.ROW_MAJOR, trans, n, n, dt(2), I.ravel(), n, x, 1, dt(0.5), out, 1)
        assert np.array_equal(out, dt(2) * x + dt(0.5) * y)
    # A[i,j] = i + j, x = 1  ->  y_i = N*i + N(N-1)/2  (N), y_j = M*j + M(M-1)/2 (T)
    m, k = 12, 20
    A = (np.arange(m)[:, None] + np.arange(k)[None, :]).astype(dt)
    out = np.zeros(m, dt)
    O.gemv(O.ROW_MAJOR, O.NO_TRANS, m, k, dt(1), A.ravel(), k, np.ones(k, dt), 1, dt(0), out, 1)
    assert np.array_equal(out, k * np.arange(m) + k * (k - 1) // 2)
    out = np.zeros(k, dt)
    O.gemv(O.ROW_MAJOR, O.TRANS, m, k, dt(1), A.ravel(), k, np.ones(m, dt), 1, dt(0), out, 1)
    assert np.array_equal(out, m * np.arange(k) + m * (m - 1) // 2)
    # single non-zero entry A[2,5] = 7 picks x[5] into y[2] (N) and x[2] into y[5] (T)
    A = np.zeros((m, k), dt); A[2, 5] = 7
    xs = np.arange(1, k + 1).astype(dt); out = np.zeros(m, dt)
    O.gemv(O.ROW_MAJOR, O.NO_TRANS, m, k, dt(1), A.ravel(), k, xs, 1, dt(0), out, 1)
    assert out[2] == 7 * 6 and np.count_nonzero(out) == 1
    xs = np.arange(1, m + 1).astype(dt); out = np.zeros(k, dt)
    O.gemv(O.ROW_MAJOR, O.TRANS, m, k, dt(1), A.ravel(), k, xs, 1, dt(0), out, 1)
    assert out[5] == 7 * 3 and np.count_nonzero(out) == 1
    # all-ones matrix ties gemv to dot
    xs = synth.uniform(9, 1, k, dt); out = np.zeros(m, dt)
    O.gemv(O.ROW_MAJOR, O.NO_TRANS, m, k, dt(1), np.ones(m * k, dt), k, xs, 1, dt(0), out, 1)
    assert (out == O.dot(k, xs, 1, np.ones(k, dt), 1)).all()


@pytest.mark.parametrize("dt", DT)
def test_gemv_epilogue_special_values(dt):
    m, n = 5, 7
    A = synth.uniform(10, 0, m * n, dt); x = synth.uniform(10, 1, n, dt)
    y = np.full(m, np.nan, dt)
    O.gemv(O.ROW_MAJOR, O.NO_TRANS, m, n, dt(1.5), A, n, x, 1, dt(0), y, 1)
    assert np.isfinite(y).all()                                # beta=0: y overwritten, not read
    y0 = synth.uniform(10, 2, m, dt); y = y0.copy()
    O.gemv(O.ROW_MAJOR, O.NO_TRANS, m, n, dt(0), np.full(m * n, np.nan, dt), n,
           np.full(n, np.nan, dt), 1, dt(0.5), y, 1)
    assert np.array_equal(y, dt(0.5) * y0)                     # alpha=0: A, x not read
    y = y0.copy()
    O.gemv(O.ROW_MAJOR, O.NO_TRANS, 0, n, dt(1), A, n, x, 1, dt(0), y, 1)
    O.gemv(O.ROW_MAJOR, O.NO_TRANS, m, 0, dt(1), A, 1, x, 1, dt(0), y, 1)
    assert y.tobytes() == y0.tobytes()                         # empty problem: quick return


@pytest.mark.parametrize("dt,tol", [(np.float32, 1e-6), (np.float64, 1e-14)])
def test_gemv_against_independent_fp64_library(dt, tol):
    m, n = 200, 300
    A = synth.uniform(11, 0, m * n, dt).reshape(m, n)
    for trans, lenx, leny in ((O.NO_TRANS, n, m), (O.TRANS, m, n)):
        x, y = synth.uniform(11, 1, lenx, dt), synth.uniform(11, 2, leny, dt)
        out = y.copy()
        D = O.gemv(O.ROW_MAJOR, trans, m, n, dt(1.5), A.ravel(), n, x, 1, dt(0.5), out, 1, want_D=True)
        Ad = A.astype(np.float64)
        ref = 1.5 * ((Ad if trans == O.NO_TRANS else Ad.T) @ x.astype(np.float64)) + 0.5 * y
        assert np.max(np.abs(out - ref) / D) < tol
        refD = 1.5 * (np.abs(Ad if trans == O.NO_TRANS else Ad.T) @ np.abs(x.astype(np.float64))) \
            + 0.5 * np.abs(y)
        assert np.allclose(D, refD, rtol=1e-12)
    # gemv-T(A) == gemv-N(explicit transpose)
    x = synth.uniform(11, 1, m, dt)
    a = np.zeros(n, dt); b = np.zeros(n, dt)
    O.gemv(O.ROW_MAJOR, O.TRANS, m, n, dt(1), A.ravel(), n, x, 1, dt(0), a, 1)
    O.gemv(O.ROW_MAJOR, O.NO_TRANS, n, m, dt(1), np.ascontiguousarray(A.T).ravel(), m, x, 1, dt(0), b, 1)
    assert a.tobytes() == b.tobytes()


def test_gemv_golden_worked_example():
    """tests/golden/gemv_3x2.txt: a 3x2 case worked by hand from the Sec. 2 loop nest."""
    rows = [l.split("#")[0].split() for l in open(os.path.join(GOLDEN, "gemv_3x2.txt"))]
    vals = {r[0]: [float(v) for v in r[1:]] for r in rows if r}
    A = np.array(vals["A"], np.float32)
    for key, trans, xk, yk in (("yN", O.NO_TRANS, "xN", "y0N"), ("yT", O.TRANS, "xT", "y0T")):
        y = np.array(vals[yk], np.float32)
        O.gemv(O.ROW_MAJOR, trans, 3, 2, np.float32(vals["alpha"][0]), A, 2,
               np.array(vals[xk], np.float32), 1, np.float32(vals["beta"][0]), y, 1)
        assert list(y) == vals[key]


# ----------------------------------------------------------------------------- trmv / symv / ger
def explicit_tri(A, uplo, diag):
    Tm = np.triu(A) if uplo == O.UPPER else np.tril(A)
    if diag == O.UNIT:
        np.fill_diagonal(Tm, 1)
    return Tm


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("layout", [O.ROW_MAJOR, O.COL_MAJOR])
@pytest.mark.parametrize("uplo", [O.UPPER, O.LOWER])
@pytest.mark.parametrize("trans", [O.NO_TRANS, O.TRANS])
@pytest.mark.parametrize("diag", [O.NON_UNIT, O.UNIT])
def test_trmv_equals_gemv_on_explicit_triangle_and_ignores_the_rest(dt, layout, uplo, trans, diag):
    n = 37
    A = ints(12, 0, n * n, dt, -3, 3).reshape(n, n)
    x = ints(12, 1, n, dt, -3, 3)
    Tm = explicit_tri(A.copy(), uplo, diag)
    exact = (Tm.astype(np.int64) if trans == O.NO_TRANS else Tm.astype(np.int64).T) @ x.astype(np.int64)
    # poison everything that must not be read
    P = A.copy()
    mask = np.tril(np.ones((n, n), bool), -1) if uplo == O.UPPER else np.triu(np.ones((n, n), bool), 1)
    P[mask] = np.nan
    if diag == O.UNIT:
        np.fill_diagonal(P, np.nan)
    lda = n + 2
    buf = np.full((n, lda), np.nan, dt)
    buf[:, :n] = P if layout == O.ROW_MAJOR else P.T
    for incx in (1, 2, -1):
        xb = synth.strided(x, incx)
        O.trmv(layout, uplo, trans, diag, n, buf.ravel(), lda, xb, incx)
        assert np.array_equal(synth.gather(xb, n, incx).astype(np.int64), exact)


def test_trmv_hand_worked():
    # U = [[2,3],[.,5]], x = (1,10): U x = (32, 50); U^T x = (2, 53); unit: (31,10) / (1,13)
    A = np.array([2, 3, np.nan, 5], np.float64)
    for trans, diag, want in ((O.NO_TRANS, O.NON_UNIT, [32, 50]), (O.TRANS, O.NON_UNIT, [2, 53]),
                              (O.NO_TRANS, O.UNIT, [31, 10]), (O.TRANS, O.UNIT, [1, 13])):
        x = np.array([1, 10], np.float64)
        O.trmv(O.ROW_MAJOR, O.UPPER, trans, diag, 2, A, 2, x, 1)
        assert list(x) == want
    # L = [[1,.,.],[2,3,.],[4,5,6]], x = (1,10,100): L x = (1, 32, 654); L^T x = (421, 530, 600)
    L = np.array([1, np.nan, np.nan, 2, 3, np.nan, 4, 5, 6], np.float32)
    x = np.array([1, 10, 100], np.float32); O.trmv(O.ROW_MAJOR, O.LOWER, O.NO_TRANS, O.NON_UNIT, 3, L, 3, x, 1)
    assert list(x) == [1, 32, 654]
    x = np.array([1, 10, 100], np.float32); O.trmv(O.ROW_MAJOR, O.LOWER, O.TRANS, O.NON_UNIT, 3, L, 3, x, 1)
    assert list(x) == [421, 530, 600]
    I = np.eye(5); x = np.arange(5.0); O.trmv(O.ROW_MAJOR, O.UPPER, O.NO_TRANS, O.NON_UNIT, 5, I.ravel(), 5, x, 1)
    assert list(x) == [0, 1, 2, 3, 4]


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("layout", [O.ROW_MAJOR, O.COL_MAJOR])
@pytest.mark.parametrize("uplo", [O.UPPER, O.LOWER])
def test_symv_equals_gemv_on_symmetrised_matrix(dt, layout, uplo):
    n = 29
    A = ints(13, 0, n * n, dt, -3, 3).reshape(n, n)
    x, y = ints(13, 1, n, dt, -3, 3), ints(13, 2, n, dt, -3, 3)
    Tm = np.triu(A) if uplo == O.UPPER else np.tril(A)
    S = Tm + Tm.T - np.diag(np.diag(A))
    exact = 2 * (S.astype(np.int64) @ x.astype(np.int64)) - 3 * y.astype(np.int64)
    P = A.copy()
    mask = np.tril(np.ones((n, n), bool), -1) if uplo == O.UPPER else np.triu(np.ones((n, n), bool), 1)
    P[mask] = np.nan
    lda = n + 1
    buf = np.full((n, lda), np.nan, dt)
    buf[:, :n] = P if layout == O.ROW_MAJOR else P.T
    for incx, incy in ((1, 1), (-2, 3)):
        xb, yb = synth.strided(x, incx), synth.strided(y, incy)
        O.symv(layout, uplo, n, dt(2), buf.ravel(), lda, xb, incx, dt(-3), yb, incy)
        assert np.array_equal(synth.gather(yb, n, incy).astype(np.int64), exact)
    # upper(A) and lower(A^T) describe the same symmetric matrix
    if layout == O.ROW_MAJOR:
        other = O.LOWER if uplo == O.UPPER else O.UPPER
        a = y.copy(); b = y.copy()
        O.symv(O.ROW_MAJOR, uplo, n, dt(1), np.nan_to_num(P).ravel(), n, x, 1, dt(1), a, 1)
        O.symv(O.ROW_MAJOR, other, n, dt(1), np.ascontiguousarray(np.nan_to_num(P).T).ravel(), n, x, 1, dt(1), b, 1)
        assert np.array_equal(a, b)
    # beta = 0 overwrites NaN; alpha = 0 reads no A
    yn = np.full(n, np.nan, dt)
    O.symv(layout, uplo, n, dt(1), buf.ravel(), lda, x, 1, dt(0), yn, 1)
    assert np.isfinite(yn).all()


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("layout", [O.ROW_MAJOR, O.COL_MAJOR])
def test_ger(dt, layout):
    m, n = 9, 14
    x, y = ints(14, 1, m, dt, -5, 5), ints(14, 2, n, dt, -5, 5)
    A = ints(14, 0, m * n, dt, -5, 5).reshape(m, n)
    exact = A.astype(np.int64) + 3 * np.outer(x.astype(np.int64), y.astype(np.int64))
    lda = (n if layout == O.ROW_MAJOR else m) + 2
    shape = (m, lda) if layout == O.ROW_MAJOR else (n, lda)
    buf = np.full(shape, np.nan, dt)
    if layout == O.ROW_MAJOR:
        buf[:, :n] = A
    else:
        buf[:, :m] = A.T
    for incx, incy in ((1, 1), (2, -1)):
        b = buf.copy()
        O.ger(layout, m, n, dt(3), synth.strided(x, incx), incx, synth.strided(y, incy), incy, b.ravel(), lda)
        got = b[:, :n] if layout == O.ROW_MAJOR else b[:, :m].T
        assert np.array_equal(got.astype(np.int64), exact)
        assert np.isnan(b[:, (n if layout == O.ROW_MAJOR else m):]).all()
    b = buf.copy(); O.ger(layout, m, n, dt(0), x, 1, y, 1, b.ravel(), lda)
    assert b.tobytes() == buf.tobytes()                        # alpha = 0: A untouched
    # A = 0 -> alpha*x_i*y_j with one rounding
    xu, yu = synth.uniform(14, 1, m, dt), synth.uniform(14, 2, n, dt)
    Z = np.zeros((m, n), dt)
    O.ger(O.ROW_MAJOR, m, n, dt(0.3), xu, 1, yu, 1, Z.ravel(), n)
    ref = np.float64(dt(0.3)) * np.outer(xu.astype(np.float64), yu.astype(np.float64))
    if dt == np.float32:
        # (double product of three floats is exact to 2^-53 relative; one rounding to float)
        assert np.max(np.abs(Z - ref.astype(np.float32)) / np.abs(ref)) <= 2.0 ** -23
    else:
        assert np.max(np.abs(Z - ref) / np.abs(ref)) <= 2.0 ** -52
    # (A + a x y^T) z = A z + a x (y^T z) on integers
    z = ints(14, 3, n, dt, -5, 5)
    B = A.copy(); O.ger(O.ROW_MAJOR, m, n, dt(3), x, 1, y, 1, B.ravel(), n)
    lhs = np.zeros(m, dt); O.gemv(O.ROW_MAJOR, O.NO_TRANS, m, n, dt(1), B.ravel(), n, z, 1, dt(0), lhs, 1)
    rhs = np.zeros(m, dt); O.gemv(O.ROW_MAJOR, O.NO_TRANS, m, n, dt(1), A.ravel(), n, z, 1, dt(0), rhs, 1)
    O.axpy(m, dt(3) * O.dot(n, y, 1, z, 1), x, 1, rhs, 1)
    assert np.array_equal(lhs, rhs)


def test_accumulation_is_wider_than_fp64():
    # 1 + 2^-60 - 1 summed left to right: survives only with a 64-bit significand
    x = np.array([1.0, 2.0 ** -60, -1.0]); one = np.ones(3)
    assert O.dot(3, x, 1, one, 1) == 2.0 ** -60
    A = x.copy(); y = np.zeros(1)
    O.gemv(O.ROW_MAJOR, O.NO_TRANS, 1, 3, 1.0, A, 3, one, 1, 0.0, y, 1)
    assert y[0] == 2.0 ** -60


def test_synth_generators_are_deterministic_and_in_range():
    a = synth.uniform(1, 1, 10000, np.float32); b = synth.uniform(1, 1, 10000, np.float32)
    assert a.tobytes() == b.tobytes() and a.min() >= -1 and a.max() < 1
    assert synth.uniform(1, 2, 100).tobytes() != synth.uniform(1, 1, 100).tobytes()
    # chunk boundaries do not matter: element i depends on (seed, tensor, i) only
    assert synth.uniform(5, 0, (1 << 20) + 10)[-10:].tobytes() == \
        np.array([synth.uniform(5, 0, (1 << 20) + k + 1)[-1] for k in range(10)], np.float32).tobytes()
    z = synth.normal(3, 0, 200000, 1 / 128.0)
    assert abs(z.std() * 128 - 1) < 0.01 and abs(z.mean()) < 1e-3


# ----------------------------------------------------------------------------- rest of level 1
@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("incx,incy", [(1, 1), (2, 3), (-1, 2), (3, -2)])
def test_copy_swap(dt, incx, incy):
    n = 301
    xd, yd = synth.uniform(20, 1, n, dt), synth.uniform(20, 2, n, dt)
    xb, yb = synth.strided(xd, incx), synth.strided(yd, incy)
    O.copy(n, xb, incx, yb, incy)
    assert np.array_equal(synth.gather(yb, n, incy), xd) and np.array_equal(synth.gather(xb, n, incx), xd)
    gaps = np.ones(yb.size, bool); gaps[::abs(incy)] = False
    assert np.isnan(yb[gaps]).all()
    xb, yb = synth.strided(xd, incx), synth.strided(yd, incy)
    O.swap(n, xb, incx, yb, incy)
    assert np.array_equal(synth.gather(xb, n, incx), yd) and np.array_equal(synth.gather(yb, n, incy), xd)
    O.swap(n, xb, incx, yb, incy)                                  # twice = identity
    assert np.array_equal(synth.gather(xb, n, incx), xd) and np.array_equal(synth.gather(yb, n, incy), yd)


@pytest.mark.parametrize("dt", DT)
def test_rot(dt):
    n = 200
    x, y = ints(21, 1, n, dt, -9, 9), ints(21, 2, n, dt, -9, 9)
    a, b = x.copy(), y.copy(); O.rot(n, a, 1, b, 1, dt(1), dt(0))
    assert np.array_equal(a, x) and np.array_equal(b, y)          # c=1, s=0: identity
    a, b = x.copy(), y.copy(); O.rot(n, a, 1, b, 1, dt(0), dt(1))
    assert np.array_equal(a, y) and np.array_equal(b, -x)         # c=0, s=1: (y, -x)
    a, b = x.copy(), y.copy(); O.rot(n, a, 1, b, 1, dt(3), dt(4))  # integer brute force, not symmetric in x, y
    xi, yi = x.astype(np.int64), y.astype(np.int64)
    assert np.array_equal(a.astype(np.int64), 3 * xi + 4 * yi) and np.array_equal(b.astype(np.int64), 3 * yi - 4 * xi)
    # a true rotation keeps x^2 + y^2
    u, v = synth.uniform(21, 1, n, dt), synth.uniform(21, 2, n, dt)
    c, s = dt(np.cos(0.7)), dt(np.sin(0.7))
    a, b = u.copy(), v.copy(); O.rot(n, a, 1, b, 1, c, s)
    assert np.allclose(a.astype(np.float64) ** 2 + b.astype(np.float64) ** 2, u.astype(np.float64) ** 2 + v.astype(np.float64) ** 2,
                       rtol=20 * np.finfo(dt).eps)
    # strided = gathered
    ub, vb = synth.strided(u, -2), synth.strided(v, 3)
    O.rot(n, ub, -2, vb, 3, c, s)
    assert np.array_equal(synth.gather(ub, n, -2), a) and np.array_equal(synth.gather(vb, n, 3), b)


@pytest.mark.parametrize("dt", DT)
def test_rotm(dt):
    n = 100
    x, y = ints(22, 1, n, dt, -9, 9), ints(22, 2, n, dt, -9, 9)
    xi, yi = x.astype(np.int64), y.astype(np.int64)
    h11, h21, h12, h22 = 2, 3, 5, 7
    cases = {
        -1: (h11 * xi + h12 * yi, h21 * xi + h22 * yi),
        0: (xi + h12 * yi, h21 * xi + yi),
        1: (h11 * xi + yi, -xi + h22 * yi),
        -2: (xi, yi),
    }
    for flag, (ex, ey) in cases.items():
        a, b = x.copy(), y.copy()
        O.rotm(n, a, 1, b, 1, np.array([flag, h11, h21, h12, h22], dt))
        assert np.array_equal(a.astype(np.int64), ex) and np.array_equal(b.astype(np.int64), ey), flag
    # flag -2 does not even read H
    a, b = x.copy(), y.copy(); O.rotm(n, a, 1, b, 1, np.array([-2, np.nan, np.nan, np.nan, np.nan], dt))
    assert np.array_equal(a, x) and np.array_equal(b, y)
    # rotm with flag -1 and H = [c s; -s c] is rot
    c, s = dt(0.6), dt(0.8)
    u, v = synth.uniform(22, 1, n, dt), synth.uniform(22, 2, n, dt)
    a, b = u.copy(), v.copy(); O.rotm(n, a, 1, b, 1, np.array([-1, c, -s, s, c], dt))
    a2, b2 = u.copy(), v.copy(); O.rot(n, a2, 1, b2, 1, c, s)
    assert np.array_equal(a, a2) and np.array_equal(b, b2)


def test_dsdot():
    n = 1001
    x, y = ints(23, 1, n, np.float32, -99, 99), ints(23, 2, n, np.float32, -99, 99)
    assert O.dsdot(n, x, 1, y, 1) == int(np.dot(x.astype(np.int64), y.astype(np.int64)))
    xb, yb = synth.strided(x, 2), synth.strided(y, -3)
    assert O.dsdot(n, xb, 2, yb, -3) == int(np.dot(x.astype(np.int64), y.astype(np.int64)))
    # products and the sum are carried wider than fp32: 1 + 2^-30 - 1
    a = np.array([1, 2.0 ** -30, -1], np.float32); one = np.ones(3, np.float32)
    assert O.dsdot(3, a, 1, one, 1) == 2.0 ** -30 and O.dot(3, a, 1, one, 1) == np.float32(2.0 ** -30)
    big = np.array([3e20, 3e20], np.float32)            # product overflows fp32, not fp64
    assert O.dsdot(2, big, 1, big, 1) == 2 * float(np.float32(3e20)) ** 2
    assert O.dsdot(0, x, 1, y, 1) == 0


@pytest.mark.parametrize("dt", DT)
def test_iamax(dt):
    assert O.iamax(5, np.array([1, -7, 3, 7, -2], dt), 1) == 1          # first of equal maxima, sign ignored
    assert O.iamax(5, np.array([0, 0, 0, 0, 0], dt), 1) == 0
    assert O.iamax(4, np.array([1, np.nan, 5, 2], dt), 1) == 2          # a NaN is never taken ...
    assert O.iamax(4, np.array([np.nan, 9, 5, 2], dt), 1) == 0          # ... unless it comes first
    assert O.iamax(3, np.array([1, np.inf, -np.inf], dt), 1) == 1
    assert O.iamax(0, np.array([1.0], dt), 1) == 0 and O.iamax(3, np.array([1, 2, 3], dt), 0) == 0
    assert O.iamax(3, np.array([1, 2, 3], dt), -1) == 0
    x = synth.uniform(24, 1, 5000, dt)
    assert O.iamax(5000, x, 1) == int(np.argmax(np.abs(x)))
    xb = synth.strided(x, 3, fill=99.0)                                  # the gaps must not be looked at
    assert O.iamax(5000, xb, 3) == int(np.argmax(np.abs(x)))


# ----------------------------------------------------------------------------- syr, syr2, trsv
def tri_buffer(A, layout, uplo, pad, dt, unit=False):
    """Row- or column-major buffer of the square matrix A with NaN in the padding, in the triangle
    opposite to uplo and (unit) on the diagonal."""
    n = A.shape[0]
    P = A.astype(dt).copy()
    outside = np.tril(np.ones((n, n), bool), -1) if uplo == O.UPPER else np.triu(np.ones((n, n), bool), 1)
    P[outside] = np.nan
    if unit:
        np.fill_diagonal(P, np.nan)
    lda = n + pad
    buf = np.full((n, lda), np.nan, dt)
    buf[:, :n] = P if layout == O.ROW_MAJOR else P.T
    return buf, lda, outside


def tri_logical(buf, layout, n):
    return buf[:, :n] if layout == O.ROW_MAJOR else buf[:, :n].T


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("layout", [O.ROW_MAJOR, O.COL_MAJOR])
@pytest.mark.parametrize("uplo", [O.UPPER, O.LOWER])
def test_syr_syr2_int64_brute_force_and_untouched_rest(dt, layout, uplo):
    n = 13
    A = ints(21, 0, n * n, dt, -5, 5).reshape(n, n)
    x, y = ints(21, 1, n, dt, -5, 5), ints(21, 2, n, dt, -5, 5)
    xi, yi, Ai = x.astype(np.int64), y.astype(np.int64), A.astype(np.int64)
    buf, lda, outside = tri_buffer(A, layout, uplo, 3, dt)
    for incx, incy in ((1, 1), (2, -3), (-1, 2)):
        xb, yb = synth.strided(x, incx), synth.strided(y, incy)
        b = buf.copy(); O.syr(layout, uplo, n, dt(3), xb, incx, b.ravel(), lda)
        got = tri_logical(b, layout, n)
        want = Ai + 3 * np.outer(xi, xi)
        assert np.array_equal(got[~outside].astype(np.int64), want[~outside])
        assert np.isnan(got[outside]).all() and np.isnan(b[:, n:]).all()     # never read, never written
        b = buf.copy(); O.syr2(layout, uplo, n, dt(-2), xb, incx, yb, incy, b.ravel(), lda)
        got = tri_logical(b, layout, n)
        want = Ai - 2 * (np.outer(xi, yi) + np.outer(yi, xi))
        assert np.array_equal(got[~outside].astype(np.int64), want[~outside])
        assert np.isnan(got[outside]).all() and np.isnan(b[:, n:]).all()
    b = buf.copy(); O.syr(layout, uplo, n, dt(0), x, 1, b.ravel(), lda)
    assert b.tobytes() == buf.tobytes()                                      # alpha = 0: untouched
    b = buf.copy(); O.syr2(layout, uplo, n, dt(0), x, 1, y, 1, b.ravel(), lda)
    assert b.tobytes() == buf.tobytes()


@pytest.mark.parametrize("dt", DT)
def test_syr_syr2_tie_to_ger_symv_and_each_other(dt):
    n = 11
    A = ints(22, 0, n * n, dt, -4, 4).reshape(n, n)
    A = np.tril(A) + np.tril(A, -1).T                                        # symmetric, integer
    x, y, z = ints(22, 1, n, dt, -4, 4), ints(22, 2, n, dt, -4, 4), ints(22, 3, n, dt, -4, 4)
    for uplo in (O.UPPER, O.LOWER):
        keep = np.triu(np.ones((n, n), bool)) if uplo == O.UPPER else np.tril(np.ones((n, n), bool))
        # syr == ger(x, x) inside the triangle
        S = A.copy(); O.syr(O.ROW_MAJOR, uplo, n, dt(2), x, 1, S.ravel(), n)
        Gm = A.copy(); O.ger(O.ROW_MAJOR, n, n, dt(2), x, 1, x, 1, Gm.ravel(), n)
        assert np.array_equal(S[keep], Gm[keep]) and np.array_equal(S[~keep], A[~keep])
        # syr2 == ger(x, y) then ger(y, x) inside the triangle; symmetric in x <-> y; syr2(x, x, a) == syr(x, 2a)
        S2 = A.copy(); O.syr2(O.ROW_MAJOR, uplo, n, dt(3), x, 1, y, 1, S2.ravel(), n)
        G2 = A.copy(); O.ger(O.ROW_MAJOR, n, n, dt(3), x, 1, y, 1, G2.ravel(), n); O.ger(O.ROW_MAJOR, n, n, dt(3), y, 1, x, 1, G2.ravel(), n)
        assert np.array_equal(S2[keep], G2[keep])
        S3 = A.copy(); O.syr2(O.ROW_MAJOR, uplo, n, dt(3), y, 1, x, 1, S3.ravel(), n)
        assert np.array_equal(S2, S3)
        S4 = A.copy(); O.syr2(O.ROW_MAJOR, uplo, n, dt(1), x, 1, x, 1, S4.ravel(), n)
        assert np.array_equal(S4, S)
        # (A + a x x^T) z = A z + a x (x^T z): symv of the updated triangle against symv + dot + axpy
        lhs = np.zeros(n, dt); O.symv(O.ROW_MAJOR, uplo, n, dt(1), S.ravel(), n, z, 1, dt(0), lhs, 1)
        rhs = np.zeros(n, dt); O.symv(O.ROW_MAJOR, uplo, n, dt(1), A.ravel(), n, z, 1, dt(0), rhs, 1)
        O.axpy(n, dt(2) * O.dot(n, x, 1, z, 1), x, 1, rhs, 1)
        assert np.array_equal(lhs, rhs)
    # one rounding: A = 0 gives alpha*x_i*x_j rounded once
    xu = synth.uniform(22, 4, n, dt)
    Z = np.zeros((n, n), dt); O.syr(O.ROW_MAJOR, O.LOWER, n, dt(0.3), xu, 1, Z.ravel(), n)
    ref = np.float64(dt(0.3)) * np.outer(xu.astype(np.float64), xu.astype(np.float64))
    low = np.tril(np.ones((n, n), bool))
    assert np.max(np.abs(Z[low] - ref[low].astype(dt)) / np.abs(ref[low])) <= 2 * np.finfo(dt).eps
    assert (Z[~low] == 0).all()


def test_trsv_hand_worked():
    # L = [[2,.,.],[1,4,.],[3,5,10]]: L z = (2, 9, 66) has z = (1, 2, 5.3); L^T z = (13, 23, 30) has z = (1, 2, 3)
    L = np.array([2, np.nan, np.nan, 1, 4, np.nan, 3, 5, 10], np.float64)
    x = np.array([2, 9, 66], np.float64); O.trsv(O.ROW_MAJOR, O.LOWER, O.NO_TRANS, O.NON_UNIT, 3, L, 3, x, 1)
    assert list(x) == [1, 2, 5.3]
    x = np.array([13, 23, 30], np.float64); O.trsv(O.ROW_MAJOR, O.LOWER, O.TRANS, O.NON_UNIT, 3, L, 3, x, 1)
    assert list(x) == [1, 2, 3]
    # unit diagonal: L1 = [[1,.,.],[1,1,.],[3,5,1]]: L1 z = (1, 3, 16) has z = (1, 2, 3)
    L[0] = L[4] = L[8] = np.nan
    x = np.array([1, 3, 16], np.float64); O.trsv(O.ROW_MAJOR, O.LOWER, O.NO_TRANS, O.UNIT, 3, L, 3, x, 1)
    assert list(x) == [1, 2, 3]
    # U = [[2,3],[.,5]]: U z = (32, 50) has z = (1, 10); U^T z = (2, 53) has z = (1, 10)
    U = np.array([2, 3, np.nan, 5], np.float32)
    x = np.array([32, 50], np.float32); O.trsv(O.ROW_MAJOR, O.UPPER, O.NO_TRANS, O.NON_UNIT, 2, U, 2, x, 1)
    assert list(x) == [1, 10]
    x = np.array([2, 53], np.float32); O.trsv(O.ROW_MAJOR, O.UPPER, O.TRANS, O.NON_UNIT, 2, U, 2, x, 1)
    assert list(x) == [1, 10]
    # a diagonal matrix divides: one correctly rounded division per element
    d = np.array([3, 7, 0.3], np.float32); b = np.array([1, 2, 5], np.float32)
    x = b.copy(); O.trsv(O.ROW_MAJOR, O.UPPER, O.NO_TRANS, O.NON_UNIT, 3, np.diag(d).ravel(), 3, x, 1)
    assert np.array_equal(x, b / d)


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("layout", [O.ROW_MAJOR, O.COL_MAJOR])
@pytest.mark.parametrize("uplo", [O.UPPER, O.LOWER])
@pytest.mark.parametrize("trans", [O.NO_TRANS, O.TRANS])
def test_trsv_inverts_trmv_exactly_on_unit_integer_triangles(dt, layout, uplo, trans):
    # unit triangular integer T and integer z: b = op(T) z is exact, and substitution stays in the integers
    n = 24
    A = ints(23, 0, n * n, dt, -1, 1).reshape(n, n)
    z = ints(23, 1, n, dt, -2, 2)
    buf, lda, _ = tri_buffer(A, layout, uplo, 2, dt, unit=True)
    for incx in (1, 3, -2):
        xb = synth.strided(z, incx)
        O.trmv(layout, uplo, trans, O.UNIT, n, buf.ravel(), lda, xb, incx)
        assert np.abs(synth.gather(xb, n, incx)).max() < 2 ** 20
        O.trsv(layout, uplo, trans, O.UNIT, n, buf.ravel(), lda, xb, incx)
        assert np.array_equal(synth.gather(xb, n, incx), z)
        gaps = np.ones(xb.size, bool); gaps[::abs(incx)] = False
        assert np.isnan(xb[gaps]).all()


@pytest.mark.parametrize("dt,tol", [(np.float32, 2e-6), (np.float64, 4e-15)])
@pytest.mark.parametrize("uplo", [O.UPPER, O.LOWER])
@pytest.mark.parametrize("trans", [O.NO_TRANS, O.TRANS])
@pytest.mark.parametrize("diag", [O.NON_UNIT, O.UNIT])
def test_trsv_against_independent_fp64_library(dt, tol, uplo, trans, diag):
    import scipy.linalg
    n = 60
    A = synth.uniform(24, 0, n * n, dt).reshape(n, n) / dt(8)               # off-diagonal small: well conditioned
    A[np.arange(n), np.arange(n)] = dt(1) + np.abs(synth.uniform(24, 5, n, dt))
    b = synth.uniform(24, 1, n, dt)
    Tm = explicit_tri(A.copy(), uplo, diag).astype(np.float64)
    want = scipy.linalg.solve_triangular(Tm, b.astype(np.float64), lower=(uplo == O.LOWER), trans=1 if trans == O.TRANS else 0)
    buf, lda, _ = tri_buffer(A, O.ROW_MAJOR, uplo, 1, dt, unit=(diag == O.UNIT))
    x = b.copy(); D = O.trsv(O.ROW_MAJOR, uplo, trans, diag, n, buf.ravel(), lda, x, 1, want_D=True)
    assert np.max(np.abs(x - want) / np.abs(want).max()) <= tol
    assert (D >= np.abs(x.astype(np.float64)) * (1 - 1e-6)).all()            # D bounds the terms of each unknown
    # the residual of the rounded solution is at rounding level: |b - op(T) x| <= eps * (|op(T)| |x| + |b|)
    opT = Tm if trans == O.NO_TRANS else Tm.T
    r = np.abs(b.astype(np.float64) - opT @ x.astype(np.float64))
    assert (r <= 2 * np.finfo(dt).eps * (np.abs(opT) @ np.abs(x.astype(np.float64)) + np.abs(b))).all()


# ----------------------------------------------------------------------------- condition denominators
# The tolerance gate of the GPU parity tests divides by the oracle's side output D (the sum of the
# absolute values of the terms of each output).  An inflated D would loosen that gate, so every
# routine's D is pinned here against an expression of numpy's own, built from explicit dense
# operands (|M| @ |v| and the like) instead of the oracle's element loops.  Integer-valued inputs
# make every term exact, so the comparison is for equality up to fp64 summation order; each check
# is followed by one that shows D reacts when a term is left out (a D that ignored alpha, beta,
# the diagonal or the second operand would pass neither).
def small(seed, tid, n, dt, lo=-4, hi=4):
    return synth.small_ints(seed, tid, n, lo, hi, dt)


def rel_eq(a, b, tol=1e-12):
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    return np.all(np.abs(a - b) <= tol * np.maximum(np.abs(b), 1e-300))


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("incx,incy", [(1, 1), (2, 3), (-1, 2)])
def test_D_level1(dt, incx, incy):
    n = 53
    x, y = small(40, 1, n, dt), small(40, 2, n, dt)
    alpha = dt(-3)
    xb, yb = synth.strided(x, incx), synth.strided(y, incy)
    D = O.axpy(n, alpha, xb, incx, yb.copy(), incy, want_D=True)
    want = np.abs(np.float64(alpha)) * np.abs(x.astype(np.float64)) + np.abs(y.astype(np.float64))
    assert rel_eq(D, want) and not rel_eq(D, np.abs(y.astype(np.float64)))
    D = O.scal(n, alpha, synth.strided(x, abs(incx)), abs(incx), want_D=True)
    assert rel_eq(D, 3 * np.abs(x.astype(np.float64)))
    _, D = O.dot(n, xb, incx, yb, incy, want_D=True)
    assert rel_eq(D, np.abs(x.astype(np.float64)) @ np.abs(y.astype(np.float64)))
    r, D = O.asum(n, synth.strided(x, abs(incx)), abs(incx), want_D=True)
    assert rel_eq(D, np.abs(x).sum()) and r == np.abs(x).sum()
    r, D = O.nrm2(n, synth.strided(x, abs(incx)), abs(incx), want_D=True)
    assert rel_eq(D, np.sqrt((x.astype(np.float64) ** 2).sum()), 1e-6 if dt == np.float32 else 1e-12)
    _, D = O.dsdot(n, synth.strided(x.astype(np.float32), incx), incx, synth.strided(y.astype(np.float32), incy), incy, want_D=True)
    assert rel_eq(D, np.abs(x.astype(np.float64)) @ np.abs(y.astype(np.float64)))
    c, s = dt(3), dt(-2)
    D = O.rot(n, synth.strided(x, incx), incx, synth.strided(y, incy), incy, c, s, want_D=True)
    ax, ay = np.abs(x.astype(np.float64)), np.abs(y.astype(np.float64))
    assert rel_eq(D[0::2], 3 * ax + 2 * ay) and rel_eq(D[1::2], 3 * ay + 2 * ax)
    for param, H in (([-1, 2, -3, 4, 5], [[2, 4], [-3, 5]]), ([0, 9, -3, 4, 9], [[1, 4], [-3, 1]]), ([1, 2, 9, 9, 5], [[2, 1], [-1, 5]])):
        D = O.rotm(n, synth.strided(x, incx), incx, synth.strided(y, incy), incy, np.array(param, dt), want_D=True)
        H = np.abs(np.array(H, np.float64))
        assert rel_eq(D[0::2], H[0, 0] * ax + H[0, 1] * ay) and rel_eq(D[1::2], H[1, 0] * ax + H[1, 1] * ay)


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("layout", [O.ROW_MAJOR, O.COL_MAJOR])
def test_D_level2_dense_and_structured(dt, layout):
    n, m = 19, 23
    f64 = np.float64
    alpha, beta = dt(-2), dt(3)
    # gemv / gemv_batched
    A = small(41, 0, m * n, dt).reshape(m, n)
    buf = np.ascontiguousarray(A if layout == O.ROW_MAJOR else A.T).ravel()
    lda = n if layout == O.ROW_MAJOR else m
    for trans, op in ((O.NO_TRANS, A), (O.TRANS, A.T)):
        lenx, leny = op.shape[1], op.shape[0]
        x, y = small(41, 1, lenx, dt), small(41, 2, leny, dt)
        D = O.gemv(layout, trans, m, n, alpha, buf, lda, x, 1, beta, y.copy(), 1, want_D=True)
        want = 2 * (np.abs(op.astype(f64)) @ np.abs(x.astype(f64))) + 3 * np.abs(y.astype(f64))
        assert rel_eq(D, want)
        assert not rel_eq(D, 2 * (np.abs(op.astype(f64)) @ np.abs(x.astype(f64))))          # beta*y counts
        D0 = O.gemv(layout, trans, m, n, alpha, buf, lda, x, 1, dt(0), y.copy(), 1, want_D=True)
        assert rel_eq(D0, 2 * (np.abs(op.astype(f64)) @ np.abs(x.astype(f64))))             # and does not when beta == 0
        Db = O.gemv_batched(layout, trans, m, n, alpha, np.concatenate([buf, buf]), lda, m * n, np.concatenate([x, x]), 1, lenx, beta,
                            np.concatenate([y, y]), 1, leny, 2, want_D=True)
        assert rel_eq(Db, np.concatenate([want, want]))
    # trmv, trsv, symv: explicit triangle / explicitly symmetrised matrix
    S = small(42, 0, n * n, dt).reshape(n, n)
    x, y = small(42, 1, n, dt), small(42, 2, n, dt)
    for uplo in (O.UPPER, O.LOWER):
        for diag in (O.NON_UNIT, O.UNIT):
            Tm = explicit_tri(S.copy(), uplo, diag).astype(f64)
            tb, tlda, _ = tri_buffer(S, layout, uplo, 2, dt, unit=(diag == O.UNIT))
            for trans in (O.NO_TRANS, O.TRANS):
                opT = Tm if trans == O.NO_TRANS else Tm.T
                D = O.trmv(layout, uplo, trans, diag, n, tb.ravel(), tlda, x.copy(), 1, want_D=True)
                assert rel_eq(D, np.abs(opT) @ np.abs(x.astype(f64)))
                if diag == O.UNIT:       # the implied 1 on the diagonal counts as a term
                    assert not rel_eq(D, np.abs(opT - np.eye(n)) @ np.abs(x.astype(f64)))
        tri = np.triu(S) if uplo == O.UPPER else np.tril(S)
        full = (tri + tri.T - np.diag(np.diag(S))).astype(f64)
        sb, slda, _ = tri_buffer(S, layout, uplo, 1, dt)
        D = O.symv(layout, uplo, n, alpha, sb.ravel(), slda, x, 1, beta, y.copy(), 1, want_D=True)
        assert rel_eq(D, 2 * (np.abs(full) @ np.abs(x.astype(f64))) + 3 * np.abs(y.astype(f64)))
        assert not rel_eq(D, 2 * (np.abs(tri.astype(f64)) @ np.abs(x.astype(f64))) + 3 * np.abs(y.astype(f64)))   # the mirrored half counts
    # ger, syr, syr2: |A_old| + |alpha x_i y_j| (+ the second product), row-major D[i*n + j] of the logical matrix
    G = small(43, 0, m * n, dt).reshape(m, n)
    gx, gy = small(43, 1, m, dt), small(43, 2, n, dt)
    gbuf = np.ascontiguousarray(G if layout == O.ROW_MAJOR else G.T).ravel()
    D = O.ger(layout, m, n, alpha, gx, 1, gy, 1, gbuf.copy(), lda, want_D=True)
    assert rel_eq(D.reshape(m, n), np.abs(G.astype(f64)) + 2 * np.outer(np.abs(gx.astype(f64)), np.abs(gy.astype(f64))))
    for uplo in (O.UPPER, O.LOWER):
        inside = np.triu(np.ones((n, n), bool)) if uplo == O.UPPER else np.tril(np.ones((n, n), bool))
        sb, slda, _ = tri_buffer(S, layout, uplo, 1, dt)
        ax, ay = np.abs(x.astype(f64)), np.abs(y.astype(f64))
        D = O.syr(layout, uplo, n, alpha, x, 1, sb.copy().ravel(), slda, want_D=True).reshape(n, n)
        assert rel_eq(D[inside], (np.abs(S.astype(f64)) + 2 * np.outer(ax, ax))[inside]) and (D[~inside] == 0).all()
        D = O.syr2(layout, uplo, n, alpha, x, 1, y, 1, sb.copy().ravel(), slda, want_D=True).reshape(n, n)
        assert rel_eq(D[inside], (np.abs(S.astype(f64)) + 2 * np.outer(ax, ay) + 2 * np.outer(ay, ax))[inside]) and (D[~inside] == 0).all()


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("uplo", [O.UPPER, O.LOWER])
@pytest.mark.parametrize("trans", [O.NO_TRANS, O.TRANS])
@pytest.mark.parametrize("diag", [O.NON_UNIT, O.UNIT])
def test_D_trsv(dt, uplo, trans, diag):
    """D[o] = (|b_o| + sum_{k != o} |op(T)[o][k] z_k|) / |op(T)[o][o]| with z the solution: checked
    with the solution of an independent fp64 solver put into that expression by dense numpy."""
    import scipy.linalg
    n = 40
    A = synth.uniform(44, 0, n * n, dt).reshape(n, n) / dt(8)
    A[np.arange(n), np.arange(n)] = dt(1) + np.abs(synth.uniform(44, 5, n, dt))
    b = synth.uniform(44, 1, n, dt)
    Tm = explicit_tri(A.copy(), uplo, diag).astype(np.float64)
    opT = Tm if trans == O.NO_TRANS else Tm.T
    z = scipy.linalg.solve_triangular(opT, b.astype(np.float64), lower=((uplo == O.LOWER) == (trans == O.NO_TRANS)))
    off = np.abs(opT - np.diag(np.diag(opT)))
    want = (np.abs(b.astype(np.float64)) + off @ np.abs(z)) / np.abs(np.diag(opT))
    buf, lda, _ = tri_buffer(A, O.ROW_MAJOR, uplo, 1, dt, unit=(diag == O.UNIT))
    D = O.trsv(O.ROW_MAJOR, uplo, trans, diag, n, buf.ravel(), lda, b.copy(), 1, want_D=True)
    assert rel_eq(D, want, 1e-5 if dt == np.float32 else 1e-12)
    assert not rel_eq(D, np.abs(b.astype(np.float64)) / np.abs(np.diag(opT)), 1e-3)     # the off-diagonal terms count
