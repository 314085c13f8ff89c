"""Sizes at which a 32-bit element index or byte offset would wrap: level-1 vectors of 2^31 + 4099
elements and a 65536 x 65536 matrix with pitch 65600 (4.3e9 elements, 17 GB).  The oracle cannot
run such sizes whole in reasonable time, so outputs are checked on samples it computes one by one
(windows of the vectors around 0, 2^31 and the end; single rows and columns of the matrix,
among them the rows where the element offset crosses 2^32) and through exact integer identities:
inputs are small periodic integers, every partial sum is exactly representable, and the results
must agree bit for bit."""
import numpy as np
import pytest
import torch

import oracle as O
from parity import bits_equal, check_close, to_host

pytestmark = pytest.mark.gpu

N1 = (1 << 31) + 4099
CHUNK = 1 << 27


def pattern_dev(n, period, shift, device, mul=1, start=0):
    """(((start + i) * mul) % period) - shift as fp32, built in chunks on the device."""
    out = torch.empty(n, dtype=torch.float32, device=device)
    for s in range(0, n, CHUNK):
        e = min(n, s + CHUNK)
        idx = torch.arange(start + s, start + e, dtype=torch.int64, device=device)
        out[s:e] = ((idx * mul) % period - shift).to(torch.float32)
    return out


def pattern_host(i0, i1, period, shift, mul=1):
    idx = np.arange(i0, i1, dtype=np.int64)
    return ((idx * mul) % period - shift).astype(np.float32)


def windows(n):
    w = 1 << 18
    return [(0, w), ((1 << 31) - w, min((1 << 31) + w, n)), (n - w, n)]


@pytest.fixture(scope="module")
def big_ctx(blas):
    need = max(blas.mxb_workspace_bytes(blas.GEMV, 4, 65536, 65536), blas.mxb_workspace_bytes(blas.SYMV, 4, 0, 65536),
               blas.mxb_workspace_bytes(blas.TRMV, 4, 0, 65536), blas.mxb_workspace_bytes(blas.DOT, 4, 0, N1), 64 << 20)
    c = blas.Context(device="cuda:0", workspace_bytes=int(need))
    yield c
    c.close()


def test_level1_beyond_2_to_31_elements(blas, big_ctx):
    B, h = blas, big_ctx.h
    dev = torch.device("cuda:0")
    free, _ = torch.cuda.mem_get_info()
    if free < 34 << 30:
        pytest.skip("needs 34 GiB of free device memory")
    x = pattern_dev(N1, 7, 3, dev)
    y = pattern_dev(N1, 5, 2, dev)
    r = torch.zeros(1, dtype=torch.float32, device=dev)
    ri = torch.zeros(1, dtype=torch.int64, device=dev)

    # reductions: whole periods of 35 (7, 7) elements plus a remainder, each summed by the oracle
    def by_periods(period, fn):
        whole, rem = divmod(N1, period)
        return whole * fn(0, period) + fn(whole * period, whole * period + rem)

    dot_exact = by_periods(35, lambda a, b: int(O.dot(b - a, pattern_host(a, b, 7, 3), 1, pattern_host(a, b, 5, 2), 1)))
    asum_exact = by_periods(7, lambda a, b: int(O.asum(b - a, pattern_host(a, b, 7, 3), 1)))
    sq_exact = by_periods(7, lambda a, b: int(O.dot(b - a, pattern_host(a, b, 7, 3), 1, pattern_host(a, b, 7, 3), 1)))
    assert B.mxb_sdot(h, N1, x, 1, y, 1, r) == 0
    assert bits_equal(to_host(r)[0], np.float32(dot_exact)), (to_host(r)[0], dot_exact)
    assert B.mxb_sasum(h, N1, x, 1, r) == 0
    assert bits_equal(to_host(r)[0], np.float32(asum_exact)), (to_host(r)[0], asum_exact)
    assert B.mxb_snrm2(h, N1, x, 1, r) == 0
    assert abs(float(to_host(r)[0]) / np.sqrt(float(sq_exact)) - 1.0) <= 2.0 ** -23

    # the largest magnitude planted beyond index 2^31
    where = (1 << 31) + 17
    x[where] = 100.0
    assert B.mxb_isamax(h, N1, x, 1, ri) == 0
    assert int(to_host(ri)[0]) == where
    x[where] = float(pattern_host(where, where + 1, 7, 3)[0])

    # x as a matrix of one row of N1 columns: the products of a handful of very long rows.  Not
    # transposed it is the dot product above; transposed, a multiple of the row, checked on windows
    one = torch.zeros(1, dtype=torch.float32, device=dev)
    assert B.mxb_sgemv(h, B.ROW_MAJOR, B.NO_TRANS, 1, N1, 1.0, x, N1, y, 1, 0.0, one, 1) == 0
    assert bits_equal(to_host(one)[0], np.float32(dot_exact)), (to_host(one)[0], dot_exact)
    z = torch.empty(N1, dtype=torch.float32, device=dev)
    one[0] = -2.0
    assert B.mxb_sgemv(h, B.ROW_MAJOR, B.TRANS, 1, N1, 1.5, x, N1, one, 1, 0.0, z, 1) == 0
    for a, b in windows(N1):
        hz = np.full(b - a, np.nan, np.float32)
        O.gemv(O.ROW_MAJOR, O.TRANS, 1, b - a, np.float32(1.5), pattern_host(a, b, 7, 3), b - a, np.array([-2.0], np.float32), 1,
               np.float32(0.0), hz, 1)
        assert bits_equal(to_host(z[a:b]), hz), f"sgemv T, one row, window {a}..{b}"
    del z

    # element-wise routines, checked on windows against the oracle run on the same windows
    assert B.mxb_saxpy(h, N1, 2.0, x, 1, y, 1) == 0
    assert B.mxb_sscal(h, N1, -3.0, x, 1) == 0
    for a, b in windows(N1):
        hx, hy = pattern_host(a, b, 7, 3), pattern_host(a, b, 5, 2)
        O.axpy(b - a, 2.0, hx, 1, hy, 1)
        O.scal(b - a, -3.0, hx, 1)
        assert bits_equal(to_host(y[a:b]), hy), f"saxpy window {a}..{b}"
        assert bits_equal(to_host(x[a:b]), hx), f"sscal window {a}..{b}"
    # nothing but the n elements is written: the same sum again, from the closed form of the new values
    assert B.mxb_sasum(h, N1, x, 1, r) == 0
    assert bits_equal(to_host(r)[0], np.float32(3 * asum_exact))

    # copy, swap and rot over the whole length; increments whose products with the index pass 2^31
    def expect(a, b):                                      # x and y as they stand now, from the oracle's own steps
        hx, hy = pattern_host(a, b, 7, 3), pattern_host(a, b, 5, 2)
        O.axpy(b - a, 2.0, hx, 1, hy, 1)
        O.scal(b - a, -3.0, hx, 1)
        return hx, hy

    assert B.mxb_sswap(h, N1, x, 1, y, 1) == 0
    assert B.mxb_srot(h, N1, x, 1, y, 1, 0.0, 1.0) == 0   # c = 0, s = 1: x' = y, y' = -x, exact
    for a, b in windows(N1):
        hx, hy = expect(a, b)
        O.swap(b - a, hx, 1, hy, 1)
        O.rot(b - a, hx, 1, hy, 1, 0.0, 1.0)
        assert bits_equal(to_host(x[a:b]), hx) and bits_equal(to_host(y[a:b]), hy), f"sswap + srot window {a}..{b}"
    n2 = (1 << 30) + 2049                                  # every other element of x into every other element of y
    assert B.mxb_scopy(h, n2, x, 2, y, 2) == 0
    assert B.mxb_saxpy(h, n2, 1.0, x, 2, y, 2) == 0        # y = 2 x on the even places
    a, b = 2 * n2 - (1 << 18), 2 * n2 - 1
    hx, hy = expect(a, b)
    O.swap(b - a, hx, 1, hy, 1); O.rot(b - a, hx, 1, hy, 1, 0.0, 1.0)
    m = (b - a + 1) // 2
    O.copy(m, hx, 2, hy, 2); O.axpy(m, 1.0, hx, 2, hy, 2)
    assert bits_equal(to_host(y[a:b]), hy), "strided scopy + saxpy at the far end"
    assert B.mxb_sdot(h, n2, x, 2, y, 2, r) == 0           # = 2 sum x_even^2: an exact integer, rounded once
    xe = x[0:2 * n2 - 1:2].double()
    assert bits_equal(to_host(r)[0], np.float32(2.0 * float((xe * xe).sum().item())))


def test_level2_beyond_2_to_32_elements(blas, big_ctx):
    B, h = blas, big_ctx.h
    dev = torch.device("cuda:0")
    free, _ = torch.cuda.mem_get_info()
    if free < 40 << 30:
        pytest.skip("needs 40 GiB of free device memory")
    M = N = 65536
    lda = 65600
    total = (M - 1) * lda + N
    assert total > 1 << 32
    A = torch.empty(total, dtype=torch.float32, device=dev)
    rows_per = CHUNK // lda
    for r0 in range(0, M, rows_per):                      # A[i][j] = ((131 i + 7 j) % 17) - 8, padding included
        r1 = min(M, r0 + rows_per)
        e = min(total, r1 * lda)
        idx = torch.arange(r0 * lda, e, dtype=torch.int64, device=dev)
        A[r0 * lda:e] = (((idx // lda) * 131 + (idx % lda) * 7) % 17 - 8).to(torch.float32)
    xn = pattern_dev(N, 5, 2, dev)
    xm = pattern_dev(M, 7, 3, dev)
    hxn, hxm = to_host(xn), to_host(xm)
    y = torch.zeros(M, dtype=torch.float32, device=dev)
    cross = (1 << 32) // lda                               # the row in which the element offset passes 2^32
    picks = [0, 1, 31, 32767, cross - 1, cross, cross + 1, 65534, 65535]

    def row(i, lo=0, hi=N):
        return to_host(A[i * lda + lo:i * lda + hi])

    def col(j, lo=0, hi=M):
        return to_host(A.as_strided((hi - lo,), (lda,), lo * lda + j))

    def dot_row(v, w):                                     # one output of a matrix-vector product, by the oracle
        out = np.zeros(1, np.float32)
        O.gemv(O.ROW_MAJOR, O.NO_TRANS, 1, v.size, 1.0, np.ascontiguousarray(v), v.size, np.ascontiguousarray(w), 1, 0.0, out, 1)
        return out[0]

    # gemv, both orientations
    assert B.mxb_sgemv(h, B.ROW_MAJOR, B.NO_TRANS, M, N, 1.0, A, lda, xn, 1, 0.0, y, 1) == 0
    got = to_host(y)
    for i in picks:
        assert bits_equal(got[i], dot_row(row(i), hxn)), f"sgemv N row {i}"
    assert B.mxb_sgemv(h, B.ROW_MAJOR, B.TRANS, M, N, 1.0, A, lda, xm, 1, 0.0, y, 1) == 0
    got = to_host(y)
    for j in picks:
        assert bits_equal(got[j], dot_row(col(j), hxm)), f"sgemv T column {j}"

    # symv on the lower triangle: row i of S is A[i][:i+1] followed by A[i+1:][i]
    assert B.mxb_ssymv(h, B.ROW_MAJOR, B.LOWER, N, 1.0, A, lda, xn, 1, 0.0, y, 1) == 0
    got = to_host(y)
    for i in picks:
        srow = np.concatenate([row(i, 0, i + 1), col(i, i + 1, M)])
        assert bits_equal(got[i], dot_row(srow, hxn)), f"ssymv row {i}"

    # trmv, lower: not transposed (row i up to the diagonal) and transposed (column j from the diagonal down)
    t = xn.clone()
    assert B.mxb_strmv(h, B.ROW_MAJOR, B.LOWER, B.NO_TRANS, B.NON_UNIT, N, A, lda, t, 1) == 0
    got = to_host(t)
    for i in picks:
        assert bits_equal(got[i], dot_row(row(i, 0, i + 1), hxn[:i + 1])), f"strmv N row {i}"
    t = xm.clone()
    assert B.mxb_strmv(h, B.ROW_MAJOR, B.LOWER, B.TRANS, B.NON_UNIT, N, A, lda, t, 1) == 0
    got = to_host(t)
    for j in picks:
        assert bits_equal(got[j], dot_row(col(j, j, M), hxm[j:])), f"strmv T column {j}"

    # ger last (it changes A): sampled rows against the oracle's rank-1 update of that row
    before = {i: row(i) for i in picks}
    pad_before = to_host(A[cross * lda + N:(cross + 1) * lda]).copy()
    assert B.mxb_sger(h, B.ROW_MAJOR, M, N, 1.0, xm, 1, xn, 1, A, lda) == 0
    for i in picks:
        want = before[i].copy()
        O.ger(O.ROW_MAJOR, 1, N, 1.0, hxm[i:i + 1].copy(), 1, hxn, 1, want, N)
        assert bits_equal(row(i), want), f"sger row {i}"
    assert bits_equal(to_host(A[cross * lda + N:(cross + 1) * lda]), pad_before), "sger wrote into the padding"

    # syr2 on the lower triangle: sampled rows, and the element right of the diagonal stays untouched
    before = {i: row(i, 0, min(i + 2, N)) for i in picks}
    assert B.mxb_ssyr2(h, B.ROW_MAJOR, B.LOWER, N, 1.0, xn, 1, xm, 1, A, lda) == 0
    for i in picks:
        got_row, want = row(i, 0, min(i + 2, N)), before[i].copy()
        want[:i + 1] += hxn[i] * hxm[:i + 1] + hxm[i] * hxn[:i + 1]      # small integers: exact in any order
        assert bits_equal(got_row, want), f"ssyr2 row {i}"

    # strided batch over the same memory: 69950 problems of 256 x 240, the last ones beyond element 2^32
    m_, n_, sA = 256, 240, 256 * 240
    batch = total // sA
    assert (batch - 1) * sA > 1 << 32
    xb = pattern_dev(n_, 5, 2, dev)
    yb = torch.zeros(batch * m_, dtype=torch.float32, device=dev)
    assert B.mxb_sgemv_batched(h, B.ROW_MAJOR, B.NO_TRANS, m_, n_, 1.0, A, n_, sA, xb, 1, 0, 0.0, yb, 1, m_, batch) == 0
    got = to_host(yb).reshape(batch, m_)
    for pb in (0, (1 << 32) // sA, (1 << 32) // sA + 1, batch - 1):
        Ap = to_host(A[pb * sA:(pb + 1) * sA])
        want = np.zeros(m_, np.float32)
        O.gemv(O.ROW_MAJOR, O.NO_TRANS, m_, n_, 1.0, Ap, n_, to_host(xb), 1, 0.0, want, 1)
        assert bits_equal(got[pb], want), f"sgemv_batched problem {pb}"

    # the skinny kernels on the same memory as 107 million rows of 40
    rows40 = total // 40
    assert (rows40 - 1) * 40 > 1 << 32
    x40 = pattern_dev(40, 5, 2, dev)
    y40 = torch.zeros(rows40, dtype=torch.float32, device=dev)
    assert B.mxb_sgemv(h, B.ROW_MAJOR, B.NO_TRANS, rows40, 40, 1.0, A, 40, x40, 1, 0.0, y40, 1) == 0
    for i in (0, (1 << 32) // 40, (1 << 32) // 40 + 1, rows40 - 1):
        assert bits_equal(to_host(y40[i:i + 1])[0], dot_row(to_host(A[i * 40:(i + 1) * 40]), to_host(x40))), f"skinny sgemv N row {i}"

    # trsv at n = 65536 (256 workgroups of the chained kernel): unit diagonal, the integers scaled by
    # 2^-20 below it (row sums of magnitudes below 1/2: substitution cannot grow)
    A.mul_(2.0 ** -20)
    for trans in (B.NO_TRANS, B.TRANS):
        z = xn.clone()
        assert B.mxb_strsv(h, B.ROW_MAJOR, B.LOWER, trans, B.UNIT, N, A, lda, z, 1) == 0
        assert big_ctx.last_status() == B.OK
        hz = to_host(z)
        for i in picks:                                    # b_i = z_i + (strictly lower or upper part of op(T)) . z
            part = dot_row(row(i, 0, i), hz[:i]) if trans == B.NO_TRANS and i > 0 else (
                dot_row(col(i, i + 1, M), hz[i + 1:]) if trans == B.TRANS and i + 1 < M else np.float32(0))
            # a row's 63 substitution steps each round a value of size |z_i|: a few units in the last place
            bound = 32 * 2.0 ** -24 * (abs(float(hxn[i])) + abs(float(hz[i])) + abs(float(part)))
            assert abs(float(hz[i]) + float(part) - float(hxn[i])) <= bound, f"strsv trans={trans} row {i}"
        if trans == B.NO_TRANS:
            # and every unknown against the oracle's substitution on the same matrix (17 GB brought to the host once)
            print("strsv n=65536: oracle solve on the host", flush=True)
            hA = to_host(A)
            ref = hxn.copy()
            D = O.trsv(O.ROW_MAJOR, O.LOWER, O.NO_TRANS, O.UNIT, N, hA, lda, ref, 1, want_D=True)
            del hA
            check_close(hz, ref, D, N, "strsv lower N unit n=65536")


def test_trsv_with_more_workgroups_than_the_device_holds(blas, big_ctx):
    """n = 100000: 391 workgroups of the chained kernel where 256 are resident at a time, so the later
    ones take their tickets only when earlier ones have left; 1e10 elements (40 GB)."""
    B, h = blas, big_ctx.h
    dev = torch.device("cuda:0")
    free, _ = torch.cuda.mem_get_info()
    if free < 60 << 30:
        pytest.skip("needs 60 GiB of free device memory")
    n = 100000
    A = torch.empty(n * n, dtype=torch.float32, device=dev)
    rows_per = CHUNK // n
    for r0 in range(0, n, rows_per):                      # ((131 i + 7 j) % 17 - 8) * 2^-20: row sums of magnitudes below 0.8
        r1 = min(n, r0 + rows_per)
        idx = torch.arange(r0 * n, r1 * n, dtype=torch.int64, device=dev)
        A[r0 * n:r1 * n] = (((idx // n) * 131 + (idx % n) * 7) % 17 - 8).to(torch.float32) * 2.0 ** -20
    b = pattern_dev(n, 5, 2, dev)
    hb = to_host(b)
    picks = [0, 1, 255, 256, 65535, 65536, 65537, 99742, 99999]

    def dot_row(v, w):
        out = np.zeros(1, np.float32)
        O.gemv(O.ROW_MAJOR, O.NO_TRANS, 1, v.size, 1.0, np.ascontiguousarray(v), v.size, np.ascontiguousarray(w), 1, 0.0, out, 1)
        return out[0]

    for trans in (B.NO_TRANS, B.TRANS):
        z = b.clone()
        assert B.mxb_strsv(h, B.ROW_MAJOR, B.LOWER, trans, B.UNIT, n, A, n, z, 1) == 0
        assert big_ctx.last_status() == B.OK
        hz = to_host(z)
        assert np.isfinite(hz).all()
        for i in picks:
            if trans == B.NO_TRANS:
                t, w = (to_host(A[i * n:i * n + i]), hz[:i]) if i > 0 else (np.zeros(1, np.float32), np.zeros(1, np.float32))
            else:
                t, w = (to_host(A.as_strided((n - i - 1,), (n,), (i + 1) * n + i)), hz[i + 1:]) if i + 1 < n else (
                    np.zeros(1, np.float32), np.zeros(1, np.float32))
            part, spread = dot_row(t, w), dot_row(np.abs(t), np.abs(w))
            # the substitution steps round values of size |z_i|; the sum of the row is exact to a fraction of
            # an ulp of the sum of its magnitudes (a tile left out would show as 1e-5 or more)
            bound = 2.0 ** -24 * (32 * (abs(float(hb[i])) + abs(float(hz[i]))) + 2 * float(spread))
            assert abs(float(hz[i]) + float(part) - float(hb[i])) <= bound, f"strsv trans={trans} row {i}"


def test_launches_that_would_need_2_to_32_threads(blas, big_ctx):
    """A launch may not have 2^32 threads or more: shapes whose natural grids would (a rank-1 update of
    2^28 + 3 rows of 2 columns; the combine pass of a transposed product with 2^28 columns) must run with
    capped grids, not fail."""
    B, h = blas, big_ctx.h
    dev = torch.device("cuda:0")
    free, _ = torch.cuda.mem_get_info()
    if free < 30 << 30:
        pytest.skip("needs 30 GiB of free device memory")
    m = (1 << 28) + 3
    A = pattern_dev(2 * m, 9, 4, dev)
    xm = pattern_dev(m, 7, 3, dev)
    y2 = pattern_dev(2, 5, 2, dev, start=3)
    assert B.mxb_sger(h, B.ROW_MAJOR, m, 2, 2.0, xm, 1, y2, 1, A, 2) == 0
    hy = to_host(y2)
    for a, b in windows(m):
        want = pattern_host(2 * a, 2 * b, 9, 4)
        O.ger(O.ROW_MAJOR, b - a, 2, 2.0, pattern_host(a, b, 7, 3), 1, hy, 1, want, 2)
        assert bits_equal(to_host(A[2 * a:2 * b]), want), f"sger rows {a}..{b}"
    del A, xm

    rows, n = 16, 1 << 28
    M = torch.empty(rows * n, dtype=torch.float32, device=dev)
    for i in range(rows):
        M[i * n:(i + 1) * n] = pattern_dev(n, 11, 5, dev, start=3 * i)
    xr = pattern_dev(rows, 5, 2, dev)
    y = torch.zeros(n, dtype=torch.float32, device=dev)
    assert B.mxb_sgemv(h, B.ROW_MAJOR, B.TRANS, rows, n, 1.0, M, n, xr, 1, 0.0, y, 1) == 0
    hx = to_host(xr)
    for j in (0, 1, 63, 64, (1 << 27) - 1, 1 << 27, n - 65, n - 2, n - 1):
        col = np.array([pattern_host(3 * i + j, 3 * i + j + 1, 11, 5)[0] for i in range(rows)], np.float32)
        want = np.zeros(1, np.float32)
        O.gemv(O.ROW_MAJOR, O.NO_TRANS, 1, rows, 1.0, col, rows, hx, 1, 0.0, want, 1)
        assert bits_equal(to_host(y[j:j + 1])[0], want[0]), f"sgemv T column {j}"

