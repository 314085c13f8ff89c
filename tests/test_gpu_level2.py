"""GPU parity of gemv, trmv, symv and ger against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

import oracle as O
from paper_2411_07211_amd import synth
from parity import bits_equal, check_close, prefix_of, to_dev, to_host

pytestmark = pytest.mark.gpu

DT = [np.float32, np.float64]


def matrix_buffer(A, layout, pad, fill=np.nan):
    """Host buffer (1-D) holding the logical matrix A in the given layout with lda = minor + pad;
    padding holds NaN canaries."""
    m, n = A.shape
    if layout == O.ROW_MAJOR:
        lda = max(n + pad, 1); buf = np.full((m, lda), fill, A.dtype); buf[:, :n] = A
    else:
        lda = max(m + pad, 1); buf = np.full((n, lda), fill, A.dtype); buf[:, :m] = A.T
    return buf.ravel(), lda


# Elements by which every matrix of a case is displaced from the start of its allocation: a base
# address that is a multiple of the element size only.
A_OFFSET = [0]


def mat_dev(buf):
    off = A_OFFSET[0]
    if off == 0:
        return to_dev(buf)
    return to_dev(np.concatenate([np.full(off, np.nan, buf.dtype), buf]))[off:]


def logical(buf, layout, m, n, lda):
    v = buf.reshape(-1, lda)
    return v[:m, :n] if layout == O.ROW_MAJOR else v[:n, :m].T


GEMV_SHAPES = [(1, 1), (3, 5), (8, 8), (7, 2), (64, 64), (65, 257), (1000, 40), (40, 1000), (130, 1024),
               (257, 1030), (1024, 1024), (300, 4097), (2049, 513), (5000, 256), (17, 20000), (9000, 131)]


def gemv_case(blas, ctx, dt, layout, trans, m, n, alpha, beta, pad, incx, incy, seed=8, ints=False, xchunk=None):
    gen = (lambda t, k: synth.small_ints(seed, t, k, -2, 2, dt)) if ints else (lambda t, k: synth.uniform(seed, t, k, dt))
    A = gen(0, m * n).reshape(m, n)
    lenx, leny = (n, m) if trans == O.NO_TRANS else (m, n)
    x, y = gen(1, lenx), gen(2, leny)
    if beta == 0:
        y = np.full(leny, np.nan, dt)          # must be overwritten, never read
    Ab, lda = matrix_buffer(A, layout, pad)
    xb, yb = synth.strided(x, incx), synth.strided(y, incy)
    ref = yb.copy()
    D = O.gemv(layout, trans, m, n, dt(alpha), Ab, lda, xb, incx, dt(beta), ref, incy, want_D=True)
    dA, dx, dy = mat_dev(Ab), to_dev(xb), to_dev(yb)
    st = blas.routine(prefix_of(dt), "gemv")(ctx.h, layout, trans, m, n, float(alpha), dA, lda, dx, incx, float(beta), dy, incy)
    assert st == 0, f"status {st}"
    got = to_host(dy)
    what = f"gemv {prefix_of(dt)} layout={layout} trans={trans} {m}x{n} pad={pad} a={alpha} b={beta} inc=({incx},{incy})"
    g, r = synth.gather(got, leny, incy), synth.gather(ref, leny, incy)
    if ints:
        assert bits_equal(g, r), what
    else:
        check_close(g, r, D, lenx, what)
    gaps = np.ones(got.size, bool); gaps[::abs(incy)] = False
    assert np.isnan(got[gaps]).all(), what + ": wrote between the strides"


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("trans", [O.NO_TRANS, O.TRANS])
def test_gemv_shapes(blas, ctx, dt, trans):
    for (m, n) in GEMV_SHAPES:
        for pad in (0, 3, 4):
            gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, 1.5, 0.5, pad, 1, 1)
    # the transposed product of a small matrix has a kernel of its own: the same shapes through the
    # general kernels, and shapes around its limits (2048 rows, one vector of columns, ragged widths)
    try:
        ctx.set_option(blas.OPT_GEMVT_SMALL_MAX, 1)
        for (m, n) in GEMV_SHAPES:
            if m * n <= 1 << 22:
                gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, 1.5, 0.5, 3, 1, 1)
    finally:
        ctx.set_option(blas.OPT_GEMVT_SMALL_MAX, 0)
    # not transposed, a cache-sized matrix has a kernel of its own too (rows of at least half a
    # wavefront of vectors): the same shapes through the persistent row-dot grid, and shapes around
    # the new kernel's limits (narrowest rows, one and two rows per wavefront, ragged widths and
    # row counts, strided and reversed vectors, batches that end in the middle of a vector)
    try:
        ctx.set_option(blas.OPT_GEMVN_SMALL_MAX, 1)
        for (m, n) in GEMV_SHAPES:
            if m * n <= 1 << 22:
                gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, 1.5, 0.5, 3, 1, 1)
    finally:
        ctx.set_option(blas.OPT_GEMVN_SMALL_MAX, 0)
    fv = 16 // np.dtype(dt).itemsize
    for (m, n) in [(3, 32 * fv), (1, 32 * fv + 1), (2047, 64 * fv * 8), (2048, 64 * fv * 8 + 1), (2049, 64 * fv * 8 - 1), (4099, 64 * fv * 4 + 3),
                   (5, 64 * fv * 8 * 2 + 2 * fv + 1), (700, 1027), (256, 64 * fv * 32), (255, 64 * fv * 33 + 1), (300, 64 * fv * 16 - 1),
                   (512, 64 * fv * 20 + 5)]:
        for beta, incx, incy in ((0.0, 1, 1), (0.5, 2, 3), (-1.0, -1, -2)):
            gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, 1.5, beta, 1, incx, incy)
    # (transposed: every lane shape of the single-kernel path: up to 256, 512, 1536 and 2048 rows, and the first size beyond)
    for (m, n) in [(1024, 4), (1024, 5), (1025, 64), (1000, 33), (37, 2049), (1, 700), (1023, 3), (300, 4099), (512, 8191),
                   (256, 130), (257, 1031), (513, 29), (1536, 515), (1537, 64), (2048, 1037), (2049, 70)]:
        for beta in (0.0, 0.5):
            gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, 1.5, beta, 1, 2, 3)
    # few, very long rows: not transposed, the columns are split into chunks that run as a batch
    # (whole chunks, a ragged last one, negative increments, a pitch larger than the width)
    for (m, n, pad, incx, incy) in [(1, 32768, 0, 1, 1), (3, 40000, 5, 1, 1), (300, 65537, 0, -1, 2), (4096, 32768, 0, 1, 1),
                                    (4097, 32768, 0, 1, 1), (17, 100001, 3, 2, -1)]:
        for beta in (0.0, -0.5):
            gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, 1.5, beta, pad, incx, incy)
    gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, 64, 70000, 2, 1, 0, 1, 1, ints=True)
    # a handful of very long rows: not transposed, dot products that share x (every row count the
    # kernel is built for and the ones between, whole tiles only, ragged vectors and elements,
    # several tiles per block, strided and reversed x)
    for (m, n, pad, incx, incy) in [(1, 32768, 0, 1, 1), (1, 5000003, 0, 1, 1), (2, 65536, 3, 1, 1), (3, 40001, 5, -1, 1),
                                    (4, 32770, 0, 1, 2), (5, 100003, 1, 3, 1), (8, 1200007, 0, 1, 1), (9, 32768, 0, 1, -1),
                                    (13, 70001, 7, 1, 1), (16, 300000, 0, 1, 1), (16, 33333, 2, -2, 3), (17, 2097152, 0, 1, 1),
                                    (29, 2100001, 1, 1, 1), (32, 2097155, 0, 1, 1)]:
        for beta in (0.0, -0.5):
            gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, 1.5, beta, pad, incx, incy)
    gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, 7, 90001, 2, 1, 0, 1, 1, ints=True)
    # transposed, up to eight rows of at least 131072 columns, up to sixteen while the matrix is small:
    # a stream over the columns (every row count the kernel is built for and the ones between, whole
    # tiles and a ragged end, y strided and reversed, a pitch larger than the width, and the widths just
    # below and at the limit)
    if trans == O.TRANS:
        for (m, n, pad, incx, incy) in [(1, 13000003, 0, 1, 1), (2, 7000001, 5, -1, 1), (3, 9000002, 0, 2, 2), (4, 7000003, 1, 1, -1),
                                        (1, 131072, 0, 1, 1), (2, 131071, 0, 1, 1), (5, 131075, 3, 1, 1), (6, 200001, 0, -1, 2),
                                        (7, 1000003, 1, 1, 1), (8, 3000001, 0, 2, -1), (9, 131072, 0, 1, 1), (12, 400003, 5, 1, 3),
                                        (16, 131073, 0, -2, 1), (16, 524288, 0, 1, 1), (16, 524289, 0, 1, 1)]:
            for beta in (0.0, -0.5):
                gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, 1.5, beta, pad, incx, incy)
        gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, 4, 7000001, 2, 1, 0, 1, 1, ints=True)


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("layout", [O.ROW_MAJOR, O.COL_MAJOR])
@pytest.mark.parametrize("trans", [O.NO_TRANS, O.TRANS])
def test_gemv_scalars_increments_layouts(blas, ctx, dt, layout, trans):
    for (m, n) in [(5, 3), (129, 260), (1030, 515), (4100, 300)]:
        for alpha, beta in [(1, 0), (1, 1), (-1, 0.5), (2, -1), (0, 0), (0, 0.5)]:
            gemv_case(blas, ctx, dt, layout, trans, m, n, alpha, beta, 4, 1, 1)
        for incx, incy in [(2, 3), (-1, 1), (1, -2), (-3, -2)]:
            gemv_case(blas, ctx, dt, layout, trans, m, n, 1.5, 0.5, 1, incx, incy)


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("trans", [O.NO_TRANS, O.TRANS])
def test_gemv_integers_bit_exact(blas, ctx, dt, trans):
    for (m, n) in [(8, 8), (257, 1030), (2049, 513), (4096, 4096)]:
        gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, 3, -2, 0, 1, 1, ints=True)
        gemv_case(blas, ctx, dt, O.COL_MAJOR, trans, m, n, 2, 0.5, 4, 1, 1, ints=True)


@pytest.mark.parametrize("dt", DT)
def test_gemv_alpha_zero_reads_nothing_and_identity(blas, ctx, dt):
    m, n = 300, 200
    A = np.full(m * n, np.nan, dt); x = np.full(n, np.nan, dt); y = synth.uniform(9, 2, m, dt)
    dA, dx, dy = to_dev(A), to_dev(x), to_dev(y)
    f = blas.routine(prefix_of(dt), "gemv")
    assert f(ctx.h, O.ROW_MAJOR, O.NO_TRANS, m, n, 0.0, dA, n, dx, 1, 0.5, dy, 1) == 0
    assert bits_equal(to_host(dy), dt(0.5) * y)
    assert f(ctx.h, O.ROW_MAJOR, O.NO_TRANS, m, n, 0.0, dA, n, dx, 1, 1.0, dy, 1) == 0     # quick return
    assert bits_equal(to_host(dy), dt(0.5) * y)
    k = 1000
    I = np.eye(k, dtype=dt); xv = synth.uniform(9, 1, k, dt)
    for trans in (O.NO_TRANS, O.TRANS):
        dy = to_dev(np.full(k, np.nan, dt))
        assert f(ctx.h, O.ROW_MAJOR, trans, k, k, 1.0, to_dev(I.ravel()), k, to_dev(xv), 1, 0.0, dy, 1) == 0
        assert bits_equal(to_host(dy), xv)              # identity returns x, bit for bit


@pytest.mark.parametrize("dt", DT)
def test_gemv_deterministic_and_geometry_invariant(blas, ctx, dt):
    m, n = 3000, 2500
    A = synth.uniform(10, 0, m * n, dt); Ad = to_dev(A)
    f = blas.routine(prefix_of(dt), "gemv")
    try:
        for trans, lenx, leny in ((O.NO_TRANS, n, m), (O.TRANS, m, n)):
            x, y = synth.uniform(10, 1, lenx, dt), synth.uniform(10, 2, leny, dt)
            ref = y.copy(); D = O.gemv(O.ROW_MAJOR, trans, m, n, dt(1.5), A, n, x, 1, dt(0.5), ref, 1, want_D=True)
            outs = []
            for opts in ({}, {}, {blas.OPT_ROWDOT_XCHUNK: 256, blas.OPT_COLACC_TARGET_BLOCKS: 64},
                         {blas.OPT_ROWDOT_XCHUNK: 1024, blas.OPT_ROWDOT_BLOCKS_PER_CU: 1, blas.OPT_COLACC_TARGET_BLOCKS: 4096,
                          blas.OPT_COLACC_MIN_ROWS: 8}):
                for o in range(14):
                    ctx.set_option(o, 0)
                for o, v in opts.items():
                    ctx.set_option(o, v)
                dy = to_dev(y)
                assert f(ctx.h, O.ROW_MAJOR, trans, m, n, 1.5, Ad, n, to_dev(x), 1, 0.5, dy, 1) == 0
                outs.append(to_host(dy))
                check_close(outs[-1], ref, D, lenx, f"gemv trans={trans} opts={opts}")
            assert outs[0].tobytes() == outs[1].tobytes(), "same launch geometry must give the same bits"
    finally:
        for o in range(14):
            ctx.set_option(o, 0)


# ----------------------------------------------------------------------------- gemv, strided batch
def gemv_batched_case(blas, ctx, dt, layout, trans, m, n, batch, alpha, beta, pad, incx, incy, gaps=(0, 0, 0), share=(False, False),
                      ints=False, seed=16):
    """`batch` problems with canaries (NaN) in the padding and between the problems; share = (A, x)
    shared among the problems through a stride of 0."""
    gen = (lambda t, k: synth.small_ints(seed, t, k, -2, 2, dt)) if ints else (lambda t, k: synth.uniform(seed, t, k, dt))
    lenx, leny = (n, m) if trans == O.NO_TRANS else (m, n)
    major = m if layout == O.ROW_MAJOR else n
    minor = n if layout == O.ROW_MAJOR else m
    lda = max(minor + pad, 1)
    spanx, spany = 1 + (lenx - 1) * abs(incx), 1 + (leny - 1) * abs(incy)
    sA = 0 if share[0] else major * lda + gaps[0]
    sx = 0 if share[1] else spanx + gaps[1]
    sy = spany + gaps[2]
    Ab = np.full(major * lda + (batch - 1) * sA, np.nan, dt)
    xb = np.full(spanx + (batch - 1) * sx, np.nan, dt)
    yb = np.full(spany + (batch - 1) * sy, np.nan, dt)
    ymask = np.zeros(yb.size, bool)
    for b in range(batch):
        if b == 0 or not share[0]:
            A = gen(3 * b, m * n).reshape(m, n)
            buf, _ = matrix_buffer(A, layout, pad)
            Ab[b * sA:b * sA + buf.size] = buf
        if b == 0 or not share[1]:
            xb[b * sx:b * sx + spanx] = synth.strided(gen(3 * b + 1, lenx), incx)
        y = np.full(leny, np.nan, dt) if beta == 0 else gen(3 * b + 2, leny)
        yb[b * sy:b * sy + spany] = synth.strided(y, incy)
        ymask[b * sy + np.arange(leny) * abs(incy)] = True
    ref = yb.copy()
    D = O.gemv_batched(layout, trans, m, n, dt(alpha), Ab, lda, sA, xb, incx, sx, dt(beta), ref, incy, sy, batch, want_D=True)
    dA, dx, dy = mat_dev(Ab), to_dev(xb), to_dev(yb)
    st = blas.routine(prefix_of(dt), "gemv_batched")(ctx.h, layout, trans, m, n, float(alpha), dA, lda, sA, dx, incx, sx,
                                                     float(beta), dy, incy, sy, batch)
    assert st == 0, f"status {st}"
    got = to_host(dy)
    what = (f"gemv_batched {prefix_of(dt)} layout={layout} trans={trans} {m}x{n} batch={batch} pad={pad} a={alpha} b={beta} "
            f"inc=({incx},{incy}) strides=({sA},{sx},{sy})")
    if ints:
        assert bits_equal(got[ymask], ref[ymask]), what
    else:
        g = np.concatenate([synth.gather(got[b * sy:], leny, incy) for b in range(batch)])
        r = np.concatenate([synth.gather(ref[b * sy:], leny, incy) for b in range(batch)])
        check_close(g, r, D, lenx, what)
    assert np.isnan(got[~ymask]).all(), what + ": wrote outside the result vectors"


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("trans", [O.NO_TRANS, O.TRANS])
def test_gemv_batched(blas, ctx, dt, trans):
    for (m, n, batch) in [(1, 1, 1), (4, 4, 5), (33, 17, 7), (64, 64, 100), (130, 257, 9), (1000, 40, 6), (40, 1000, 6),
                          (513, 1030, 3), (2049, 300, 2), (300, 4100, 2)]:
        gemv_batched_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, batch, 1.5, 0.5, 0, 1, 1)
        gemv_batched_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, batch, -1, 0, 3, 1, 1, gaps=(5, 2, 3))
    for layout in (O.ROW_MAJOR, O.COL_MAJOR):
        gemv_batched_case(blas, ctx, dt, layout, trans, 129, 260, 5, 1.5, 0.5, 1, 2, -3, gaps=(1, 1, 1))
        gemv_batched_case(blas, ctx, dt, layout, trans, 129, 260, 5, 2, -1, 0, -1, 1, share=(True, False))
        gemv_batched_case(blas, ctx, dt, layout, trans, 129, 260, 5, 2, 1, 0, 1, 1, share=(False, True))
        gemv_batched_case(blas, ctx, dt, layout, trans, 96, 200, 11, 3, -2, 2, 1, 1, ints=True)
        gemv_batched_case(blas, ctx, dt, layout, trans, 96, 200, 4, 0, 0.5, 0, 1, 2)          # alpha == 0: A, x never read
        gemv_batched_case(blas, ctx, dt, layout, trans, 96, 200, 4, 0, 0, 0, 1, 1)
    # rows narrower than one vector, in small and large batches; transposed, short rows go to the
    # whole-problem-per-wavefront kernel only when the batch fills the device or the problems are short
    for (m, n, batch) in [(8, 1, 5), (100, 1, 3000), (7, 2, 2500), (300, 3, 40), (33, 3, 2100), (700, 40, 8), (700, 40, 2048),
                          (64, 8, 512), (64, 8, 511), (32, 40, 20), (33, 40, 20), (2048, 8, 16)]:
        if dt == np.float64 and n in (2, 3): continue          # two doubles are a vector
        gemv_batched_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, batch, 1.5, 0.5, 0, 1, 1)
        gemv_batched_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, batch, -1, 0, 1, 2, -1, gaps=(3, 1, 2))
    # problems of a few rows each (up to 32 rows take one wavefront per row over the rows of all problems)
    for (m, n, batch) in [(1, 65, 7), (1, 100, 3000), (2, 257, 33), (5, 1030, 9), (32, 130, 5), (33, 130, 5), (3, 5001, 4), (1, 70000, 3)]:
        gemv_batched_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, batch, 1.5, 0.5, 0, 1, 1)
        gemv_batched_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, batch, -1, 0, 3, -1, 2, gaps=(5, 2, 3))
    gemv_batched_case(blas, ctx, dt, O.ROW_MAJOR, trans, 4, 300, 11, 3, -2, 1, 1, 1, ints=True, share=(True, False))
    # transposed, problems of up to 16 rows and 64 columns: a lane per vector of columns (every row count
    # the kernel is built for and the ones between, whole and ragged widths, the first size beyond)
    for (m, n, batch) in [(1, 8, 1000), (2, 4, 3), (3, 3, 2000), (3, 7, 50), (5, 40, 300), (8, 64, 100), (9, 1, 77), (16, 16, 500),
                          (16, 63, 9), (17, 16, 500), (1, 1, 3000)]:
        if dt == np.float64 and n == 3: continue
        gemv_batched_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, batch, 1.5, 0.5, 0, 1, 1)
        gemv_batched_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, batch, -1, 0, 2, -1, 2, gaps=(3, 1, 2))
    gemv_batched_case(blas, ctx, dt, O.ROW_MAJOR, trans, 6, 12, 40, 3, -2, 0, 1, 1, ints=True, share=(False, True))
    # more problems than one grid dimension holds
    gemv_batched_case(blas, ctx, dt, O.ROW_MAJOR, trans, 3, 5, 70000, 1.5, 0.5, 0, 1, 1, share=(True, False), ints=True)
    # one large problem goes the same way as gemv
    gemv_batched_case(blas, ctx, dt, O.ROW_MAJOR, trans, 3000, 2500, 1, 1.5, 0.5, 0, 1, 1)


# ----------------------------------------------------------------------------- any base address, pitch and width
@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("off", [1, 2, 3])
def test_matrices_at_any_element_offset_pitch_and_width(blas, ctx, dt, off):
    """Rows that start at arbitrary elements (odd pitch, displaced base) and widths that are not a
    whole number of 16-byte vectors take the same kernels as aligned matrices."""
    A_OFFSET[0] = off
    try:
        for (m, n) in [(130, 1027), (1030, 515), (300, 4101), (2049, 6), (9000, 131), (700, 2050)]:
            for trans in (O.NO_TRANS, O.TRANS):
                gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, 1.5, 0.5, off, 1, 1)
            gemv_case(blas, ctx, dt, O.COL_MAJOR, O.NO_TRANS, m, n, 1.5, 0.0, 0, 1, 1)
            ger_case(blas, ctx, dt, O.ROW_MAJOR, m, n, 0.75, off, 1, 1)
        gemv_case(blas, ctx, dt, O.ROW_MAJOR, O.TRANS, 2049, 1030 + off, 3, -2, 0, 1, 1, ints=True)
        ger_case(blas, ctx, dt, O.ROW_MAJOR, 300, 1030 + off, 2, 0, 1, 1, ints=True)
        for n in (5, 259, 1031, 2310, 4101):
            for uplo in (O.UPPER, O.LOWER):
                symv_case(blas, ctx, dt, O.ROW_MAJOR, uplo, n, 1.5, 0.5, off - 1, 1, 1)
                syr_case(blas, ctx, dt, O.ROW_MAJOR, uplo, n, 0.75, off - 1, 1, 1, False)
                syr_case(blas, ctx, dt, O.ROW_MAJOR, uplo, n, 0.75, off, 1, 1, True)
                for trans in (O.NO_TRANS, O.TRANS):
                    for diag in (O.NON_UNIT, O.UNIT):
                        trmv_case(blas, ctx, dt, O.ROW_MAJOR, uplo, trans, diag, n, off - 1, 1)
                    trsv_case(blas, ctx, dt, O.ROW_MAJOR, uplo, trans, O.NON_UNIT, n, off, 1)
        for uplo in (O.UPPER, O.LOWER):
            symv_case(blas, ctx, dt, O.ROW_MAJOR, uplo, 1535 + off, 3, -2, 0, 1, 1, ints=True)
            trmv_case(blas, ctx, dt, O.ROW_MAJOR, uplo, O.TRANS, O.NON_UNIT, 1535 + off, 0, 1, ints=True)
        # wide tiles of the triangle sweep with a ragged last vector
        ctx.set_option(blas.OPT_SYMV_TILE_VECTORS, 2)
        for uplo in (O.UPPER, O.LOWER):
            symv_case(blas, ctx, dt, O.ROW_MAJOR, uplo, 8190 + off, 1.5, 0.5, 0, 1, 1)
            trmv_case(blas, ctx, dt, O.ROW_MAJOR, uplo, O.TRANS, O.UNIT, 8190 + off, 0, 1)
    finally:
        A_OFFSET[0] = 0
        ctx.set_option(blas.OPT_SYMV_TILE_VECTORS, 0)


# ----------------------------------------------------------------------------- trmv
def trmv_case(blas, ctx, dt, layout, uplo, trans, diag, n, pad, incx, ints=False, seed=11):
    gen = (lambda t, k: synth.small_ints(seed, t, k, -2, 2, dt)) if ints else (lambda t, k: synth.uniform(seed, t, k, dt))
    A = gen(0, n * n).reshape(n, n).copy()
    outside = np.tril(np.ones((n, n), bool), -1) if uplo == O.UPPER else np.triu(np.ones((n, n), bool), 1)
    A[outside] = np.nan                                   # the opposite triangle must never be used
    if diag == O.UNIT:
        np.fill_diagonal(A, np.nan)                       # nor the diagonal
    x = gen(1, n)
    Ab, lda = matrix_buffer(A, layout, pad)
    xb = synth.strided(x, incx)
    ref = xb.copy()
    D = O.trmv(layout, uplo, trans, diag, n, Ab, lda, ref, incx, want_D=True)
    dx = to_dev(xb)
    st = blas.routine(prefix_of(dt), "trmv")(ctx.h, layout, uplo, trans, diag, n, mat_dev(Ab), lda, dx, incx)
    assert st == 0, f"status {st}"
    got = to_host(dx)
    what = f"trmv {prefix_of(dt)} layout={layout} uplo={uplo} trans={trans} diag={diag} n={n} pad={pad} incx={incx}"
    g, r = synth.gather(got, n, incx), synth.gather(ref, n, incx)
    if ints:
        assert bits_equal(g, r), what
    else:
        check_close(g, r, D, n, what)
    gaps = np.ones(got.size, bool); gaps[::abs(incx)] = False
    assert np.isnan(got[gaps]).all(), what


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("layout", [O.ROW_MAJOR, O.COL_MAJOR])
@pytest.mark.parametrize("uplo", [O.UPPER, O.LOWER])
@pytest.mark.parametrize("trans", [O.NO_TRANS, O.TRANS])
@pytest.mark.parametrize("diag", [O.NON_UNIT, O.UNIT])
def test_trmv(blas, ctx, dt, layout, uplo, trans, diag):
    for n in (1, 2, 3, 5, 17, 64, 65, 130, 257, 1000, 2310):
        trmv_case(blas, ctx, dt, layout, uplo, trans, diag, n, 0 if n % 2 else 4, 1)
    trmv_case(blas, ctx, dt, layout, uplo, trans, diag, 515, 1, 2)
    trmv_case(blas, ctx, dt, layout, uplo, trans, diag, 515, 0, -1)
    trmv_case(blas, ctx, dt, layout, uplo, trans, diag, 1536, 0, 1, ints=True)
    if trans == O.NO_TRANS:
        # not transposed, a cache-sized triangle takes the wavefront-per-row kernel: sizes around its
        # limits (narrowest rows, 2, 4 and 8 loads per row, one and two rows per wavefront), and the
        # same sizes through the persistent row-dot grid
        for small_max in (0, 1):
            try:
                ctx.set_option(blas.OPT_GEMVN_SMALL_MAX, small_max)
                fv = 16 // np.dtype(dt).itemsize
                for n in (32 * fv - 1, 32 * fv, 128 * fv, 128 * fv + 1, 256 * fv + 3, 513 * fv, 2047, 2048, 2049, 3001):
                    trmv_case(blas, ctx, dt, layout, uplo, trans, diag, n, 0 if n % 2 else 4, 1)
                trmv_case(blas, ctx, dt, layout, uplo, trans, diag, 700, 1, -2)
                trmv_case(blas, ctx, dt, layout, uplo, trans, diag, 2100, 0, 1, ints=True)
            finally:
                ctx.set_option(blas.OPT_GEMVN_SMALL_MAX, 0)
    # sizes at which the triangle sweep takes its medium and its long batches
    trmv_case(blas, ctx, dt, layout, uplo, trans, diag, 7001, 0, 1)
    if dt == np.float32 and layout == O.ROW_MAJOR and diag == O.NON_UNIT:
        trmv_case(blas, ctx, dt, layout, uplo, trans, diag, 12500, 0, 1)
    # the triangle sweep behind the transposed product with wider tiles and other grid sizes
    try:
        for cv, n in ((2, 4100), (4, 6000)):
            ctx.set_option(blas.OPT_SYMV_TILE_VECTORS, cv)
            trmv_case(blas, ctx, dt, layout, uplo, trans, diag, n, 0, 1)
        ctx.set_option(blas.OPT_SYMV_TILE_VECTORS, 0)
        for tb in (1, 7, 1000):
            ctx.set_option(blas.OPT_SYMV_TARGET_BLOCKS, tb)
            trmv_case(blas, ctx, dt, layout, uplo, trans, diag, 2310, 2, 1)
    finally:
        ctx.set_option(blas.OPT_SYMV_TARGET_BLOCKS, 0)
        ctx.set_option(blas.OPT_SYMV_TILE_VECTORS, 0)


# ----------------------------------------------------------------------------- symv
def symv_case(blas, ctx, dt, layout, uplo, n, alpha, beta, pad, incx, incy, ints=False, seed=12):
    gen = (lambda t, k: synth.small_ints(seed, t, k, -2, 2, dt)) if ints else (lambda t, k: synth.uniform(seed, t, k, dt))
    A = gen(0, n * n).reshape(n, n).copy()
    outside = np.tril(np.ones((n, n), bool), -1) if uplo == O.UPPER else np.triu(np.ones((n, n), bool), 1)
    A[outside] = np.nan
    x, y = gen(1, n), gen(2, n)
    if beta == 0:
        y = np.full(n, np.nan, dt)
    Ab, lda = matrix_buffer(A, layout, pad)
    xb, yb = synth.strided(x, incx), synth.strided(y, incy)
    ref = yb.copy()
    D = O.symv(layout, uplo, n, dt(alpha), Ab, lda, xb, incx, dt(beta), ref, incy, want_D=True)
    dy = to_dev(yb)
    st = blas.routine(prefix_of(dt), "symv")(ctx.h, layout, uplo, n, float(alpha), mat_dev(Ab), lda, to_dev(xb), incx, float(beta), dy, incy)
    assert st == 0, f"status {st}"
    got = to_host(dy)
    what = f"symv {prefix_of(dt)} layout={layout} uplo={uplo} n={n} pad={pad} a={alpha} b={beta} inc=({incx},{incy})"
    g, r = synth.gather(got, n, incy), synth.gather(ref, n, incy)
    if ints:
        assert bits_equal(g, r), what
    else:
        check_close(g, r, D, n, what)
    gaps = np.ones(got.size, bool); gaps[::abs(incy)] = False
    assert np.isnan(got[gaps]).all(), what


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("layout", [O.ROW_MAJOR, O.COL_MAJOR])
@pytest.mark.parametrize("uplo", [O.UPPER, O.LOWER])
def test_symv(blas, ctx, dt, layout, uplo):
    # small n twice: the single-kernel path, then (switched off) the triangle sweep
    for small_max in (0, 1):
        ctx.set_option(blas.OPT_SYMV_SMALL_MAX, small_max)
        try:
            for n in (1, 2, 3, 4, 5, 15, 16, 17, 31, 32, 33, 64, 65, 130, 257, 1000, 1024, 1600, 1601, 2047, 2048, 2310, 2400, 2401):
                symv_case(blas, ctx, dt, layout, uplo, n, 1.5, 0.5, 0 if n % 2 else 4, 1, 1)
            symv_case(blas, ctx, dt, layout, uplo, 515, 1.5, 0.5, 1, 2, -3)
            symv_case(blas, ctx, dt, layout, uplo, 1536, 3, -2, 0, 1, 1, ints=True)
            symv_case(blas, ctx, dt, layout, uplo, 700, 1, 0, 0, 1, 1)
        finally:
            ctx.set_option(blas.OPT_SYMV_SMALL_MAX, 0)
    for alpha, beta in [(1, 0), (1, 1), (0, 0.5), (0, 0), (-2, -1)]:
        symv_case(blas, ctx, dt, layout, uplo, 700, alpha, beta, 0, 1, 1)
    symv_case(blas, ctx, dt, layout, uplo, 515, 1.5, 0.5, 1, 2, -3)
    symv_case(blas, ctx, dt, layout, uplo, 1536, 3, -2, 0, 1, 1, ints=True)
    # sizes at which the triangle sweep takes its medium and its long batches
    symv_case(blas, ctx, dt, layout, uplo, 7001, 1.5, 0.5, 0, 1, 1)
    if dt == np.float32 and layout == O.ROW_MAJOR:
        symv_case(blas, ctx, dt, layout, uplo, 12500, 1.5, 0.5, 0, 1, 1)
    try:
        for tb in (1, 7, 64, 1000):
            ctx.set_option(blas.OPT_SYMV_TARGET_BLOCKS, tb)
            symv_case(blas, ctx, dt, layout, uplo, 2310, 1.5, 0.5, 2, 1, 1)
            symv_case(blas, ctx, dt, layout, uplo, 5000, 1.5, 0.5, 0, 1, 1)
        # wider tiles (2 and 4 vectors per lane) over several row bands, ragged last tile included
        ctx.set_option(blas.OPT_SYMV_TARGET_BLOCKS, 0)
        for cv, n in ((2, 4100), (4, 4096), (4, 9000)):
            ctx.set_option(blas.OPT_SYMV_TILE_VECTORS, cv)
            symv_case(blas, ctx, dt, layout, uplo, n, 1.5, 0.5, 0, 1, 1)
    finally:
        ctx.set_option(blas.OPT_SYMV_TARGET_BLOCKS, 0)
        ctx.set_option(blas.OPT_SYMV_TILE_VECTORS, 0)


# ----------------------------------------------------------------------------- ger
def ger_case(blas, ctx, dt, layout, m, n, alpha, pad, incx, incy, ints=False, seed=13):
    gen = (lambda t, k: synth.small_ints(seed, t, k, -3, 3, dt)) if ints else (lambda t, k: synth.uniform(seed, t, k, dt))
    A = gen(0, m * n).reshape(m, n)
    x, y = gen(1, m), gen(2, n)
    Ab, lda = matrix_buffer(A, layout, pad)
    xb, yb = synth.strided(x, incx), synth.strided(y, incy)
    ref = Ab.copy()
    D = O.ger(layout, m, n, dt(alpha), xb, incx, yb, incy, ref, lda, want_D=True)
    dA = mat_dev(Ab)
    st = blas.routine(prefix_of(dt), "ger")(ctx.h, layout, m, n, float(alpha), to_dev(xb), incx, to_dev(yb), incy, dA, lda)
    assert st == 0, f"status {st}"
    got = to_host(dA)
    what = f"ger {prefix_of(dt)} layout={layout} {m}x{n} pad={pad} a={alpha} inc=({incx},{incy})"
    g, r = logical(got, layout, m, n, lda), logical(ref, layout, m, n, lda)
    if ints:
        assert bits_equal(g, r), what
    else:
        check_close(np.ascontiguousarray(g).ravel(), np.ascontiguousarray(r).ravel(), D, 1, what)
    # padding untouched (still NaN), nothing else changed
    mask = np.ones(got.size, bool).reshape(-1, lda)
    if layout == O.ROW_MAJOR: mask[:m, :n] = False
    else: mask[:n, :m] = False
    assert np.isnan(got.reshape(-1, lda)[mask]).all(), what + ": padding written"


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("layout", [O.ROW_MAJOR, O.COL_MAJOR])
def test_ger(blas, ctx, dt, layout):
    for (m, n) in [(1, 1), (3, 5), (64, 64), (65, 257), (1000, 40), (40, 1000), (257, 1030), (1024, 1024), (300, 4097)]:
        for pad in (0, 3, 4):
            ger_case(blas, ctx, dt, layout, m, n, 0.3, pad, 1, 1)
    ger_case(blas, ctx, dt, layout, 515, 260, -1.5, 4, 2, -3)
    ger_case(blas, ctx, dt, layout, 515, 260, -1.5, 1, -1, 2)
    ger_case(blas, ctx, dt, layout, 1030, 2052, 3, 0, 1, 1, ints=True)
    # alpha = 0: A untouched even if x, y hold NaN
    A = synth.uniform(13, 0, 100 * 100, dt); dA = to_dev(A); nan = to_dev(np.full(100, np.nan, dt))
    assert blas.routine(prefix_of(dt), "ger")(ctx.h, layout, 100, 100, 0.0, nan, 1, nan, 1, dA, 100) == 0
    assert bits_equal(to_host(dA), A)


@pytest.mark.parametrize("dt", DT)
def test_ger_very_long_rows(blas, ctx, dt):
    """Rows of a megabyte and more are updated one by one, in the tiles of the level-1 kernels: whole
    tiles, a ragged rest of vectors and of elements, a pitch beyond the width, a displaced base, a
    negative increment of x; with a strided y the general kernel takes over."""
    w = (1 << 20) // np.dtype(dt).itemsize
    for (m, n, pad, incx) in [(3, w, 0, 1), (2, w + 8192 * 3 + 5, 7, -1), (5, 2 * w + 16384 + 1, 0, 2), (1, 3 * w - 3, 1, 1)]:
        ger_case(blas, ctx, dt, O.ROW_MAJOR, m, n, 0.3, pad, incx, 1)
    ger_case(blas, ctx, dt, O.COL_MAJOR, w + 100, 3, -1.5, 0, 1, 1)
    ger_case(blas, ctx, dt, O.ROW_MAJOR, 4, w + 37, 3, 0, 1, 1, ints=True)
    ger_case(blas, ctx, dt, O.ROW_MAJOR, 2, w + 64, 0.3, 0, 1, 3)
    A_OFFSET[0] = 1
    try:
        ger_case(blas, ctx, dt, O.ROW_MAJOR, 3, w + 1029, 0.3, 2, 1, 1)
    finally:
        A_OFFSET[0] = 0


# ----------------------------------------------------------------------------- syr, syr2
def syr_case(blas, ctx, dt, layout, uplo, n, alpha, pad, incx, incy, two, ints=False, seed=14):
    gen = (lambda t, k: synth.small_ints(seed, t, k, -3, 3, dt)) if ints else (lambda t, k: synth.uniform(seed, t, k, dt))
    A = gen(0, n * n).reshape(n, n).copy()
    outside = np.tril(np.ones((n, n), bool), -1) if uplo == O.UPPER else np.triu(np.ones((n, n), bool), 1)
    A[outside] = np.nan                                   # never read, never written
    x, y = gen(1, n), gen(2, n)
    Ab, lda = matrix_buffer(A, layout, pad)
    xb, yb = synth.strided(x, incx), synth.strided(y, incy)
    ref = Ab.copy()
    if two:
        D = O.syr2(layout, uplo, n, dt(alpha), xb, incx, yb, incy, ref, lda, want_D=True)
    else:
        D = O.syr(layout, uplo, n, dt(alpha), xb, incx, ref, lda, want_D=True)
    dA = mat_dev(Ab)
    f = blas.routine(prefix_of(dt), "syr2" if two else "syr")
    if two:
        st = f(ctx.h, layout, uplo, n, float(alpha), to_dev(xb), incx, to_dev(yb), incy, dA, lda)
    else:
        st = f(ctx.h, layout, uplo, n, float(alpha), to_dev(xb), incx, dA, lda)
    assert st == 0, f"status {st}"
    got = to_host(dA)
    what = f"{'syr2' if two else 'syr'} {prefix_of(dt)} layout={layout} uplo={uplo} n={n} pad={pad} a={alpha} inc=({incx},{incy})"
    g, r = logical(got, layout, n, n, lda), logical(ref, layout, n, n, lda)
    keep = ~outside
    if ints:
        assert bits_equal(g[keep], r[keep]), what
    else:
        check_close(g[keep], r[keep], D.reshape(n, n)[keep], 1, what)
    # opposite triangle and padding untouched (still NaN)
    assert np.isnan(g[outside]).all(), what + ": wrote outside the triangle"
    mask = np.ones(got.size, bool).reshape(-1, lda); mask[:n, :n] = False
    assert np.isnan(got.reshape(-1, lda)[mask]).all(), what + ": padding written"


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("layout", [O.ROW_MAJOR, O.COL_MAJOR])
@pytest.mark.parametrize("uplo", [O.UPPER, O.LOWER])
@pytest.mark.parametrize("two", [False, True])
def test_syr_syr2(blas, ctx, dt, layout, uplo, two):
    for n in (1, 2, 3, 7, 8, 9, 64, 65, 257, 1000, 1024, 1030, 2310):
        syr_case(blas, ctx, dt, layout, uplo, n, 0.3, 0 if n % 2 else 4, 1, 1, two)
    syr_case(blas, ctx, dt, layout, uplo, 515, -1.5, 1, 2, -3, two)
    syr_case(blas, ctx, dt, layout, uplo, 515, -1.5, 3, -1, 2, two)
    syr_case(blas, ctx, dt, layout, uplo, 2052, 3, 0, 1, 1, two, ints=True)
    # alpha = 0: A untouched even if x, y hold NaN
    A = synth.uniform(14, 0, 100 * 100, dt); dA = to_dev(A); nan = to_dev(np.full(100, np.nan, dt))
    f = blas.routine(prefix_of(dt), "syr2" if two else "syr")
    st = f(ctx.h, layout, uplo, 100, 0.0, nan, 1, nan, 1, dA, 100) if two else f(ctx.h, layout, uplo, 100, 0.0, nan, 1, dA, 100)
    assert st == 0 and bits_equal(to_host(dA), A)


# ----------------------------------------------------------------------------- trsv
def trsv_matrix(dt, n, uplo, diag, seed, exact):
    """A triangular system that substitution solves stably: small off-diagonal elements and a
    diagonal in [1, 2) (exact: entries in {-1, 0, 1} and power-of-two diagonals, so that products
    with an integer solution and the reciprocal of the diagonal are exact).  The opposite triangle
    and, for a unit diagonal, the diagonal hold NaN."""
    if exact:
        A = synth.small_ints(seed, 0, n * n, -1, 1, dt).reshape(n, n).copy()
        d = np.array([1, 2, 0.5, -1, -2, 4], dt)[np.arange(n) % 6]
    else:
        A = (synth.uniform(seed, 0, n * n, dt).reshape(n, n) / dt(2 * np.sqrt(n))).astype(dt)
        d = (dt(1) + np.abs(synth.uniform(seed, 5, n, dt))).astype(dt)
    A[np.arange(n), np.arange(n)] = d
    outside = np.tril(np.ones((n, n), bool), -1) if uplo == O.UPPER else np.triu(np.ones((n, n), bool), 1)
    A[outside] = np.nan
    if diag == O.UNIT:
        np.fill_diagonal(A, np.nan)
    return A


def trsv_case(blas, ctx, dt, layout, uplo, trans, diag, n, pad, incx, exact=False, seed=15):
    A = trsv_matrix(dt, n, uplo, diag, seed, exact)
    Ab, lda = matrix_buffer(A, layout, pad)
    z = synth.small_ints(seed, 1, n, -2, 2, dt) if exact else synth.uniform(seed, 1, n, dt)
    # right-hand side b = op(T) z from the oracle's trmv, so that the solution is known (exact case) and O(1)
    bb = synth.strided(z, incx)
    O.trmv(layout, uplo, trans, diag, n, Ab, lda, bb, incx)
    ref = bb.copy()
    D = O.trsv(layout, uplo, trans, diag, n, Ab, lda, ref, incx, want_D=True)
    dx = to_dev(bb)
    st = blas.routine(prefix_of(dt), "trsv")(ctx.h, layout, uplo, trans, diag, n, mat_dev(Ab), lda, dx, incx)
    assert st == 0, f"status {st}"
    got = to_host(dx)
    what = f"trsv {prefix_of(dt)} layout={layout} uplo={uplo} trans={trans} diag={diag} n={n} pad={pad} incx={incx}"
    g, r = synth.gather(got, n, incx), synth.gather(ref, n, incx)
    if exact:
        assert bits_equal(r, z), what + ": oracle"
        assert bits_equal(g, z), what
    else:
        check_close(g, r, D, n, what)
        # backward error: |b - op(T) g| <= tol * (|op(T)| |g| + |b|), evaluated in fp64
        Tm = np.nan_to_num(logical(Ab, layout, n, n, lda).astype(np.float64))
        if diag == O.UNIT:
            np.fill_diagonal(Tm, 1.0)
        opT = Tm if trans == O.NO_TRANS else Tm.T
        b = synth.gather(bb, n, incx).astype(np.float64)
        res = np.abs(b - opT @ g.astype(np.float64))
        bound = np.abs(opT) @ np.abs(g.astype(np.float64)) + np.abs(b)
        from parity import tight_tolerance
        assert (res <= tight_tolerance(dt, n) * bound).all(), what + f": residual {np.max(res / bound):.3e}"
    gaps = np.ones(got.size, bool); gaps[::abs(incx)] = False
    assert np.isnan(got[gaps]).all(), what


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("layout", [O.ROW_MAJOR, O.COL_MAJOR])
@pytest.mark.parametrize("uplo", [O.UPPER, O.LOWER])
@pytest.mark.parametrize("trans", [O.NO_TRANS, O.TRANS])
@pytest.mark.parametrize("diag", [O.NON_UNIT, O.UNIT])
def test_trsv(blas, ctx, dt, layout, uplo, trans, diag):
    # every size through both paths: one launch per block, then the single chained kernel
    for chain_min in (1 << 30, 1):
        ctx.set_option(blas.OPT_TRSV_CHAIN_MIN, chain_min)
        try:
            for n in (1, 2, 3, 5, 17, 63, 64, 65, 130, 255, 256, 257, 511, 512, 513, 1000, 1030, 2310):
                trsv_case(blas, ctx, dt, layout, uplo, trans, diag, n, 0 if n % 2 else 4, 1)
            trsv_case(blas, ctx, dt, layout, uplo, trans, diag, 700, 1, 2)
            trsv_case(blas, ctx, dt, layout, uplo, trans, diag, 700, 0, -1)
            for n in (64, 515, 1536):
                trsv_case(blas, ctx, dt, layout, uplo, trans, diag, n, 0, 1, exact=True)
        finally:
            ctx.set_option(blas.OPT_TRSV_CHAIN_MIN, 0)
    trsv_case(blas, ctx, dt, layout, uplo, trans, diag, 5000, 0, 1)      # the default choice at a size with many workgroups


def test_trsv_matrices_beyond_the_last_level_cache(blas, ctx):
    """From 384 MiB on (64 MiB in single precision, not transposed, which test_trsv's n = 5000 covers) the
    chained kernel asks for a tile's solutions ahead of the next piece; ragged last blocks, both triangles."""
    for dt, n, pad in ((np.float32, 10250, 2), (np.float64, 7170, 2)):
        for uplo, trans, diag in ((O.LOWER, O.TRANS, O.NON_UNIT), (O.UPPER, O.TRANS, O.UNIT)):
            trsv_case(blas, ctx, dt, O.ROW_MAJOR, uplo, trans, diag, n, pad, 1)
    for uplo, diag in ((O.LOWER, O.UNIT), (O.UPPER, O.NON_UNIT)):
        trsv_case(blas, ctx, np.float64, O.ROW_MAJOR, uplo, O.NO_TRANS, diag, 7170, 2, 1)


def test_trsv_on_several_handles_in_turn(blas, ctx):
    """Each handle has hand-over words of its own (in its workspace, cleared by every call): repeated solves,
    sizes in turn, handles in turn."""
    extra = [blas.Context("cuda:0", workspace_bytes=8 << 20) for _ in range(3)]
    try:
        for rep in range(2):
            for c in [ctx] + extra:
                for n in (1500, 300, 2310):
                    trsv_case(blas, c, np.float32, O.ROW_MAJOR, O.LOWER, O.NO_TRANS, O.NON_UNIT, n, 0, 1, seed=15 + rep)
                trsv_case(blas, c, np.float64, O.ROW_MAJOR, O.UPPER, O.TRANS, O.UNIT, 1030, 2, 1)
    finally:
        for c in extra:
            c.close()


def test_trsv_bounded_wait_reports_timeout(blas, ctx):
    """A wait that the host makes too short to succeed: every wavefront still leaves the kernel, the
    call returns, mxb_last_status names the timeout, and the next call with the default limit is right."""
    dt, n, seed = np.float32, 4096, 23
    A = trsv_matrix(dt, n, O.LOWER, O.NON_UNIT, seed, False)
    Ab, lda = matrix_buffer(A, O.ROW_MAJOR, 0)
    bb = synth.strided(synth.uniform(seed, 1, n, dt), 1)
    O.trmv(O.ROW_MAJOR, O.LOWER, O.NO_TRANS, O.NON_UNIT, n, Ab, lda, bb, 1)
    ref = bb.copy()
    D = O.trsv(O.ROW_MAJOR, O.LOWER, O.NO_TRANS, O.NON_UNIT, n, Ab, lda, ref, 1, want_D=True)
    Ad = mat_dev(Ab)

    def solve():
        dx = to_dev(bb)
        st = blas.mxb_strsv(ctx.h, O.ROW_MAJOR, O.LOWER, O.NO_TRANS, O.NON_UNIT, n, Ad, lda, dx, 1)
        assert st == 0, f"status {st}"
        return dx

    try:
        ctx.set_option(blas.OPT_TRSV_CHAIN_MIN, 1)
        ctx.set_option(blas.OPT_TRSV_SPIN_LIMIT, 1)
        solve()
        assert ctx.last_status() == blas.ERR_TIMEOUT
        # a later call that uses the workspace overwrites the status word: the handle forgets it
        r = to_dev(np.zeros(1, dt))
        assert blas.mxb_sdot(ctx.h, n, to_dev(bb), 1, to_dev(bb), 1, r) == 0
        assert ctx.last_status() == blas.OK
        ctx.set_option(blas.OPT_TRSV_SPIN_LIMIT, 0)
        dx = solve()
        assert ctx.last_status() == blas.OK
        check_close(to_host(dx), ref, D, n, "trsv after a timed-out call")
        ctx.set_option(blas.OPT_TRSV_CHAIN_MIN, 1 << 30)      # the blocked path has no waits and says so
        dx = solve()
        assert ctx.last_status() == blas.OK
        check_close(to_host(dx), ref, D, n, "trsv, blocked, after a timed-out call")
    finally:
        ctx.set_option(blas.OPT_TRSV_CHAIN_MIN, 0)
        ctx.set_option(blas.OPT_TRSV_SPIN_LIMIT, 0)


# ----------------------------------------------------------------------------- skinny matrices
def test_gemv_skinny(blas, ctx):
    """Very short fp32 rows take the kernels that put several rows side by side in a wavefront
    (row-major m x n with small n, or column-major with small m)."""
    dt = np.float32
    for trans in (O.NO_TRANS, O.TRANS):
        for (m, n) in [(500000, 40), (600001, 12), (524288, 48), (500003, 4), (500000, 44)]:
            for pad in (0, 4):
                gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, 1.5, 0.5, pad, 1, 1)
        for alpha, beta in [(1, 0), (1, 1), (-1, 0.5), (0, 0.5)]:
            gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, 500000, 40, alpha, beta, 0, 1, 1)
        for incx, incy in [(2, 3), (-1, 1), (1, -2)]:
            gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, 500000, 24, 1.5, 0.5, 4, incx, incy)
        gemv_case(blas, ctx, dt, O.COL_MAJOR, trans, 40, 500000, 1.5, 0.5, 0, 1, 1)       # the same bytes seen column-major
        gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, 500000, 16, 3, -2, 0, 1, 1, ints=True)
    for (m, n) in [(100000, 40), (131072, 16), (100001, 24), (150000, 48)]:             # not transposed: from 100000 rows
        gemv_case(blas, ctx, dt, O.ROW_MAJOR, O.NO_TRANS, m, n, 1.5, 0.5, 0, 1, 1)
    # not transposed: up to 32 vectors per row (two or more rows per wavefront), and 48 to 64 (one row)
    for (m, n) in [(100000, 49), (100001, 65), (100000, 100), (120000, 127), (100000, 128), (100000, 200), (100003, 255), (100000, 256),
                   (100000, 190), (100000, 129), (100000, 145), (100001, 150), (100000, 160), (100000, 170), (100003, 188)]:
        for pad in (0, 1):
            gemv_case(blas, ctx, dt, O.ROW_MAJOR, O.NO_TRANS, m, n, 1.5, 0.5, pad, 1, 1)
    gemv_case(blas, ctx, dt, O.ROW_MAJOR, O.NO_TRANS, 100000, 255, 3, -2, 0, 2, -1, ints=True)
    # transposed: up to 17 vectors per row
    for (m, n) in [(500000, 56), (500001, 65), (500000, 68), (500000, 69)]:
        gemv_case(blas, ctx, dt, O.ROW_MAJOR, O.TRANS, m, n, 1.5, 0.5, 1, 1, 1)
    gemv_case(blas, ctx, dt, O.ROW_MAJOR, O.TRANS, 500000, 64, 3, -2, 0, 1, 1, ints=True)
    # rows that are not a whole number of vectors, odd pitches, a displaced base
    for off in (0, 1):
        A_OFFSET[0] = off
        try:
            for trans in (O.NO_TRANS, O.TRANS):
                for (m, n) in [(500000, 41), (500001, 5), (500000, 47), (500000, 6), (500000, 39)]:
                    for pad in (0, 1):
                        gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, 1.5, 0.5, pad, 1, 1)
                gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, 500000, 41, 3, -2, 0, 1, 1, ints=True)
        finally:
            A_OFFSET[0] = 0


def test_gemv_skinny_double(blas, ctx):
    """The same kernels in double precision: up to 16 columns from 65536 rows (transposed from 2049), up to 46
    (40) columns from a million (half a million) rows; whole and ragged widths, pitches, increments."""
    dt = np.float64
    for (m, n) in [(100000, 2), (100001, 3), (120000, 8), (100000, 16), (65535, 4), (65536, 2), (65537, 16), (70000, 5)]:
        for pad in (0, 1):
            gemv_case(blas, ctx, dt, O.ROW_MAJOR, O.NO_TRANS, m, n, 1.5, 0.5, pad, 1, 1)
    for (m, n) in [(100000, 2), (100001, 5), (120000, 8)]:
        for pad in (0, 1):
            gemv_case(blas, ctx, dt, O.ROW_MAJOR, O.TRANS, m, n, 1.5, 0.5, pad, 1, 1)
    for (m, n) in [(1000000, 41), (1000001, 46), (1000000, 24), (1000000, 49), (1000000, 64), (1000000, 63), (1000000, 65),
                   (1000000, 42), (1000003, 50), (1000000, 62)]:
        gemv_case(blas, ctx, dt, O.ROW_MAJOR, O.NO_TRANS, m, n, 1.5, 0.5, 1, 1, 1)
    for (m, n) in [(500000, 40), (500001, 33), (600000, 12)]:
        gemv_case(blas, ctx, dt, O.ROW_MAJOR, O.TRANS, m, n, 1.5, 0.5, 1, 1, 1)
    for trans in (O.NO_TRANS, O.TRANS):
        for incx, incy in [(2, 3), (-1, 1), (1, -2)]:
            gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, 500000, 8, 1.5, 0.0, 4, incx, incy)
        gemv_case(blas, ctx, dt, O.COL_MAJOR, trans, 8, 500000, 1.5, 0.5, 0, 1, 1)
        gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, 500000, 7, 3, -2, 0, 1, 1, ints=True)
        A_OFFSET[0] = 1
        try:
            gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, 500000, 5, 1.5, 0.5, 1, 1, 1)
        finally:
            A_OFFSET[0] = 0


@pytest.mark.parametrize("dt", DT)
def test_ger_skinny(blas, ctx, dt):
    for (m, n) in [(100000, 40), (131072, 16), (100001, 24), (150000, 4), (100000, 8), (16383, 4), (16384, 8), (20001, 40), (30000, 6)] + (
            [(120000, 48), (100000, 56), (100000, 64), (100000, 60), (100000, 68), (100001, 72), (100000, 80), (100000, 84)] if dt == np.float32 else []):
        for pad in (0, 4):
            ger_case(blas, ctx, dt, O.ROW_MAJOR, m, n, 0.3, pad, 1, 1)
    ger_case(blas, ctx, dt, O.ROW_MAJOR, 100000, 40, -1.5, 4, 2, -3)
    ger_case(blas, ctx, dt, O.COL_MAJOR, 40, 100000, -1.5, 0, 1, 1)
    ger_case(blas, ctx, dt, O.ROW_MAJOR, 100000, 32, 3, 0, 1, 1, ints=True)
    # rows that are not a whole number of vectors, odd pitches, a displaced base
    for off in (0, 1):
        A_OFFSET[0] = off
        try:
            for (m, n) in [(100000, 41), (100001, 5), (100000, 39), (100000, 3 if dt == np.float64 else 6)]:
                for pad in (0, 1):
                    ger_case(blas, ctx, dt, O.ROW_MAJOR, m, n, 0.3, pad, 1, 1)
            ger_case(blas, ctx, dt, O.ROW_MAJOR, 100000, 37, 3, 1, 1, 1, ints=True)
        finally:
            A_OFFSET[0] = 0


def test_streaming_variants_just_past_the_cache_limits(blas, ctx):
    """Kernels come in two variants, for a matrix that stays in the caches between calls and for one
    that streams from HBM (192 MiB apart).  The other tests of this file are on the small side; these
    shapes lie just past the limit: 1300000 x 40 floats (short rows: A*x, A^t*x, rank-1 update), a
    7300^2 double triangle (syr), 7200^2 floats (A^t*x through the partial vectors)."""
    for trans in (O.NO_TRANS, O.TRANS):
        gemv_case(blas, ctx, np.float32, O.ROW_MAJOR, trans, 1300000, 40, 0.75, 0.5, 0, 1, 1)
    ger_case(blas, ctx, np.float32, O.ROW_MAJOR, 1300000, 40, 0.3, 0, 1, 1)
    syr_case(blas, ctx, np.float64, O.ROW_MAJOR, O.UPPER, 7300, 0.3, 0, 1, 1, False)
    gemv_case(blas, ctx, np.float32, O.ROW_MAJOR, O.TRANS, 7200, 7200, 0.75, 0.5, 0, 1, 1)


@pytest.mark.parametrize("dt", DT)
def test_rows_narrower_than_one_vector(blas, ctx, dt):
    """Matrices of 1 to 3 columns (1 in double precision) with many rows take the side-by-side kernels
    with one element per lane: A*x from 65536 rows, A^t*x from 200000, x*y^t from 16384; whole and
    ragged tiles, a pitch larger than the width, increments, a displaced base, exact integers, and the
    sizes just below the limits, which stay with the general kernels."""
    widths = (1, 2, 3) if dt == np.float32 else (1,)
    for n in widths:
        for m in (65535, 65536, 200001, 262144 + 7):
            for pad in (0, 1, 5):
                gemv_case(blas, ctx, dt, O.ROW_MAJOR, O.NO_TRANS, m, n, 1.5, 0.5, pad, 1, 1)
        for m in (199999, 200000, 300007):
            for pad in (0, 2):
                gemv_case(blas, ctx, dt, O.ROW_MAJOR, O.TRANS, m, n, 1.5, 0.5, pad, 1, 1)
        for m in (16383, 16384, 70001):
            for pad in (0, 3):
                ger_case(blas, ctx, dt, O.ROW_MAJOR, m, n, 0.3, pad, 1, 1)
        for trans, m in ((O.NO_TRANS, 100003), (O.TRANS, 250000)):
            gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, 1.5, 0.0, 0, 2, -3)
            gemv_case(blas, ctx, dt, O.ROW_MAJOR, trans, m, n, 3, -2, 1, -1, 1, ints=True)
            gemv_case(blas, ctx, dt, O.COL_MAJOR, trans, n, m, 1.5, 0.5, 0, 1, 1)     # the same bytes seen column-major
        ger_case(blas, ctx, dt, O.ROW_MAJOR, 50001, n, -1.5, 1, 2, -3)
        ger_case(blas, ctx, dt, O.ROW_MAJOR, 40000, n, 3, 0, 1, 1, ints=True)
        ger_case(blas, ctx, dt, O.COL_MAJOR, n, 40000, 0.3, 0, 1, 1)
    A_OFFSET[0] = 1
    try:
        gemv_case(blas, ctx, dt, O.ROW_MAJOR, O.NO_TRANS, 100000, widths[-1], 1.5, 0.5, 1, 1, 1)
        gemv_case(blas, ctx, dt, O.ROW_MAJOR, O.TRANS, 250001, widths[-1], 1.5, 0.5, 1, 1, 1)
        ger_case(blas, ctx, dt, O.ROW_MAJOR, 30000, widths[-1], 0.3, 1, 1, 1)
    finally:
        A_OFFSET[0] = 0
