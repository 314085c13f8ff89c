"""mxb_sgemv_static (gemv for callers that cannot allocate: partial vectors in the library's static
device array) against mxb_sgemv with a workspace, through the C ABI: bitwise the same result, on
calls in a row of which the later ones are smaller, and against the CPU oracle."""
import numpy as np
import pytest

import oracle as O
from paper_2411_07211_amd import synth
from parity import check_close, to_dev, to_host

pytestmark = pytest.mark.gpu


def both(blas, ctx, bare, trans, m, n, alpha, beta, pad=0, incx=1, incy=1, seed=21):
    """One problem through mxb_sgemv (handle with workspace) and mxb_sgemv_static (handle without)."""
    f = np.float32
    lda = n + pad
    A = np.full((m, lda), np.nan, f)
    A[:, :n] = synth.uniform(seed, 0, m * n, f).reshape(m, n)
    lenx, leny = (n, m) if trans == O.NO_TRANS else (m, n)
    x = synth.strided(synth.uniform(seed, 1, lenx, f), incx)
    y = synth.strided(synth.uniform(seed, 2, leny, f) if beta != 0 else np.full(leny, np.nan, f), incy)
    dA, dx = to_dev(A.ravel()), to_dev(x)
    y_ws, y_st = to_dev(y), to_dev(y)
    what = f"sgemv trans={trans} {m}x{n} lda={lda} beta={beta} inc=({incx},{incy})"
    print(what, flush=True)
    assert blas.mxb_sgemv(ctx.h, O.ROW_MAJOR, trans, m, n, alpha, dA, lda, dx, incx, beta, y_ws, incy) == 0, what
    assert blas.mxb_sgemv_static(bare, O.ROW_MAJOR, trans, m, n, alpha, dA, lda, dx, incx, beta, y_st, incy) == 0, what
    got_ws, got_st = to_host(y_ws), to_host(y_st)
    assert got_ws.tobytes() == got_st.tobytes(), what + ": differs from mxb_sgemv"
    ref = y.copy()
    D = O.gemv(O.ROW_MAJOR, trans, m, n, f(alpha), A.ravel(), lda, x, incx, f(beta), ref, incy, want_D=True)
    check_close(synth.gather(got_st, leny, incy), synth.gather(ref, leny, incy), D, lenx, what)


def test_static_scratch_matches_workspace_path(blas, ctx):
    st, bare = blas.mxb_create()          # no workspace on this handle
    assert st == 0
    import torch
    assert blas.mxb_set_stream(bare, torch.cuda.current_stream().cuda_stream) == 0
    try:
        # without a workspace the plain call refuses a transposed product that needs partial vectors
        f = np.float32
        dA, dx, dy = to_dev(np.zeros(4096 * 4096, f)), to_dev(np.zeros(4096, f)), to_dev(np.zeros(4096, f))
        assert blas.mxb_sgemv(bare, O.ROW_MAJOR, O.TRANS, 4096, 4096, 1.0, dA, 4096, dx, 1, 0.0, dy, 1) == blas.ERR_WORKSPACE
        del dA, dx, dy
        # transposed: column-accumulate kernel + combine pass (partial vectors in the scratch array);
        # the second and third calls are smaller than the first, so they find its leftovers there
        both(blas, ctx, bare, O.TRANS, 6000, 5000, 1.25, 0.5, pad=8)
        both(blas, ctx, bare, O.TRANS, 2500, 1037, -0.75, 0.0)
        both(blas, ctx, bare, O.TRANS, 300, 130, 2.0, 1.0, incx=2, incy=3)
        # skinny transposed (one partial vector per block), then few very long rows not transposed
        both(blas, ctx, bare, O.TRANS, 600000, 40, 1.0, 0.5)
        both(blas, ctx, bare, O.NO_TRANS, 3, 100000, 1.0, 0.5)
        both(blas, ctx, bare, O.NO_TRANS, 200, 40000, 1.0, 0.0)
        # not transposed, no partial vectors at all
        both(blas, ctx, bare, O.NO_TRANS, 3000, 2000, 1.5, 0.5, pad=3)
        both(blas, ctx, bare, O.TRANS, 1500, 700, 1.5, 0.5)
    finally:
        blas.mxb_destroy(bare)


def test_static_scratch_limit_and_argument_errors(blas, ctx):
    st, bare = blas.mxb_create()
    assert st == 0
    try:
        m, n = 512, 782336          # two partial vectors of 782336 floats: 6 MiB, more than the array holds
        assert blas.mxb_workspace_bytes(blas.GEMV, 4, m, n) > blas.STATIC_SCRATCH_BYTES
        import torch
        A = torch.zeros(m * n, dtype=torch.float32, device="cuda")
        x = torch.zeros(m, dtype=torch.float32, device="cuda")
        y = torch.full((n,), 7.0, dtype=torch.float32, device="cuda")
        assert blas.mxb_sgemv_static(bare, O.ROW_MAJOR, O.TRANS, m, n, 1.0, A, n, x, 1, 0.0, y, 1) == blas.ERR_STATIC_LIMIT
        torch.cuda.synchronize()
        assert float(y.min()) == 7.0 and float(y.max()) == 7.0          # nothing was launched
        # argument errors as mxb_sgemv
        assert blas.mxb_sgemv_static(bare, 7, O.TRANS, 4, 4, 1.0, A, 4, x, 1, 0.0, y, 1) == -1
        assert blas.mxb_sgemv_static(bare, O.ROW_MAJOR, O.TRANS, 4, 4, 1.0, A, 3, x, 1, 0.0, y, 1) == -7
        assert blas.mxb_sgemv_static(bare, O.ROW_MAJOR, O.TRANS, 0, 4, 1.0, A, 4, x, 1, 0.0, y, 1) == 0
        # the handle's own workspace is left alone
        assert blas.mxb_sgemv_static(ctx.h, O.ROW_MAJOR, O.TRANS, 64, 64, 1.0, A, 64, x, 1, 0.0, y, 1) == 0
        r = torch.zeros(1, dtype=torch.float32, device="cuda")
        assert blas.mxb_sdot(ctx.h, 512, x, 1, x, 1, r) == 0         # still has its workspace
    finally:
        blas.mxb_destroy(bare)
