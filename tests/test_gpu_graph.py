"""The library only enqueues kernels on the handle's stream (no allocation, no memset, no
synchronisation), so a sequence of calls can be captured into a HIP graph.  Every replay must give
the bits of the eager run, also with other work and synchronisations between the replays.  The
chained trsv kernel, whose workgroups wait for each other, is part of the sequence."""
import numpy as np
import pytest
import torch

from paper_2411_07211_amd import synth
from parity import to_dev, to_host

pytestmark = pytest.mark.gpu


def test_captured_sequence_replays_bit_for_bit(blas, ctx):
    B, h = blas, ctx.h
    n, m = 3000, 1500
    f = np.float32
    A = to_dev(synth.uniform(40, 0, n * n, f)); x0 = synth.uniform(40, 1, n, f); y0 = synth.uniform(40, 2, n, f)
    x, y, z, t = to_dev(x0), to_dev(y0), to_dev(y0), to_dev(x0)
    r = torch.zeros(2, dtype=torch.float32, device=A.device)
    k = 600                                          # a well-conditioned triangular system for trsv
    T = (A[:k * k] * 0.02).view(k, k).contiguous()
    T.diagonal().add_(1.5)
    s = torch.zeros(k, dtype=torch.float32, device=A.device)

    def sequence():
        # reads and writes chained through y, z, t and r: gemv N and T, both symv paths, trmv, level 1
        assert B.mxb_sgemv(h, B.ROW_MAJOR, B.NO_TRANS, n, n, 1.0, A, n, x, 1, 0.0, y, 1) == 0
        assert B.mxb_sgemv(h, B.ROW_MAJOR, B.TRANS, n, n, 0.5, A, n, y, 1, 0.5, z, 1) == 0
        assert B.mxb_ssymv(h, B.ROW_MAJOR, B.LOWER, n, 1.0, A, n, z, 1, 0.0, y, 1) == 0          # triangle sweep + combine
        assert B.mxb_ssymv(h, B.ROW_MAJOR, B.UPPER, m, 1.0, A, n, y, 1, 1.0, z, 1) == 0          # single kernel
        assert B.mxb_scopy(h, n, z, 1, t, 1) == 0
        assert B.mxb_strmv(h, B.ROW_MAJOR, B.UPPER, B.NO_TRANS, B.UNIT, n, A, n, t, 1) == 0      # snapshot + row-dot
        assert B.mxb_strmv(h, B.ROW_MAJOR, B.LOWER, B.TRANS, B.NON_UNIT, m, A, n, t, 1) == 0
        assert B.mxb_sscal(h, n, 1e-3, t, 1) == 0
        assert B.mxb_saxpy(h, n, -0.75, t, 1, z, 1) == 0
        assert B.mxb_sdot(h, n, t, 1, z, 1, r) == 0
        assert B.mxb_snrm2(h, n, z, 1, r[1:]) == 0
        assert B.mxb_sgemv_batched(h, B.ROW_MAJOR, B.NO_TRANS, 100, 30, 1.0, A, 30, 3000, z, 1, 30, 0.0, y, 1, 100, 30) == 0
        assert B.mxb_scopy(h, k, z, 1, s, 1) == 0
        assert B.mxb_strsv(h, B.ROW_MAJOR, B.LOWER, B.NO_TRANS, B.NON_UNIT, k, T, k, s, 1) == 0  # one chained kernel (and the one that clears its words)
        assert B.mxb_strsv(h, B.ROW_MAJOR, B.UPPER, B.TRANS, B.NON_UNIT, 200, T, k, s, 1) == 0   # one launch per block

    def reset():
        x.copy_(to_dev(x0)); y.copy_(to_dev(y0)); z.copy_(to_dev(y0)); t.copy_(to_dev(x0)); r.zero_(); s.zero_()

    reset(); sequence(); torch.cuda.synchronize()
    eager = [to_host(v).copy() for v in (y, z, t, r, s)]
    assert all(np.isfinite(e).all() for e in eager)

    reset(); torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        ctx.use_current_stream()
        sequence()
    ctx.use_current_stream()
    for rep in range(4):
        reset()
        if rep % 2:                                   # the program's own eager work between replays
            assert B.mxb_sscal(h, n, 2.0, to_dev(x0), 1) == 0
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = [to_host(v) for v in (y, z, t, r, s)]
        for a, b in zip(got, eager):
            assert a.tobytes() == b.tobytes(), f"replay {rep} differs from the eager run"
