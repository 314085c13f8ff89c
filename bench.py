#!/usr/bin/env python3
"""Benchmark of the BLAS level-1 / level-2 hot path on one MI355X.

A *step* is one pass over the whole routine family at full size on seeded synthetic data that is
already resident in HBM: the level-1 suite at n = 2^28 (unit stride and incx=2/incy=3), sgemv N/T
at 16384^2 and 1048576x256 with beta in {0, 1, 0.5}, dgemv N/T at 16384^2 with lda = 16392,
strmv (4 variants), ssymv and sger at 16384, plus the small 1024^2 sgemv.  `value` is the
algorithmic bytes of a step divided by its wall time.  Every routine is also bracketed by events on
the stream it is launched on; those give the per-routine GB/s and the `roofline` object (for the
row-dot kernel behind sgemv N at 16384^2, the shape the headline metric is quoted on).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--only NAME[,NAME...]] [--no-cpu-baseline]

`--only` restricts the step to the named routines (see --list), e.g. for profiling one kernel.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
GiB = 1 << 30


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--only", type=str, default="")
    ap.add_argument("--list", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--traffic-from", nargs=2, metavar=("FETCH_DIR", "WRITE_DIR"),
                    help="no GPU work: parse two rocprofv3 --pmc output folders of `bench.py --only $(bench.py --traffic-list)` "
                         "(FETCH_SIZE, WRITE_SIZE) into profiles/traffic.json")
    ap.add_argument("--traffic-list", action="store_true", help="print the --only list the traffic counters are collected on")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the step: time every routine over a sweep of sizes (small, medium, large buckets, "
                         "skinny N = 40 shapes) and print a markdown table with the geometric mean per bucket")
    ap.add_argument("--scale", type=int, default=1, help="divide every problem size by this (debugging only; "
                    "a scaled run is not the benchmark and says so in its output)")
    return ap.parse_args()


class Suite:
    """Device buffers and the list of routine calls that make up one step."""

    def __init__(self, blas, ctx, torch, scale=1):
        self.B, self.ctx, self.torch = blas, ctx, torch
        dev = ctx.device
        g = torch.Generator(device=dev)
        self.calls = []            # (name, kernel family, fn(step_index), algorithmic bytes, untimed set-up or None)
        f32, f64 = torch.float32, torch.float64

        def uni(n, dtype, seed):
            g.manual_seed(seed)
            return torch.rand(n, dtype=dtype, device=dev, generator=g).mul_(2).sub_(1)

        def nrm(n, dtype, seed, std=1.0):
            g.manual_seed(seed)
            return torch.randn(n, dtype=dtype, device=dev, generator=g).mul_(std)

        h, B = ctx.h, blas
        n1 = (1 << 28) // scale
        NS = 16384 // (scale if scale <= 16 else 16)
        MT, NT = (1 << 20) // scale, 256

        # ---- level 1, n = 2^28, seed 1: dense and strided (incx = 2, incy = 3) ----------------
        self.res = {"s": torch.zeros(1, dtype=f32, device=dev), "d": torch.zeros(1, dtype=f64, device=dev)}
        for p, dt, e in (("s", f32, 4), ("d", f64, 8)):
            x, y = uni(n1, dt, 101), uni(n1, dt, 102)
            xs_, ys_ = uni(2 * n1, dt, 103), uni(3 * n1, dt, 104)
            r = self.res[p]
            for tag, xx, ix, yy, iy in (("", x, 1, y, 1), ("_strided", xs_, 2, ys_, 3)):
                ax = B.routine(p, "axpy")
                self.add(f"{p}axpy{tag}", "axpy", lambda s, ax=ax, xx=xx, ix=ix, yy=yy, iy=iy: ax(h, n1, -0.75, xx, ix, yy, iy), 3 * n1 * e)
                dot = B.routine(p, "dot")
                self.add(f"{p}dot{tag}", "dot", lambda s, dot=dot, xx=xx, ix=ix, yy=yy, iy=iy, r=r: dot(h, n1, xx, ix, yy, iy, r), 2 * n1 * e)
                if p == "s":
                    sc, asum, nrm2 = B.mxb_sscal, B.mxb_sasum, B.mxb_snrm2
                    # alternate 1.25 and 0.8 so that repeated scaling stays bounded
                    self.add(f"sscal{tag}", "scal", lambda s, xx=xx, ix=ix: sc(h, n1, 1.25 if s % 2 == 0 else 0.8, xx, ix), 2 * n1 * e)
                    self.add(f"sasum{tag}", "asum", lambda s, xx=xx, ix=ix, r=r: asum(h, n1, xx, ix, r), n1 * e)
                    self.add(f"snrm2{tag}", "nrm2", lambda s, xx=xx, ix=ix, r=r: nrm2(h, n1, xx, ix, r), n1 * e)
            self.__dict__[f"keep_{p}"] = (x, y, xs_, ys_)

        # ---- sgemv, seed 2: 16384^2 and 1048576 x 256, rotating over three copies of A --------
        A32 = [uni(NS * NS, f32, 200 + k) for k in range(3)]
        assert MT * NT <= NS * NS
        xs, ys = uni(max(NS, MT), f32, 210), uni(max(NS, MT), f32, 211)
        self.rot = 0

        def nextA(pool):
            self.rot += 1
            return pool[self.rot % len(pool)]

        for beta in (0.0, 1.0, 0.5):
            for tname, trans in (("n", B.NO_TRANS), ("t", B.TRANS)):
                rd = 0 if beta == 0 else 1
                self.add(f"sgemv_{tname}_{NS}_b{beta:g}", "gemv_" + tname,
                         lambda s, trans=trans, beta=beta: B.mxb_sgemv(h, B.ROW_MAJOR, trans, NS, NS, 1.0, nextA(A32), NS, xs, 1, beta, ys, 1),
                         4 * (NS * NS + NS + NS * (1 + rd)))
                lenx, leny = (NT, MT) if trans == B.NO_TRANS else (MT, NT)
                self.add(f"sgemv_{tname}_{MT}x{NT}_b{beta:g}", "gemv_" + tname,
                         lambda s, trans=trans, beta=beta: B.mxb_sgemv(h, B.ROW_MAJOR, trans, MT, NT, 1.0, nextA(A32), NT, xs, 1, beta, ys, 1),
                         4 * (MT * NT + lenx + leny * (1 + rd)))
        # the small, latency-bound case (1024^2, alpha = 1.5, beta = 0.5)
        n0 = 1024
        self.add("sgemv_n_1024", "gemv_n", lambda s: B.mxb_sgemv(h, B.ROW_MAJOR, B.NO_TRANS, n0, n0, 1.5, A32[0], n0, xs, 1, 0.5, ys, 1),
                 4 * (n0 * n0 + n0 + 2 * n0))

        # ---- dgemv, seed 3: 16384^2, lda = 16392, A ~ N(0, 1/sqrt(N)), beta = 0 ---------------
        lda = NS + 8
        A64 = [nrm(NS * lda, f64, 300 + k, 1.0 / np.sqrt(NS)) for k in range(2)]
        xd, yd = nrm(NS, f64, 310), nrm(NS, f64, 311)
        for tname, trans in (("n", B.NO_TRANS), ("t", B.TRANS)):
            self.add(f"dgemv_{tname}_{NS}", "gemv_" + tname,
                     lambda s, trans=trans: B.mxb_dgemv(h, B.ROW_MAJOR, trans, NS, NS, 2.0, nextA(A64), lda, xd, 1, 0.0, yd, 1),
                     8 * (NS * NS + NS + NS))

        # ---- structured level 2, fp32, n = 16384, seed 4 ---------------------------------------
        x0 = uni(NS, f32, 410)
        xt = x0.clone()
        tri = NS * (NS + 1) // 2
        for uname, uplo in (("u", B.UPPER), ("l", B.LOWER)):
            for dname, diag in (("n", B.NON_UNIT), ("u", B.UNIT)):
                def trmv(s, uplo=uplo, diag=diag):
                    return B.mxb_strmv(h, B.ROW_MAJOR, uplo, B.NO_TRANS, diag, NS, nextA(A32), NS, xt, 1)
                nel = tri if diag == B.NON_UNIT else tri - NS
                # x := T x would blow up over repeated steps: restart from the same x before every call
                # (a torch copy, outside the call's own events)
                self.add(f"strmv_{uname}{dname}_{NS}", "trmv", trmv, 4 * (nel + 2 * NS), pre=lambda: xt.copy_(x0))
        self.add(f"ssymv_l_{NS}", "symv", lambda s: B.mxb_ssymv(h, B.ROW_MAJOR, B.LOWER, NS, 0.52, nextA(A32), NS, xs, 1, 0.49, ys, 1),
                 4 * (tri + 3 * NS))
        self.add(f"sger_{NS}", "ger", lambda s: B.mxb_sger(h, B.ROW_MAJOR, NS, NS, 1e-3, xs, 1, x0, 1, nextA(A32), NS),
                 4 * (2 * NS * NS + 2 * NS))
        self.keep = (A32, A64, xs, ys, xd, yd, x0, xt)

        # ---- bandwidth probes: not part of a step, selectable with --only ----------------------
        nb = NS * NS * 4
        reset = lambda: xt.copy_(x0)
        self.extra = [
            ("probe_copy", "probe", lambda s: B.mxb_probe_copy(h, nb, A32[1], A32[2]), 2 * nb, None),
            ("probe_read", "probe", lambda s: B.mxb_probe_read(h, nb, nextA(A32)), nb, None),
            # the variants of the structured routines that the step does not contain
            (f"strmv_ut_{NS}", "trmv_t", lambda s: B.mxb_strmv(h, B.ROW_MAJOR, B.UPPER, B.TRANS, B.NON_UNIT, NS, nextA(A32), NS, xt, 1),
             4 * (tri + 2 * NS), reset),
            (f"strmv_lt_{NS}", "trmv_t", lambda s: B.mxb_strmv(h, B.ROW_MAJOR, B.LOWER, B.TRANS, B.NON_UNIT, NS, nextA(A32), NS, xt, 1),
             4 * (tri + 2 * NS), reset),
            (f"ssymv_u_{NS}", "symv", lambda s: B.mxb_ssymv(h, B.ROW_MAJOR, B.UPPER, NS, 0.52, nextA(A32), NS, xs, 1, 0.49, ys, 1),
             4 * (tri + 3 * NS), None),
            (f"dsymv_l_{NS}", "symv", lambda s: B.mxb_dsymv(h, B.ROW_MAJOR, B.LOWER, NS, 0.52, nextA(A64), lda, xd, 1, 0.49, yd, 1),
             8 * (tri + 3 * NS), None),
            # trsv: unit diagonal over small off-diagonal elements (a random triangle is exponentially ill conditioned)
            (f"strsv_ln_{NS}", "trsv", lambda s: B.mxb_strsv(h, B.ROW_MAJOR, B.LOWER, B.NO_TRANS, B.UNIT, NS, self.small(), NS, xt, 1),
             4 * (tri - NS + 2 * NS), reset),
            (f"strsv_lt_{NS}", "trsv", lambda s: B.mxb_strsv(h, B.ROW_MAJOR, B.LOWER, B.TRANS, B.UNIT, NS, self.small(), NS, xt, 1),
             4 * (tri - NS + 2 * NS), reset),
        ]
        self._small = None
        self._small_from = A32[0]

    def small(self):
        """A 16384^2 matrix of elements below 1e-4, made on first use (only the trsv extras want it)."""
        if self._small is None:
            self._small = self._small_from * 1e-4
        return self._small

    def add(self, name, family, fn, nbytes, pre=None):
        self.calls.append((name, family, fn, int(nbytes), pre))


def cpu_baseline(torch):
    """The oracle, as it stands, timed single-threaded on this host on a bounded sample of the
    step: level-1 at n = 2^27 (unit stride), the matrix routines at full size, each once."""
    import oracle as O
    from paper_2411_07211_amd import synth
    n1, ns, mt, nt = 1 << 27, 16384, 1 << 20, 256
    total = 0
    t_total = 0.0

    def timed(fn, nbytes):
        nonlocal total, t_total
        t0 = time.perf_counter(); fn(); t_total += time.perf_counter() - t0
        total += nbytes

    for dt, e in ((np.float32, 4), (np.float64, 8)):
        x, y = synth.uniform(1, 1, n1, dt), synth.uniform(1, 2, n1, dt)
        timed(lambda: O.axpy(n1, dt(-0.75), x, 1, y, 1), 3 * n1 * e)
        timed(lambda: O.dot(n1, x, 1, y, 1), 2 * n1 * e)
        if dt == np.float32:
            timed(lambda: O.scal(n1, dt(1.25), x, 1), 2 * n1 * e)
            timed(lambda: O.asum(n1, x, 1), n1 * e)
            timed(lambda: O.nrm2(n1, x, 1), n1 * e)
    A = synth.uniform(2, 0, ns * ns, np.float32)
    xs, ys = synth.uniform(2, 1, mt, np.float32), synth.uniform(2, 2, mt, np.float32)
    f = np.float32
    for trans in (O.NO_TRANS, O.TRANS):
        timed(lambda: O.gemv(O.ROW_MAJOR, trans, ns, ns, f(1), A, ns, xs, 1, f(0.5), ys, 1), 4 * (ns * ns + 3 * ns))
        timed(lambda: O.gemv(O.ROW_MAJOR, trans, mt, nt, f(1), A, nt, xs, 1, f(0.5), ys, 1), 4 * (mt * nt + mt + nt + (mt if trans == O.NO_TRANS else nt)))
    Ad = synth.normal(3, 0, ns * ns, 1 / np.sqrt(ns), np.float64)
    xd, yd = synth.normal(3, 1, ns, 1.0, np.float64), synth.normal(3, 2, ns, 1.0, np.float64)
    for trans in (O.NO_TRANS, O.TRANS):
        timed(lambda: O.gemv(O.ROW_MAJOR, trans, ns, ns, 2.0, Ad, ns, xd, 1, 0.0, yd, 1), 8 * (ns * ns + 2 * ns))
    tri = ns * (ns + 1) // 2
    xt = xs[:ns].copy()
    timed(lambda: O.trmv(O.ROW_MAJOR, O.UPPER, O.NO_TRANS, O.NON_UNIT, ns, A, ns, xt, 1), 4 * (tri + 2 * ns))
    timed(lambda: O.symv(O.ROW_MAJOR, O.LOWER, ns, f(0.5), A, ns, xs, 1, f(0.5), ys, 1), 4 * (tri + 3 * ns))
    timed(lambda: O.ger(O.ROW_MAJOR, ns, ns, f(1e-3), xs, 1, ys, 1, A, ns), 4 * (2 * ns * ns + 2 * ns))
    return {
        "value": round(total / t_total / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": "each routine of the step once (level-1 at n=2^27 unit stride, s+d; s/dgemv N,T 16384^2; sgemv N,T "
                  "1048576x256; strmv, ssymv, sger 16384^2), single thread, gcc -O2, long-double accumulation, "
                  f"{total / 1e9:.2f} GB algorithmic in {t_total:.1f} s",
    }


def sweep(B, ctx, torch):
    """Size sweeps in the style of the paper's evaluation (Sec. 6.2: problem sizes in buckets,
    one geometric mean per bucket; skinny matrices with N = 40 and M powers of 2 and 3).  Buckets
    by the bytes a call moves: small < 4 MiB (launch latency), medium < 256 MiB (fits the
    last-level cache), large beyond.  Times are medians of 20 event-timed calls after 3 warm-ups."""
    h, dev = ctx.h, ctx.device
    f32 = torch.float32

    def timed(fn, pre=None, iters=20, warm=3):
        for _ in range(warm):
            if pre: pre()
            assert fn() == 0
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
        for a, b in ev:
            if pre: pre()
            a.record(); st = fn(); b.record()
            assert st == 0, st
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) for a, b in ev)
        return ts[len(ts) // 2] * 1e3          # us

    def replayed(fn, pre=None, calls=20, reps=5):
        """us per call when `calls` calls in a row are captured into one HIP graph and replayed:
        what the GPU needs for a call once the host's launch cost is out of the way."""
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            ctx.use_current_stream()
            for _ in range(calls):
                if pre: pre()
                assert fn() == 0
        ctx.use_current_stream()
        g.replay()
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in ev:
            a.record(); g.replay(); b.record()
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) for a, b in ev)
        return ts[len(ts) // 2] * 1e3 / calls

    rows = []          # (routine, shape text, bytes, us of a single call, us per call in a replayed graph or None)

    def rec(name, shape, nbytes, fn, pre=None):
        us = timed(fn, pre)
        gus = replayed(fn, pre) if us < 60 else None
        rows.append((name, shape, nbytes, us, gus))
        print(f"{name:10s} {shape:>16s} {nbytes / 2**20:10.2f} MiB {us:9.1f} us {nbytes / us / 1e3:8.1f} GB/s"
              + (f"   in a graph {gus:7.1f} us {nbytes / gus / 1e3:8.1f} GB/s" if gus else ""), file=sys.stderr, flush=True)

    nmax = 1 << 28
    x = torch.rand(nmax, dtype=f32, device=dev); y = torch.rand(nmax, dtype=f32, device=dev)
    r = torch.zeros(1, dtype=f32, device=dev)
    for e in range(10, 29, 2):
        n = 1 << e
        for n_ in (n, n - 3 if e < 28 else n):
            t = f"n={n_}"
            rec("saxpy", t, 12 * n_, lambda: B.mxb_saxpy(h, n_, -0.75, x, 1, y, 1))
            rec("sscal", t, 8 * n_, lambda: B.mxb_sscal(h, n_, 1.0, x, 1))
            rec("sdot", t, 8 * n_, lambda: B.mxb_sdot(h, n_, x, 1, y, 1, r))
            rec("sasum", t, 4 * n_, lambda: B.mxb_sasum(h, n_, x, 1, r))
            rec("snrm2", t, 4 * n_, lambda: B.mxb_snrm2(h, n_, x, 1, r))
    NS = 16384
    A = x                       # 2^28 floats hold a 16384 x 16384 matrix
    xv = torch.rand(1 << 22, dtype=f32, device=dev); yv = torch.rand(1 << 22, dtype=f32, device=dev)
    x0 = torch.rand(NS, dtype=f32, device=dev); xt = x0.clone()
    reset = lambda: xt.copy_(x0)
    for n in (256, 512, 1000, 1024, 2048, 3000, 4096, 6001, 8192, 12000, 16384):
        t, full, tri = f"{n}x{n}", 4 * n * n, 4 * (n * (n + 1) // 2)
        rec("sgemv_n", t, full, lambda: B.mxb_sgemv(h, B.ROW_MAJOR, B.NO_TRANS, n, n, 1.0, A, n, xv, 1, 0.0, yv, 1))
        rec("sgemv_t", t, full, lambda: B.mxb_sgemv(h, B.ROW_MAJOR, B.TRANS, n, n, 1.0, A, n, xv, 1, 0.0, yv, 1))
        rec("sger", t, 2 * full, lambda: B.mxb_sger(h, B.ROW_MAJOR, n, n, 1e-6, xv, 1, yv, 1, A, n))
        rec("ssymv_l", t, tri, lambda: B.mxb_ssymv(h, B.ROW_MAJOR, B.LOWER, n, 0.5, A, n, xv, 1, 0.5, yv, 1))
        rec("ssyr_l", t, 2 * tri, lambda: B.mxb_ssyr(h, B.ROW_MAJOR, B.LOWER, n, 1e-6, xv, 1, A, n))
        rec("strmv_un", t, tri, lambda: B.mxb_strmv(h, B.ROW_MAJOR, B.UPPER, B.NO_TRANS, B.NON_UNIT, n, A, n, xt, 1), reset)
        rec("strmv_lt", t, tri, lambda: B.mxb_strmv(h, B.ROW_MAJOR, B.LOWER, B.TRANS, B.NON_UNIT, n, A, n, xt, 1), reset)
    # trsv wants a well-conditioned triangle: unit diagonal, small off-diagonal elements
    T = torch.rand(NS * NS, dtype=f32, device=dev).mul_(1e-4)
    for n in (256, 1024, 4096, 16384):
        tri = 4 * (n * (n + 1) // 2)
        rec("strsv_lu", f"{n}x{n}", tri, lambda: B.mxb_strsv(h, B.ROW_MAJOR, B.LOWER, B.NO_TRANS, B.UNIT, n, T, n, xt, 1), reset)
        rec("strsv_ltu", f"{n}x{n}", tri, lambda: B.mxb_strsv(h, B.ROW_MAJOR, B.LOWER, B.TRANS, B.UNIT, n, T, n, xt, 1), reset)
    del T
    # skinny matrices (Sec. 6.2.2): N = 40, M powers of 2 and 3
    for M in (2 ** 10, 3 ** 7, 2 ** 13, 3 ** 9, 2 ** 16, 3 ** 11, 2 ** 19, 3 ** 13, 2 ** 22):
        t, full = f"{M}x40", 4 * M * 40
        rec("sgemv_n", t, full, lambda: B.mxb_sgemv(h, B.ROW_MAJOR, B.NO_TRANS, M, 40, 1.0, A, 40, xv, 1, 0.0, yv, 1))
        rec("sgemv_t", t, full, lambda: B.mxb_sgemv(h, B.ROW_MAJOR, B.TRANS, M, 40, 1.0, A, 40, xv, 1, 0.0, yv, 1))
        rec("sger", t, 2 * full, lambda: B.mxb_sger(h, B.ROW_MAJOR, M, 40, 1e-6, xv, 1, yv, 1, A, 40))

    # batches of small matrices in one call: 1 GiB of matrices per case (half for 32 x 32), both orientations
    for n, batch in ((32, 1 << 17), (64, 1 << 16), (128, 1 << 14), (256, 1 << 12), (512, 1 << 10), (1024, 1 << 8), (4096, 1 << 4)):
        for tn, tr in (("n", B.NO_TRANS), ("t", B.TRANS)):
            rec(f"sgemv_{tn}_b", f"{n}x{n} x{batch}", 4 * n * n * batch,
                lambda: B.mxb_sgemv_batched(h, B.ROW_MAJOR, tr, n, n, 1.0, A, n, n * n, xv, 1, n, 0.0, yv, 1, n, batch))

    # a few rows of millions of columns (256 MiB and 1 GiB of matrix; the long vector counts in the bytes)
    for m, n in ((1, 1 << 26), (4, 1 << 24), (16, 1 << 22), (256, 1 << 18), (2, 1 << 27), (4, 1 << 26), (16, 1 << 24), (256, 1 << 20)):
        rec("sgemv_n_w", f"{m}x{n}", 4 * (m * n + n), lambda: B.mxb_sgemv(h, B.ROW_MAJOR, B.NO_TRANS, m, n, 1.0, A, n, y, 1, 0.0, yv, 1))
        rec("sgemv_t_w", f"{m}x{n}", 4 * (m * n + n), lambda: B.mxb_sgemv(h, B.ROW_MAJOR, B.TRANS, m, n, 1.0, A, n, xv, 1, 0.0, y, 1))

    def bucket(nb):
        return "small (< 4 MiB)" if nb < (4 << 20) else "medium (< 256 MiB)" if nb < (256 << 20) else "large"

    print("| routine | shape | MiB | us, one call | GB/s | % of 8 TB/s | us per call, 20 calls in a replayed graph | GB/s |")
    print("|---|---|---|---|---|---|---|---|")
    for name, shape, nb, us, gus in rows:
        print(f"| {name} | {shape} | {nb / 2**20:.2f} | {us:.1f} | {nb / us / 1e3:.0f} | {nb / us / 1e3 / 80:.1f} | "
              + (f"{gus:.1f} | {nb / gus / 1e3:.0f} |" if gus else "| |"))
    print()
    print("| routine | bucket | cases | geometric mean GB/s, one call | in a replayed graph |")
    print("|---|---|---|---|---|")
    label = lambda name, shape: name + (" (N=40)" if shape.endswith("x40") else "")
    keys = []
    for name, shape, nb, us, gus in rows:
        k = (label(name, shape), bucket(nb))
        if k not in keys: keys.append(k)
    for k in keys:
        sel = [(nb, us, gus) for name, shape, nb, us, gus in rows if (label(name, shape), bucket(nb)) == k]
        gm = float(np.exp(np.mean([np.log(nb / us / 1e3) for nb, us, gus in sel])))
        gg = float(np.exp(np.mean([np.log(nb / (gus or us) / 1e3) for nb, us, gus in sel])))
        print(f"| {k[0]} | {k[1]} | {len(sel)} | {gm:.0f} | {gg:.0f} |")


CSRC = os.path.join(ROOT, "paper_2411_07211_amd", "csrc")
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "traffic.json")
# Kernels (demangled-name fragments) behind the calls whose HBM traffic is recorded; the calls are
# chosen so that no kernel is shared between two of them within one profiling run.
TRAFFIC_KERNELS = {
    "sgemv_n_16384_b0": ["rowdot_kernel<float, 4, 64, 2, 4, 0, false>"],
    "sgemv_t_16384_b0": ["colacc_kernel<float, 4, 4, 1>", "colacc_combine_kernel<float>"],
    "dgemv_n_16384": ["rowdot_kernel<double, 2, 64, 2, 4, 0, false>"],
    "dgemv_t_16384": ["colacc_kernel<double, 2, 4, 1>", "colacc_combine_kernel<double>"],
    "strmv_un_16384": ["gather_kernel<float>", "rowdot_kernel<float, 4, 64, 2, 4, 1, false>"],
    "ssymv_l_16384": ["trisweep_kernel<float, 4, 2, 16, false, 0, false>", "trisweep_combine_kernel<float, false, 0>"],
    "sger_16384": ["ger_kernel<float, 4>"],
    "saxpy": ["axpy_vec_kernel<float>"],
    "sscal": ["scal_vec_kernel<float>"],
    "sdot": ["reduce_vec_kernel<float, 0, float>", "reduce_final_kernel<float, 0, float>"],
    "probe_copy": ["probe_copy_kernel"],
    "probe_read": ["probe_read_kernel"],
}
TRAFFIC_ONLY = ",".join(TRAFFIC_KERNELS)


def source_hash():
    import hashlib
    h = hashlib.sha256()
    for f in sorted(os.listdir(CSRC)):
        if f.endswith((".hip", ".hpp")):
            h.update(open(os.path.join(CSRC, f), "rb").read())
    return h.hexdigest()


def measured_traffic():
    """HBM bytes per call taken from the rocprofv3 counter runs recorded in profiles/traffic.json;
    empty when the kernel sources have changed since those counters were collected."""
    try:
        rec = json.load(open(TRAFFIC_JSON))
        if source_hash() != rec["source_sha256"]:
            return {}
        return {k: v["hbm_bytes"] for k, v in rec["calls"].items()}
    except (OSError, KeyError, ValueError):
        return {}


def write_traffic(fetch_dir, write_dir):
    """Turns two rocprofv3 --pmc runs of `bench.py --only TRAFFIC_ONLY` (FETCH_SIZE in fetch_dir,
    WRITE_SIZE in write_dir; both counters are KiB per dispatch) into profiles/traffic.json.  Each
    counter is scaled by what it reports for mxb_probe_copy of 1 GiB, whose true traffic is known."""
    import csv
    import glob

    def means(d, counter):
        acc = {}
        for f in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
            for r in csv.DictReader(open(f)):
                if r["Counter_Name"] == counter:
                    acc.setdefault(r["Kernel_Name"], []).append(float(r["Counter_Value"]))
        return {k: sum(v) / len(v) for k, v in acc.items()}

    fetch, write = means(fetch_dir, "FETCH_SIZE"), means(write_dir, "WRITE_SIZE")

    def find(table, frag):
        hits = [v for k, v in table.items() if frag in k]
        if len(hits) != 1:
            raise SystemExit(f"bench.py: {len(hits)} kernels match '{frag}' in the counter run")
        return hits[0]

    copy_kib = 16384 * 16384 * 4 / 1024.0          # probe_copy moves this much each way
    fscale = copy_kib / find(fetch, "probe_copy_kernel")
    wscale = copy_kib / find(write, "probe_copy_kernel")
    calls = {}
    for call, frags in TRAFFIC_KERNELS.items():
        ks, total = {}, 0.0
        for frag in frags:
            f, w = find(fetch, frag), find(write, frag)
            ks[frag] = {"FETCH_SIZE_KiB": round(f, 1), "WRITE_SIZE_KiB": round(w, 1)}
            total += (f * fscale + w * wscale) * 1024.0
        calls[call] = {"kernels": ks, "hbm_bytes": int(round(total))}
    rec = {
        "note": "HBM traffic per call from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch, mean over the "
                "dispatches of the run), each scaled by what the same counter reports for mxb_probe_copy of 1 GiB "
                "(1048576 KiB each way).  Valid only for the kernel sources whose hash is recorded here; bench.py "
                "reports null otherwise.  Written by `python bench.py --traffic-from FETCH_DIR WRITE_DIR`.",
        "source_sha256": source_hash(), "fetch_scale": round(fscale, 6), "write_scale": round(wscale, 6), "calls": calls,
    }
    json.dump(rec, open(TRAFFIC_JSON, "w"), indent=1)
    for call, v in calls.items():
        print(f"{call:24s} {v['hbm_bytes']:>14d} B")


def main():
    args = parse()
    if args.traffic_list:
        print(TRAFFIC_ONLY)
        return
    if args.traffic_from:
        write_traffic(*args.traffic_from)
        return
    if args.gpus != 1:
        print(f"bench.py: this library runs on one GPU only (got --gpus {args.gpus}); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2411_07211_amd import blas as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    ctx = B.Context("cuda:0", workspace_bytes=256 << 20)
    if args.sweep:
        sweep(B, ctx, torch)
        return
    suite = Suite(B, ctx, torch, scale=args.scale)
    calls = suite.calls
    if args.list:
        for name, fam, _, nb, _ in calls + suite.extra:
            print(f"{name:32s} {fam:8s} {nb / GiB:8.3f} GiB")
        return
    if args.only:
        want = set(args.only.split(","))
        calls = [c for c in calls + suite.extra if c[0] in want or c[1] in want]
        if not calls:
            print("bench.py: --only matched nothing (see --list)", file=sys.stderr)
            sys.exit(2)

    def step(s, events=None):
        for k, (name, fam, fn, nb, pre) in enumerate(calls):
            if pre is not None:
                pre()
            if events is not None:
                events[k][0].record()
            st = fn(s)
            if events is not None:
                events[k][1].record()
            if st != 0:
                raise RuntimeError(f"{name} returned status {st}")

    for w in range(args.warmup):
        step(w)
    torch.cuda.synchronize()

    K = args.steps
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in calls] for _ in range(K)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(K):
        step(args.warmup + s, ev[s])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / K
    step_bytes = sum(c[3] for c in calls)
    per = {}
    for k, (name, fam, fn, nb, pre) in enumerate(calls):
        ts = sorted(ev[s][k][0].elapsed_time(ev[s][k][1]) for s in range(K))    # ms
        avg = sum(ts) / len(ts)
        per[name] = {"bytes": nb, "us_avg": round(avg * 1e3, 2), "us_min": round(ts[0] * 1e3, 2),
                     "us_med": round(ts[len(ts) // 2] * 1e3, 2), "GBps": round(nb / (avg * 1e-3) / 1e9, 1),
                     "frac_of_8TBps": round(nb / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}

    # what this machine reaches with the plainest kernels (a read-only and a copy kernel over 1 GiB), beside the 8 TB/s peak
    ceiling = {}
    if not args.only:
        for name, fam, fn, nb, pre in suite.extra:
            if fam != "probe":
                continue
            pe = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
            for w in range(3):
                fn(w)
            for i, (a, b) in enumerate(pe):
                a.record(); st = fn(i); b.record()
                if st != 0:
                    raise RuntimeError(f"{name} returned status {st}")
            torch.cuda.synchronize()
            avg = sum(a.elapsed_time(b) for a, b in pe) / len(pe)
            ceiling[name + "_GBps"] = round(nb / (avg * 1e-3) / 1e9, 1)

    NS = 16384 // (args.scale if args.scale <= 16 else 16)
    head = f"sgemv_n_{NS}_b0"
    traffic = measured_traffic()
    for name in per:
        per[name]["hbm_traffic_bytes"] = traffic.get(name)
    roofline = None
    if head in per:
        p = per[head]
        roofline = {"bound": "hbm", "kernel": "rowdot_kernel<float,4,64,2,4,general> (sgemv N 16384x16384, beta=0)",
                    "achieved": p["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(p["GBps"] / HBM_PEAK_GBS, 4),
                    "traffic": traffic.get(head), "algorithmic_bytes_per_launch": p["bytes"], "avg_launch_us": p["us_avg"]}
        if "probe_read_GBps" in ceiling:
            roofline["frac_of_measured_read_ceiling"] = round(p["GBps"] / ceiling["probe_read_GBps"], 4)

    # the figures the headline metric names, one by one: gemv N/T at 16384^2 against the peak, level-1 GB/s
    headline = {}
    for name in (f"sgemv_n_{NS}_b0", f"sgemv_t_{NS}_b0", f"dgemv_n_{NS}", f"dgemv_t_{NS}", "saxpy", "daxpy", "sscal", "sdot", "ddot",
                 "sasum", "snrm2", "saxpy_strided", "daxpy_strided", "sscal_strided", "sdot_strided", "ddot_strided", "sasum_strided",
                 "snrm2_strided"):
        if name in per:
            headline[name] = {"GBps": per[name]["GBps"], "frac_of_8TBps": per[name]["frac_of_8TBps"]}

    out = {
        "metric": "achieved HBM GB/s (% of peak) for sgemv/dgemv N,T at 16384^2; level-1 GB/s: algorithmic bytes / time over "
                  "one pass of the whole level-1/level-2 suite (`headline` lists the named figures one by one)",
        "value": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32+f64", "data": "synthetic",
        "config": {"workload": "level-1 n=2^28 (s,d; unit and incx=2/incy=3) + sgemv N,T 16384^2 and 1048576x256 (beta 0,1,0.5) "
                               "+ dgemv N,T 16384^2 lda=16392 + strmv x4, ssymv, sger at 16384 + sgemv 1024^2"
                               + ("" if args.scale == 1 else f" [SCALED DOWN by {args.scale}: not the benchmark]")
                               + ("" if not args.only else f" [ONLY {args.only}]"),
                   "step_algorithmic_GiB": round(step_bytes / GiB, 3)},
        "roofline": roofline,
        "headline": headline,
        "stream_ceiling": ceiling or None,
        "kernels": per,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(torch)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
