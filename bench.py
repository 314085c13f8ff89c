#!/usr/bin/env python3
"""Benchmark of the BLAS level-1 / level-2 hot path on one MI355X.

A *step* is one pass over the whole routine family at full size on seeded synthetic data that is
already resident in HBM: the level-1 suite at n = 2^28 (unit stride and incx=2/incy=3), sgemv N/T
at 16384^2 and 1048576x256 with beta in {0, 1, 0.5}, dgemv N/T at 16384^2 with lda = 16392,
strmv (4 variants), ssymv and sger at 16384, plus the small 1024^2 sgemv.  Every routine is
bracketed by events on the stream it is launched on; those give the per-routine GB/s (algorithmic
bytes / median time).  `value` is the headline metric: the lowest of the four gemv figures at
16384^2 (sgemv N, T with beta = 0; dgemv N, T); `step_GBps` is the algorithmic bytes of a whole
step divided by its wall time.  The `roofline` object is for the row-dot kernel behind sgemv N at
16384^2.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--only NAME[,NAME...]] [--no-cpu-baseline]
    python bench.py --sweep                      # size sweep (profiles/size_sweep.md)
    python bench.py --traffic-from F_DIR W_DIR   # rocprofv3 --pmc output -> profiles/traffic.json
    python bench.py --profile-from DIR [DIR...]  # rocprofv3 --kernel-trace --stats output -> profiles/*_rocprofv3.md

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
    ap.add_argument("--extra-list", action="store_true", help="print the --only list of the calls outside the step that the profiles cover")
    ap.add_argument("--profile-from", nargs="+", metavar="DIR",
                    help="no GPU work: parse rocprofv3 --kernel-trace --stats output folders (csv) of `bench.py` and of "
                         "`bench.py --only $(bench.py --extra-list)` into profiles/*_rocprofv3.md (needs profiles/traffic.json)")
    ap.add_argument("--cpu-baseline-reps", type=int, default=1, help="time every oracle routine this often and keep the best")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the step: time every routine over a sweep of sizes (small, medium, large buckets, "
                         "skinny N = 40 shapes) and print a markdown table with the geometric mean per bucket")
    ap.add_argument("--scan", action="store_true",
                    help="instead of the step: time every routine (gemv N/T, ger and gemv_batched over a grid of shapes of 1 to millions of rows "
                         "and columns, up to 192 MiB) in a replayed graph and list the shapes that take more than 1.8 times "
                         "2.5 us + bytes / 5 TB/s, i.e. the shapes no kernel serves well")
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
        self.hw = {}               # strided calls: least bytes the hardware moves (whole lines)
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
                if tag:
                    # what the hardware has to move at least, whole lines: every line of the strided
                    # operands is read, and written where the routine writes
                    self.hw.update({f"{p}axpy{tag}": (ix + 2 * iy) * n1 * e, f"{p}dot{tag}": (ix + iy) * n1 * e,
                                    f"sscal{tag}": 2 * ix * n1 * 4, f"sasum{tag}": ix * n1 * 4, f"snrm2{tag}": ix * n1 * 4})
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
        xdt = xd.clone()
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
        self.keep = (A32, A64, xs, ys, xd, yd, x0, xt, xdt)

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
            # the same matrices with rows that begin on 128-byte boundaries (lda = n): the odd pitch of 16392 costs the sweep 8-12 %
            (f"dsymv_u_{NS}_dense", "symv", lambda s: B.mxb_dsymv(h, B.ROW_MAJOR, B.UPPER, NS, 0.52, nextA(A64), NS, xd, 1, 0.49, yd, 1),
             8 * (tri + 3 * NS), None),
            (f"dtrmv_lt_{NS}_dense", "trmv_t", lambda s: B.mxb_dtrmv(h, B.ROW_MAJOR, B.LOWER, B.TRANS, B.NON_UNIT, NS, nextA(A64), NS, xdt, 1),
             8 * (tri + 2 * NS), lambda: xdt.copy_(xd)),
            # trsv: unit diagonal over small off-diagonal elements (a random triangle is exponentially ill conditioned)
            (f"strsv_ln_{NS}", "trsv", lambda s: B.mxb_strsv(h, B.ROW_MAJOR, B.LOWER, B.NO_TRANS, B.UNIT, NS, self.small(), NS, xt, 1),
             4 * (tri - NS + 2 * NS), reset),
            (f"strsv_lt_{NS}", "trsv", lambda s: B.mxb_strsv(h, B.ROW_MAJOR, B.LOWER, B.TRANS, B.UNIT, NS, self.small(), NS, xt, 1),
             4 * (tri - NS + 2 * NS), reset),
            (f"dtrsv_ln_{NS}_dense", "trsv", lambda s: B.mxb_dtrsv(h, B.ROW_MAJOR, B.LOWER, B.NO_TRANS, B.UNIT, NS, self.small(f64), NS, xdt, 1),
             8 * (tri - NS + 2 * NS), lambda: xdt.copy_(xd)),
            (f"dtrsv_lt_{NS}_dense", "trsv", lambda s: B.mxb_dtrsv(h, B.ROW_MAJOR, B.LOWER, B.TRANS, B.UNIT, NS, self.small(f64), NS, xdt, 1),
             8 * (tri - NS + 2 * NS), lambda: xdt.copy_(xd)),
        ]
        self._small = {}
        self._small_from = {f32: A32[0], f64: A64[0][:NS * NS]}

    def small(self, dtype=None):
        """A 16384^2 matrix of elements below 1e-4, made on first use (only the trsv extras want it)."""
        dtype = dtype or next(iter(self._small_from))
        if dtype not in self._small:
            self._small[dtype] = self._small_from[dtype] * 1e-4
        return self._small[dtype]

    def add(self, name, family, fn, nbytes, pre=None):
        self.calls.append((name, family, fn, int(nbytes), pre))


def cpu_baseline(reps=1):
    """The oracle, as it stands, timed single-threaded on this host on the benchmark's own
    configurations: the level-1 suite at n = 2^28 (unit stride and incx=2/incy=3, gaps NaN),
    sgemv N/T at 16384^2 and 1048576x256 (one beta of the three: the oracle's time does not depend
    on it), dgemv N/T at 16384^2 with lda = 16392 and NaN padding, the four strmv variants with
    the other triangle NaN, ssymv lower, sger, and the 1024^2 sgemv; each routine `reps` times,
    best kept.  Values are a tiled block of uniform numbers: they do not matter for the timing."""
    import oracle as O
    n1, ns, mt, nt = 1 << 28, 16384, 1 << 20, 256
    total = 0
    t_total = 0.0
    block = np.random.default_rng(1).random(1 << 22) * 2 - 1

    def filled(n, dt):
        out = np.empty(n, dt)
        src = block.astype(dt)
        for k in range(0, n, src.size):
            out[k:k + src.size] = src[:min(src.size, n - k)]
        return out

    def gaps_nan(a, inc):
        v = a.reshape(-1, inc)
        v[:, 1:] = np.nan
        return a

    def timed(fn, nbytes):
        nonlocal total, t_total
        best = None
        for _ in range(max(reps, 1)):
            t0 = time.perf_counter(); fn(); t = time.perf_counter() - t0
            best = t if best is None or t < best else best
        t_total += best
        total += nbytes

    for dt, e in ((np.float32, 4), (np.float64, 8)):
        x, y = filled(n1, dt), filled(n1, dt)
        xs, ys = gaps_nan(filled(2 * n1, dt), 2), gaps_nan(filled(3 * n1, dt), 3)
        for xx, ix, yy, iy in ((x, 1, y, 1), (xs, 2, ys, 3)):
            timed(lambda: O.axpy(n1, dt(-0.75), xx, ix, yy, iy), 3 * n1 * e)
            timed(lambda: O.dot(n1, xx, ix, yy, iy), 2 * n1 * e)
            if dt == np.float32:
                timed(lambda: O.scal(n1, dt(1.25), xx, ix), 2 * n1 * e)
                timed(lambda: O.asum(n1, xx, ix), n1 * e)
                timed(lambda: O.nrm2(n1, xx, ix), n1 * e)
        del x, y, xs, ys
    f = np.float32
    A = filled(ns * ns, f)
    xv, yv = filled(mt, f), filled(mt, f)
    for trans in (O.NO_TRANS, O.TRANS):
        timed(lambda: O.gemv(O.ROW_MAJOR, trans, ns, ns, f(1), A, ns, xv, 1, f(0.5), yv, 1), 4 * (ns * ns + 3 * ns))
        timed(lambda: O.gemv(O.ROW_MAJOR, trans, mt, nt, f(1), A, nt, xv, 1, f(0.5), yv, 1),
              4 * (mt * nt + mt + nt + (mt if trans == O.NO_TRANS else nt)))
    timed(lambda: O.gemv(O.ROW_MAJOR, O.NO_TRANS, 1024, 1024, f(1.5), A, 1024, xv, 1, f(0.5), yv, 1), 4 * (1024 * 1024 + 3 * 1024))
    lda = ns + 8
    Ad = filled(ns * lda, np.float64).reshape(ns, lda)
    Ad *= 1.0 / 128
    Ad[:, ns:] = np.nan
    Ad = Ad.ravel()
    xd, yd = filled(ns, np.float64), np.full(ns, np.nan)
    for trans in (O.NO_TRANS, O.TRANS):
        timed(lambda: O.gemv(O.ROW_MAJOR, trans, ns, ns, 2.0, Ad, lda, xd, 1, 0.0, yd, 1), 8 * (ns * ns + 2 * ns))
    del Ad
    tri = ns * (ns + 1) // 2
    A2 = A.reshape(ns, ns)
    below = np.tri(ns, k=-1, dtype=bool)
    for uplo in (O.UPPER, O.LOWER):
        T = A2.copy()
        T[below if uplo == O.UPPER else below.T] = np.nan      # the other triangle is never read
        for diag in (O.NON_UNIT, O.UNIT):
            if diag == O.UNIT:
                np.fill_diagonal(T, np.nan)
            xt = xv[:ns].copy()
            timed(lambda: O.trmv(O.ROW_MAJOR, uplo, O.NO_TRANS, diag, ns, T.ravel(), ns, xt, 1),
                  4 * ((tri if diag == O.NON_UNIT else tri - ns) + 2 * ns))
        if uplo == O.LOWER:
            np.fill_diagonal(T, np.diag(A2))
            timed(lambda: O.symv(O.ROW_MAJOR, O.LOWER, ns, f(0.52), T.ravel(), ns, xv, 1, f(0.49), yv, 1), 4 * (tri + 3 * ns))
        del T
    timed(lambda: O.ger(O.ROW_MAJOR, ns, ns, f(1e-3), xv, 1, yv, 1, A, ns), 4 * (2 * ns * ns + 2 * ns))
    return {
        "value": round(total / t_total / 1e9, 4), "unit": "GB/s", "cores": 1, "host_cores": os.cpu_count(), "kind": "oracle",
        "sample": "every configuration of the step once: level-1 at n=2^28 (s: axpy, scal, dot, asum, nrm2; d: axpy, dot; unit stride and "
                  "incx=2/incy=3); sgemv N,T 16384^2 and 1048576x256 (beta 0.5 only; the step's other two betas cost the oracle the "
                  "same); sgemv N 1024^2; dgemv N,T 16384^2 lda=16392 with NaN padding; strmv x4 with the other triangle NaN; ssymv "
                  f"lower; sger; single thread of {os.cpu_count()} host cores, gcc -O2, long-double accumulation, best of {max(reps, 1)}; "
                  f"{total / 1e9:.2f} GB algorithmic in {t_total:.1f} s",
    }


def scan(B, ctx, torch):
    """Looks for shapes that fall between the kernels: every combination of the row and column counts
    below, fp32 and fp64, gemv N / T and ger as single calls and gemv_batched at 1 and 64 MiB per
    call, timed as 10 calls in a replayed graph, against a plain model of a call (2.5 us of launch +
    bytes at 5 TB/s).  Prints every case and, at the end, those beyond 1.8 times the model."""
    h = ctx.h

    def replayed(fn, calls=10, reps=5):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            ctx.use_current_stream()
            for _ in range(calls):
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

    bad, every = [], []

    def rec(name, shape, nbytes, us):
        r = us / (2.5 + nbytes / 5e6)
        line = f"{name:10s} {shape:>28s} {nbytes / 2**20:9.2f} MiB {us:9.2f} us  {r:6.2f} x model"
        print(line, flush=True)
        every.append(line)
        if r > 1.8: bad.append(line)

    dims = [1, 2, 3, 5, 8, 16, 33, 64, 100, 256, 700, 1024, 3000, 8192, 20000, 65536, 200000, 1 << 20, 3000000, 1 << 23]
    bdims = (1, 3, 8, 16, 40, 64, 100, 256, 700, 2048)
    for dt, T, e in (("s", torch.float32, 4), ("d", torch.float64, 8)):
        A = torch.rand((1 << 28) // e, dtype=T, device=ctx.device); x = torch.rand(1 << 24, dtype=T, device=ctx.device)
        y = torch.rand(1 << 24, dtype=T, device=ctx.device)
        gemv, ger, gemvb = getattr(B, f"mxb_{dt}gemv"), getattr(B, f"mxb_{dt}ger"), getattr(B, f"mxb_{dt}gemv_batched")
        for m in dims:
            for n in dims:
                nb = m * n * e
                if nb > (192 << 20) or nb < 4096: continue
                rec(dt + "gemv_n", f"{m}x{n}", nb + (n + 2 * m) * e, replayed(lambda: gemv(h, B.ROW_MAJOR, B.NO_TRANS, m, n, 1.0, A, n, x, 1, 0.5, y, 1)))
                rec(dt + "gemv_t", f"{m}x{n}", nb + (m + 2 * n) * e, replayed(lambda: gemv(h, B.ROW_MAJOR, B.TRANS, m, n, 1.0, A, n, x, 1, 0.5, y, 1)))
                rec(dt + "ger", f"{m}x{n}", 2 * nb + (m + n) * e, replayed(lambda: ger(h, B.ROW_MAJOR, m, n, 1e-6, x, 1, y, 1, A, n)))
        for total in (1 << 20, 64 << 20):
            for m in bdims:
                for n in bdims:
                    batch = total // (m * n * e)
                    if batch < 2 or batch > 1 << 22 or max(m, n) * batch > 1 << 24: continue
                    for nm, tr in (("n", B.NO_TRANS), ("t", B.TRANS)):
                        lx, ly = (n, m) if tr == B.NO_TRANS else (m, n)
                        us = replayed(lambda: gemvb(h, B.ROW_MAJOR, tr, m, n, 1.0, A, n, m * n, x, 1, lx, 0.5, y, 1, ly, batch))
                        rec(f"{dt}gemvb_{nm}", f"{m}x{n} x{batch}", batch * (m * n + lx + 2 * ly) * e, us)
        # level 1 (unit and strided) and the structured level-2 routines over n
        r = torch.zeros(4, dtype=T, device=ctx.device); ri = torch.zeros(2, dtype=torch.int64, device=ctx.device)
        f = lambda nm: getattr(B, f"mxb_{dt}{nm}")
        for n in (100, 4096, 65536, 300000, 1 << 20, 3000001, 1 << 23):
            for inc, tag in ((1, ""), (2, "/inc2")):
                if n * inc > 1 << 24: continue
                rec(f"{dt}axpy{tag}", str(n), 3 * n * e, replayed(lambda: f("axpy")(h, n, 1e-3, x, inc, y, inc)))
                rec(f"{dt}scal{tag}", str(n), 2 * n * e, replayed(lambda: f("scal")(h, n, 1.0, x, inc)))
                rec(f"{dt}dot{tag}", str(n), 2 * n * e, replayed(lambda: f("dot")(h, n, x, inc, y, inc, r)))
                rec(f"{dt}nrm2{tag}", str(n), n * e, replayed(lambda: f("nrm2")(h, n, x, inc, r)))
                rec(f"{dt}swap{tag}", str(n), 4 * n * e, replayed(lambda: f("swap")(h, n, x, inc, y, inc)))
                rec(f"i{dt}amax{tag}", str(n), n * e, replayed(lambda: getattr(B, f"mxb_i{dt}amax")(h, n, x, inc, ri)))
        A.mul_(1e-4)       # small off-diagonal elements: trmv repeated on one vector stays finite
        for n in (33, 100, 300, 700, 1500, 2500, 3500, 5000):
            tri = n * (n + 1) // 2 * e
            for up, ut in ((B.UPPER, "u"), (B.LOWER, "l")):
                rec(f"{dt}symv_{ut}", str(n), tri, replayed(lambda: f("symv")(h, B.ROW_MAJOR, up, n, 0.5, A, n, x, 1, 0.5, y, 1)))
                rec(f"{dt}syr_{ut}", str(n), 2 * tri, replayed(lambda: f("syr")(h, B.ROW_MAJOR, up, n, 1e-9, x, 1, A, n)))
                rec(f"{dt}syr2_{ut}", str(n), 2 * tri, replayed(lambda: f("syr2")(h, B.ROW_MAJOR, up, n, 1e-9, x, 1, y, 1, A, n)))
                for tr, tt in ((B.NO_TRANS, "n"), (B.TRANS, "t")):
                    rec(f"{dt}trmv_{ut}{tt}", str(n), tri, replayed(lambda: f("trmv")(h, B.ROW_MAJOR, up, tr, B.UNIT, n, A, n, x, 1)))
        del A, x, y
    # the summary kept in profiles/shape_scan.md
    import statistics
    ratio = lambda line: float(line.split()[-3])
    fam = {}
    for line in every: fam.setdefault(line.split()[0], []).append(ratio(line))
    print("# Shape scan: every routine over a grid of shapes against a plain model of a call\n")
    print("Command (one MI355X, committed files only): `python bench.py --scan | sed -n '/^# Shape scan/,$p' > profiles/shape_scan.md`.\n"
          "Every combination of 20 row and column counts from 1 to 8388608 (up to 192 MiB per matrix), single and double precision,\n"
          "for gemv N / T and ger; gemv_batched over 10 x 10 problem shapes at 1 and 64 MiB per call; the level-1 routines at 7\n"
          "lengths, unit increment and increment 2; symv, syr, syr2 and trmv at 8 orders, both triangles.  10 calls in a replayed\n"
          "HIP graph, median of 5 replays; the model of a call is 2.5 us + bytes / 5 TB/s.  A call that needs two kernels on\n"
          "little data (reductions, trmv, the transposed product of a tall matrix) sits at 2-3 times the model.\n")
    print("| routine | cases | median ratio to the model | worst | cases beyond 1.8 |\n|---|---|---|---|---|")
    for k, v in fam.items():
        print(f"| {k} | {len(v)} | {statistics.median(v):.2f} | {max(v):.2f} | {sum(1 for r in v if r > 1.8)} |")
    print("\n## Cases beyond 2.5 times the model\n\n```")
    for line in bad:
        if ratio(line) > 2.5: print(line)
    print("```")


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
    ri = torch.zeros(1, dtype=torch.int64, device=dev)
    for e in range(10, 29, 2):
        n = 1 << e
        for n_ in (n, n - 3 if e < 28 else n):
            t = f"n={n_}"
            rec("saxpy", t, 12 * n_, lambda: B.mxb_saxpy(h, n_, -0.75, x, 1, y, 1))
            rec("sscal", t, 8 * n_, lambda: B.mxb_sscal(h, n_, 1.0, x, 1))
            rec("sdot", t, 8 * n_, lambda: B.mxb_sdot(h, n_, x, 1, y, 1, r))
            rec("sasum", t, 4 * n_, lambda: B.mxb_sasum(h, n_, x, 1, r))
            rec("snrm2", t, 4 * n_, lambda: B.mxb_snrm2(h, n_, x, 1, r))
            rec("isamax", t, 4 * n_, lambda: B.mxb_isamax(h, n_, x, 1, ri))
            rec("scopy", t, 8 * n_, lambda: B.mxb_scopy(h, n_, x, 1, y, 1))
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
    # the other variants of the structured routines (upper / lower, unit diagonal, transposed) ...
    for n in (1024, 4096, 16384):
        t, tri = f"{n}x{n}", 4 * (n * (n + 1) // 2)
        rec("strmv_uu", t, tri - 4 * n, lambda: B.mxb_strmv(h, B.ROW_MAJOR, B.UPPER, B.NO_TRANS, B.UNIT, n, A, n, xt, 1), reset)
        rec("strmv_ln", t, tri, lambda: B.mxb_strmv(h, B.ROW_MAJOR, B.LOWER, B.NO_TRANS, B.NON_UNIT, n, A, n, xt, 1), reset)
        rec("strmv_ut", t, tri, lambda: B.mxb_strmv(h, B.ROW_MAJOR, B.UPPER, B.TRANS, B.NON_UNIT, n, A, n, xt, 1), reset)
        rec("strmv_ltu", t, tri - 4 * n, lambda: B.mxb_strmv(h, B.ROW_MAJOR, B.LOWER, B.TRANS, B.UNIT, n, A, n, xt, 1), reset)
        rec("ssymv_u", t, tri, lambda: B.mxb_ssymv(h, B.ROW_MAJOR, B.UPPER, n, 0.5, A, n, xv, 1, 0.5, yv, 1))
        rec("ssyr_u", t, 2 * tri, lambda: B.mxb_ssyr(h, B.ROW_MAJOR, B.UPPER, n, 1e-6, xv, 1, A, n))
        rec("ssyr2_l", t, 2 * tri, lambda: B.mxb_ssyr2(h, B.ROW_MAJOR, B.LOWER, n, 1e-6, xv, 1, yv, 1, A, n))
    # ... the level-2 routines with strided vectors (incx = 2, incy = 3) ...
    xs3 = torch.rand(3 * NS, dtype=f32, device=dev); xt3 = xs3.clone()
    reset3 = lambda: xt3.copy_(xs3)
    for n in (1024, 4096, 16384):
        t, full, tri = f"{n}x{n}", 4 * n * n, 4 * (n * (n + 1) // 2)
        rec("sgemv_n (inc 2,3)", t, full, lambda: B.mxb_sgemv(h, B.ROW_MAJOR, B.NO_TRANS, n, n, 1.0, A, n, xv, 2, 0.5, yv, 3))
        rec("sgemv_t (inc 2,3)", t, full, lambda: B.mxb_sgemv(h, B.ROW_MAJOR, B.TRANS, n, n, 1.0, A, n, xv, 2, 0.5, yv, 3))
        rec("ssymv_l (inc 2,3)", t, tri, lambda: B.mxb_ssymv(h, B.ROW_MAJOR, B.LOWER, n, 0.5, A, n, xv, 2, 0.5, yv, 3))
        rec("sger (inc 2,3)", t, 2 * full, lambda: B.mxb_sger(h, B.ROW_MAJOR, n, n, 1e-6, xv, 2, yv, 3, A, n))
        rec("strmv_un (inc 2,3)", t, tri, lambda: B.mxb_strmv(h, B.ROW_MAJOR, B.UPPER, B.NO_TRANS, B.NON_UNIT, n, A, n, xt3, 3), reset3)
        rec("strmv_lt (inc 2,3)", t, tri, lambda: B.mxb_strmv(h, B.ROW_MAJOR, B.LOWER, B.TRANS, B.NON_UNIT, n, A, n, xt3, 3), reset3)
    # ... and double precision (the 2^28 floats hold a 8192 x 16384 matrix of doubles)
    f64 = torch.float64
    Ad, xd, yd = A.view(f64), xv.view(f64), yv.view(f64)
    rd = torch.zeros(1, dtype=f64, device=dev)
    xd0 = torch.rand(NS, dtype=f64, device=dev); xdt = xd0.clone()
    resetd = lambda: xdt.copy_(xd0)
    for e in (12, 20, 26):
        n_ = 1 << e
        t = f"n={n_}"
        rec("daxpy", t, 24 * n_, lambda: B.mxb_daxpy(h, n_, -0.75, Ad, 1, Ad[n_:], 1))
        rec("dscal", t, 16 * n_, lambda: B.mxb_dscal(h, n_, 1.0, Ad, 1))
        rec("ddot", t, 16 * n_, lambda: B.mxb_ddot(h, n_, Ad, 1, Ad[n_:], 1, rd))
        rec("dasum", t, 8 * n_, lambda: B.mxb_dasum(h, n_, Ad, 1, rd))
        rec("dnrm2", t, 8 * n_, lambda: B.mxb_dnrm2(h, n_, Ad, 1, rd))
    for n in (1024, 4096, 11000):
        t, full, tri = f"{n}x{n}", 8 * n * n, 8 * (n * (n + 1) // 2)
        rec("dgemv_n", t, full, lambda: B.mxb_dgemv(h, B.ROW_MAJOR, B.NO_TRANS, n, n, 1.0, Ad, n, xd, 1, 0.0, yd, 1))
        rec("dgemv_t", t, full, lambda: B.mxb_dgemv(h, B.ROW_MAJOR, B.TRANS, n, n, 1.0, Ad, n, xd, 1, 0.0, yd, 1))
        rec("dger", t, 2 * full, lambda: B.mxb_dger(h, B.ROW_MAJOR, n, n, 1e-9, xd, 1, yd, 1, Ad, n))
        rec("dsymv_l", t, tri, lambda: B.mxb_dsymv(h, B.ROW_MAJOR, B.LOWER, n, 0.5, Ad, n, xd, 1, 0.5, yd, 1))
        rec("dsymv_u", t, tri, lambda: B.mxb_dsymv(h, B.ROW_MAJOR, B.UPPER, n, 0.5, Ad, n, xd, 1, 0.5, yd, 1))
        rec("dsyr_l", t, 2 * tri, lambda: B.mxb_dsyr(h, B.ROW_MAJOR, B.LOWER, n, 1e-9, xd, 1, Ad, n))
        rec("dtrmv_un", t, tri, lambda: B.mxb_dtrmv(h, B.ROW_MAJOR, B.UPPER, B.NO_TRANS, B.NON_UNIT, n, Ad, n, xdt, 1), resetd)
        rec("dtrmv_lt", t, tri, lambda: B.mxb_dtrmv(h, B.ROW_MAJOR, B.LOWER, B.TRANS, B.NON_UNIT, n, Ad, n, xdt, 1), resetd)
        rec("dtrmv_uu", t, tri - 8 * n, lambda: B.mxb_dtrmv(h, B.ROW_MAJOR, B.UPPER, B.NO_TRANS, B.UNIT, n, Ad, n, xdt, 1), resetd)
    # trsv wants a well-conditioned triangle: unit diagonal, small off-diagonal elements
    T = torch.rand(NS * NS, dtype=f32, device=dev).mul_(1e-4)
    for n in (256, 1024, 4096, 16384):
        tri = 4 * (n * (n + 1) // 2)
        rec("strsv_lu", f"{n}x{n}", tri, lambda: B.mxb_strsv(h, B.ROW_MAJOR, B.LOWER, B.NO_TRANS, B.UNIT, n, T, n, xt, 1), reset)
        rec("strsv_ltu", f"{n}x{n}", tri, lambda: B.mxb_strsv(h, B.ROW_MAJOR, B.LOWER, B.TRANS, B.UNIT, n, T, n, xt, 1), reset)
    del T
    T = torch.rand(NS * NS, dtype=f64, device=dev).mul_(1e-4)
    for n in (1024, 4096, 16384):
        tri = 8 * (n * (n + 1) // 2)
        rec("dtrsv_lu", f"{n}x{n}", tri, lambda: B.mxb_dtrsv(h, B.ROW_MAJOR, B.LOWER, B.NO_TRANS, B.UNIT, n, T, n, xdt, 1), resetd)
        rec("dtrsv_ltu", f"{n}x{n}", tri, lambda: B.mxb_dtrsv(h, B.ROW_MAJOR, B.LOWER, B.TRANS, B.UNIT, n, T, n, xdt, 1), resetd)
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

    # the whole of profiles/size_sweep.md
    print("# Size sweep: every routine from launch-bound to HBM-bound sizes, single calls and graph replay\n")
    print("Command (one MI355X, committed files only): `python bench.py --sweep > profiles/size_sweep.md`.  Times are medians of 20\n"
          "event-timed calls after 3 warm-ups; the last two columns are the time per call of 20 calls captured into one HIP graph and\n"
          "replayed (only where a single call takes less than 60 us): what the GPU needs once the host's launch cost is out of the\n"
          "way.  Buckets by the bytes a call moves: small < 4 MiB, medium < 256 MiB (fits the last-level cache), large beyond.  s/d:\n"
          "fp32 / fp64; trmv and symv variants: u/l = upper / lower, n/t = not transposed / transposed, a trailing u = unit diagonal;\n"
          "(inc 2,3): the same call with incx = 2, incy = 3 (trmv: incx = 3); N = 40 shapes are the skinny matrices of Sec. 6.2.2 (M\n"
          "powers of 2 and 3); sgemv_n_b / sgemv_t_b are strided batches of square matrices in one call; sgemv_n_w / sgemv_t_w are a few\n"
          "rows of millions of columns (the long vector counts in the bytes); strsv: unit diagonal over small off-diagonal elements;\n"
          "isamax writes an index; scopy moves 2 n elements.\n")
    print("## Geometric means per bucket\n")
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
    print("\n## Every case\n")
    print("| routine | shape | MiB | us, one call | GB/s | % of 8 TB/s | us per call, 20 calls in a replayed graph | GB/s |")
    print("|---|---|---|---|---|---|---|---|")
    for name, shape, nb, us, gus in rows:
        print(f"| {name} | {shape} | {nb / 2**20:.2f} | {us:.1f} | {nb / us / 1e3:.0f} | {nb / us / 1e3 / 80:.1f} | "
              + (f"{gus:.1f} | {nb / gus / 1e3:.0f} |" if gus else "| |"))


CSRC = os.path.join(ROOT, "paper_2411_07211_amd", "csrc")
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "traffic.json")
# Kernels (demangled-name fragments) behind every call of the step and of the extra list, as the
# library dispatches them at these sizes; a second kernel is the combine pass of the first.
NS_, N1_ = 16384, 1 << 28
TRI_ = NS_ * (NS_ + 1) // 2
RED = lambda t, op: [f"reduce_vec_kernel<{t}, {op}, {t}, false>", f"reduce_final_kernel<{t}, {op}, {t}>"]
REDS = lambda t, op: [f"reduce_strided_kernel<{t}, {op}, {t}>", f"reduce_final_kernel<{t}, {op}, {t}>"]
SWEEP = lambda t, v, up, kind: [f"trisweep_kernel<{t}, {v}, 2, 16, {up}, {kind}, false>", f"trisweep_combine_kernel<{t}, {up}, {kind}>"]
CALL_KERNELS = {
    "saxpy": ["axpy_vec_kernel<float, false>"], "daxpy": ["axpy_vec_kernel<double, false>"], "sscal": ["scal_vec_kernel<float, false>"],
    "sdot": RED("float", 0), "ddot": RED("double", 0), "sasum": RED("float", 1), "snrm2": RED("float", 2),
    "saxpy_strided": ["axpy_strided_kernel<float>"], "daxpy_strided": ["axpy_strided_kernel<double>"],
    "sscal_strided": ["scal_strided_kernel<float>"], "sdot_strided": REDS("float", 0), "ddot_strided": REDS("double", 0),
    "sasum_strided": REDS("float", 1), "snrm2_strided": REDS("float", 2),
    "sgemv_n_16384_b0": ["rowdot_kernel<float, 4, 64, 2, 4, 0, false>"],
    "sgemv_t_16384_b0": ["colacc_kernel<float, 4, 4, 1, false>", "colacc_combine_kernel<float>"],
    "sgemv_n_1048576x256_b0": ["skinny_gemv_n_onerow_kernel<float, 4, false, 8, false>"],
    "sgemv_n_1048576x256_b0.5": ["skinny_gemv_n_onerow_kernel<float, 4, true, 8, false>"],
    "sgemv_t_1048576x256_b0": ["colacc_kernel<float, 4, 1, 4, false>", "colacc_combine_kernel<float>"],
    "sgemv_n_1024": ["rowsmall_kernel<float, 4, 1, 4, 1, 0, false>"],
    "dgemv_n_16384": ["rowdot_kernel<double, 2, 64, 2, 4, 0, false>"],
    "dgemv_t_16384": ["colacc_kernel<double, 2, 4, 1, false>", "colacc_combine_kernel<double>"],
    "strmv_un_16384": ["gather_kernel<float>", "rowdot_kernel<float, 4, 64, 2, 4, 1, false>"],
    "strmv_uu_16384": ["gather_kernel<float>", "rowdot_kernel<float, 4, 64, 2, 4, 1, true>"],
    "strmv_ln_16384": ["gather_kernel<float>", "rowdot_kernel<float, 4, 64, 2, 4, 2, false>"],
    "strmv_lu_16384": ["gather_kernel<float>", "rowdot_kernel<float, 4, 64, 2, 4, 2, true>"],
    "ssymv_l_16384": SWEEP("float", 4, "false", 0), "sger_16384": ["ger_kernel<float, 4, false>"],
    "strmv_ut_16384": SWEEP("float", 4, "true", 1), "strmv_lt_16384": SWEEP("float", 4, "false", 1),
    "ssymv_u_16384": SWEEP("float", 4, "true", 0), "dsymv_l_16384": SWEEP("double", 2, "false", 0),
    "dsymv_u_16384_dense": SWEEP("double", 2, "true", 0), "dtrmv_lt_16384_dense": SWEEP("double", 2, "false", 1),
    "strsv_ln_16384": ["trsv_chain_init_kernel", "trsv_chain_kernel<float, true, false, true, true>"],
    "strsv_lt_16384": ["trsv_chain_init_kernel", "trsv_chain_kernel<float, false, true, true, true>"],
    "dtrsv_ln_16384_dense": ["trsv_chain_init_kernel", "trsv_chain_kernel<double, true, false, true, true>"],
    "dtrsv_lt_16384_dense": ["trsv_chain_init_kernel", "trsv_chain_kernel<double, false, true, true, true>"],
    "probe_copy": ["probe_copy_kernel"], "probe_read": ["probe_read_kernel"],
}
# The calls whose HBM traffic is recorded from counters (the dense ones share no kernel with each
# other within the profiling run; the strided reductions share only the tiny final pass).
TRAFFIC_CALLS = ["sgemv_n_16384_b0", "sgemv_t_16384_b0", "dgemv_n_16384", "dgemv_t_16384", "sgemv_n_1048576x256_b0", "strmv_un_16384",
                 "ssymv_l_16384", "sger_16384", "saxpy", "sscal", "sdot", "saxpy_strided", "sscal_strided", "sdot_strided",
                 "probe_copy", "probe_read"]
TRAFFIC_KERNELS = {c: CALL_KERNELS[c] for c in TRAFFIC_CALLS}
TRAFFIC_ONLY = ",".join(TRAFFIC_KERNELS)
EXTRA_ONLY = "strmv_ut_16384,strmv_lt_16384,ssymv_u_16384,dsymv_l_16384,dsymv_u_16384_dense,dtrmv_lt_16384_dense,strsv_ln_16384,strsv_lt_16384,dtrsv_ln_16384_dense,dtrsv_lt_16384_dense,probe_copy,probe_read"
# (title of the summary, file, [(row label, call, algorithmic bytes)])
PROFILE_TABLES = [
    ("gemv at 16384 x 16384 (fp32; fp64 with lda = 16392), 1048576 x 256, 1024 x 1024, and the bandwidth probes", "gemv_16384_rocprofv3.md", [
        ("sgemv N 16384^2 (beta 0, 1, 0.5: one kernel)", "sgemv_n_16384_b0", 4 * (NS_ * NS_ + 2 * NS_)),
        ("sgemv T 16384^2 (beta 0, 1, 0.5: one kernel)", "sgemv_t_16384_b0", 4 * (NS_ * NS_ + 2 * NS_)),
        ("dgemv N 16384^2 lda 16392", "dgemv_n_16384", 8 * (NS_ * NS_ + 2 * NS_)),
        ("dgemv T 16384^2 lda 16392", "dgemv_t_16384", 8 * (NS_ * NS_ + 2 * NS_)),
        ("sgemv N 1048576x256 beta 0", "sgemv_n_1048576x256_b0", 4 * ((1 << 20) * 256 + 256 + (1 << 20))),
        ("sgemv N 1048576x256 beta 1, 0.5", "sgemv_n_1048576x256_b0.5", 4 * ((1 << 20) * 256 + 256 + 2 * (1 << 20))),
        ("sgemv T 1048576x256", "sgemv_t_1048576x256_b0", 4 * ((1 << 20) * 256 + 256 + (1 << 20))),
        ("sgemv N 1024^2 (cache-resident, launch-bound)", "sgemv_n_1024", 4 * (1024 * 1024 + 3 * 1024)),
        ("probe_read 1 GiB", "probe_read", NS_ * NS_ * 4), ("probe_copy 1 GiB", "probe_copy", 2 * NS_ * NS_ * 4)]),
    ("trmv, symv, ger and trsv at n = 16384 (fp32; dsymv, dtrmv and dtrsv with lda = 16392 and 16384)", "triangular_16384_rocprofv3.md", [
        ("strmv upper N non-unit", "strmv_un_16384", 4 * (TRI_ + 2 * NS_)), ("strmv upper N unit", "strmv_uu_16384", 4 * (TRI_ + NS_)),
        ("strmv lower N non-unit", "strmv_ln_16384", 4 * (TRI_ + 2 * NS_)), ("strmv lower N unit", "strmv_lu_16384", 4 * (TRI_ + NS_)),
        ("strmv upper T non-unit", "strmv_ut_16384", 4 * (TRI_ + 2 * NS_)), ("strmv lower T non-unit", "strmv_lt_16384", 4 * (TRI_ + 2 * NS_)),
        ("ssymv lower", "ssymv_l_16384", 4 * (TRI_ + 3 * NS_)), ("ssymv upper", "ssymv_u_16384", 4 * (TRI_ + 3 * NS_)),
        ("dsymv lower lda 16392", "dsymv_l_16384", 8 * (TRI_ + 3 * NS_)), ("dsymv upper lda 16384", "dsymv_u_16384_dense", 8 * (TRI_ + 3 * NS_)),
        ("dtrmv lower T non-unit lda 16384", "dtrmv_lt_16384_dense", 8 * (TRI_ + 2 * NS_)), ("sger 16384^2", "sger_16384", 4 * (2 * NS_ * NS_ + 2 * NS_)),
        ("strsv lower N unit (latency-bound chain)", "strsv_ln_16384", 4 * (TRI_ + NS_)),
        ("strsv lower T unit (latency-bound chain)", "strsv_lt_16384", 4 * (TRI_ + NS_)),
        ("dtrsv lower N unit lda 16384 (latency-bound chain)", "dtrsv_ln_16384_dense", 8 * (TRI_ + NS_)),
        ("dtrsv lower T unit lda 16384 (latency-bound chain)", "dtrsv_lt_16384_dense", 8 * (TRI_ + NS_))]),
    ("level-1 routines at n = 2^28 (unit stride and incx = 2 / incy = 3)", "level1_n2p28_rocprofv3.md", [
        ("saxpy", "saxpy", 3 * N1_ * 4), ("daxpy", "daxpy", 3 * N1_ * 8), ("sscal", "sscal", 2 * N1_ * 4), ("sdot", "sdot", 2 * N1_ * 4),
        ("ddot", "ddot", 2 * N1_ * 8), ("sasum", "sasum", N1_ * 4), ("snrm2", "snrm2", N1_ * 4),
        ("saxpy incx=2 incy=3 (stride ceiling 37.5 %)", "saxpy_strided", 3 * N1_ * 4),
        ("daxpy incx=2 incy=3 (37.5 %)", "daxpy_strided", 3 * N1_ * 8), ("sscal incx=2 (50 %)", "sscal_strided", 2 * N1_ * 4),
        ("sdot incx=2 incy=3 (40 %)", "sdot_strided", 2 * N1_ * 4), ("ddot incx=2 incy=3 (40 %)", "ddot_strided", 2 * N1_ * 8),
        ("sasum incx=2 (50 %)", "sasum_strided", N1_ * 4), ("snrm2 incx=2 (50 %)", "snrm2_strided", N1_ * 4)]),
]


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


def write_profiles(dirs):
    """Turns rocprofv3 --kernel-trace --stats output (csv) of this benchmark into the three
    summaries under profiles/: per call the kernels it launches (CALL_KERNELS), their average and
    minimum durations, GB/s against the 8 TB/s peak and, where counters were taken, HBM bytes."""
    import csv
    import glob
    acc = {}          # kernel name -> [calls, total ns, min ns]
    for d in dirs:
        for f in glob.glob(os.path.join(d, "**", "*kernel_stats.csv"), recursive=True):
            for r in csv.DictReader(open(f)):
                e = acc.setdefault(r["Name"], [0, 0.0, float("inf")])
                e[0] += int(r["Calls"]); e[1] += float(r["TotalDurationNs"]); e[2] = min(e[2], float(r["MinNs"]))

    def find(frag):
        hits = [v for k, v in acc.items() if frag + "(" in k or k.endswith(frag) or frag + " [" in k]
        return hits[0] if len(hits) == 1 else None

    try:
        T = json.load(open(TRAFFIC_JSON))
    except (OSError, ValueError):
        T = {"calls": {}, "fetch_scale": float("nan"), "write_scale": float("nan")}
    head = f"""Commands (run from /tmp with TMPDIR=/tmp on one MI355X; `bench.py` is the committed one, `$R` the repository root):

```
rocprofv3 --kernel-trace --stats --output-format csv -d out/prof_step  -o step  -- python3 $R/bench.py --steps 10 --warmup 2 --no-cpu-baseline
rocprofv3 --kernel-trace --stats --output-format csv -d out/prof_extra -o extra -- python3 $R/bench.py --only $(python3 $R/bench.py --extra-list) --steps 10 --warmup 2 --no-cpu-baseline
rocprofv3 --pmc FETCH_SIZE --output-format csv -d out/pmc_fetch -o f -- python3 $R/bench.py --only $(python3 $R/bench.py --traffic-list) --steps 3 --warmup 1 --no-cpu-baseline
rocprofv3 --pmc WRITE_SIZE --output-format csv -d out/pmc_write -o w -- python3 $R/bench.py --only $(python3 $R/bench.py --traffic-list) --steps 3 --warmup 1 --no-cpu-baseline
python3 $R/bench.py --traffic-from out/pmc_fetch out/pmc_write      # writes profiles/traffic.json
python3 $R/bench.py --profile-from out/prof_step out/prof_extra     # writes this file
```

Durations are rocprofv3 kernel durations (`--kernel-trace --stats`; 12 dispatches per kernel and call: 2 warm-up + 10 timed
steps; a kernel shared by several calls has more and is listed with each).  A call that needs a second kernel lists both.
GB/s = algorithmic bytes of the call / sum of the average durations; peak = 8 TB/s.  HBM bytes: FETCH_SIZE and WRITE_SIZE
(KiB per dispatch, mean over the dispatches of the counter runs), each scaled by what the same counter reports for
`mxb_probe_copy` of 1 GiB (1,048,576 KiB each way): FETCH_SIZE x {T.get('fetch_scale', float('nan')):.5f}, WRITE_SIZE x {T.get('write_scale', float('nan')):.6f}.
The event-bracketed figures that `bench.py` prints for the same calls are 3-5 us longer per call (the gap between an event
and the kernel next to it).
"""
    for title, fn, rows in PROFILE_TABLES:
        out = ["| call | kernels | dispatches | avg us (each; sum) | min us (sum) | algorithmic bytes | GB/s at avg | of 8 TB/s | HBM bytes by counters | vs algorithmic |",
               "|---|---|---|---|---|---|---|---|---|---|"]
        for label, call, nb in rows:
            ks = CALL_KERNELS[call]
            st = [find(k) for k in ks]
            if any(x is None for x in st):
                out.append(f"| {label} | " + " + ".join(f"`{k}`" for k in ks) + " | not in this run | | | | | | | |")
                continue
            avgs = [x[1] / x[0] / 1e3 for x in st]
            avg, mn = sum(avgs), sum(x[2] for x in st) / 1e3
            hb = T["calls"].get(call, {}).get("hbm_bytes")
            # a strided call is compared with the whole lines it has to move (incx = 2, incy = 3)
            whole = nb * {"axpy": 8 / 3, "dot": 5 / 2, "scal": 2, "asum": 2, "nrm2": 2}[call[1:].split("_")[0]] if call.endswith("_strided") else nb
            out.append(f"| {label} | " + " + ".join(f"`{k}`" for k in ks) + f" | {' + '.join(str(x[0]) for x in st)} | "
                       + " + ".join(f"{a:.2f}" for a in avgs) + (f" = {avg:.2f}" if len(avgs) > 1 else "")
                       + f" | {mn:.2f} | {nb:,} | {nb / avg / 1e3:.0f} | {nb / avg / 1e3 / 80:.1f} % | "
                       + (f"{hb:,} | {(hb / whole - 1) * 100:+.2f} %{' (of the whole lines)' if whole != nb else ''} |" if hb else "- | - |"))
        text = f"# rocprofv3 summary: {title}\n\n" + head + "\n" + "\n".join(out) + "\n"
        open(os.path.join(ROOT, "profiles", fn), "w").write(text)
        print("\n".join(out))


def main():
    args = parse()
    if args.traffic_list:
        print(TRAFFIC_ONLY)
        return
    if args.extra_list:
        print(EXTRA_ONLY)
        return
    if args.profile_from:
        write_profiles(args.profile_from)
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
    if args.scan:
        scan(B, ctx, torch)
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
        med = ts[len(ts) // 2]
        per[name] = {"bytes": nb, "us_avg": round(avg * 1e3, 2), "us_min": round(ts[0] * 1e3, 2),
                     "us_med": round(med * 1e3, 2), "GBps": round(nb / (med * 1e-3) / 1e9, 1),
                     "frac_of_8TBps": round(nb / (med * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        if name in suite.hw:
            # a strided call: the hardware moves whole lines, so the useful bytes can reach only
            # stride_ceiling_frac of the peak; fetched_GBps is the rate of those whole lines
            hw = suite.hw[name]
            per[name].update({"hw_line_bytes": hw, "fetched_GBps": round(hw / (med * 1e-3) / 1e9, 1),
                              "stride_ceiling_frac": round(nb / hw, 4),
                              "frac_of_stride_ceiling": round(hw / (med * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)})

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
        ach = round(p["bytes"] / (p["us_avg"] * 1e-6) / 1e9, 1)        # per launch: bytes / average launch duration
        roofline = {"bound": "hbm", "kernel": "rowdot_kernel<float,4,64,2,4,general> (sgemv N 16384x16384, beta=0)",
                    "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
                    "traffic": traffic.get(head), "algorithmic_bytes_per_launch": p["bytes"], "avg_launch_us": p["us_avg"]}
        if "probe_read_GBps" in ceiling:
            roofline["frac_of_measured_read_ceiling"] = round(ach / ceiling["probe_read_GBps"], 4)

    # the figures the headline metric names, one by one: gemv N/T at 16384^2 against the peak, level-1 GB/s
    headline = {}
    for name in (f"sgemv_n_{NS}_b0", f"sgemv_t_{NS}_b0", f"dgemv_n_{NS}", f"dgemv_t_{NS}", "saxpy", "daxpy", "sscal", "sdot", "ddot",
                 "sasum", "snrm2", "saxpy_strided", "daxpy_strided", "sscal_strided", "sdot_strided", "ddot_strided", "sasum_strided",
                 "snrm2_strided"):
        if name in per:
            headline[name] = {"GBps": per[name]["GBps"], "frac_of_8TBps": per[name]["frac_of_8TBps"]}

    four = [headline[k]["GBps"] for k in (f"sgemv_n_{NS}_b0", f"sgemv_t_{NS}_b0", f"dgemv_n_{NS}", f"dgemv_t_{NS}") if k in headline]
    step_gbps = round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1)
    if len(four) == 4:
        value = min(four)
        if roofline is not None:
            roofline["min_headline_frac"] = round(value / HBM_PEAK_GBS, 4)
    else:
        value = step_gbps          # a run restricted with --only: not the benchmark
    out = {
        "metric": "achieved HBM GB/s (% of peak) for sgemv/dgemv N,T at 16384^2; level-1 GB/s: `value` is the lowest of the four "
                  "gemv figures (sgemv N, T beta=0; dgemv N, T lda=16392; algorithmic bytes / median time); `headline` lists them "
                  "and the level-1 figures one by one; `step_GBps` is the whole step's algorithmic bytes / wall time",
        "value": value, "unit": "GB/s", "step_GBps": step_gbps,
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
        out["cpu_baseline"] = cpu_baseline(args.cpu_baseline_reps)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
