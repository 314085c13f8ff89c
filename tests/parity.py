"""Helpers shared by the GPU parity tests: tolerance gates and host<->device plumbing."""
from __future__ import annotations

import math

import numpy as np

F32_TOL, F64_TOL = 1e-5, 1e-13      # x sqrt(reduction length): the stated acceptance bound


def tolerance(dtype, n_red: int) -> float:
    base = F32_TOL if np.dtype(dtype) == np.float32 else F64_TOL
    return base * math.sqrt(max(int(n_red), 1))


def tight_tolerance(dtype, n_red: int) -> float:
    """What the kernels' arithmetic should comfortably reach (16 eps sqrt(n)); stricter than the
    acceptance bound, so that a slightly wrong kernel cannot hide inside the loose one."""
    return 16.0 * float(np.finfo(dtype).eps) * math.sqrt(max(int(n_red), 1))


def check_close(got, ref, D, n_red, what=""):
    """Gate a GPU result against the oracle: (i) norm-wise max|g-r|/max|r| and (ii)
    condition-aware max|g-r|/D, both under the acceptance bound and the tighter kernel bound;
    where D == 0 the two must be equal.  Returns the two error figures."""
    got = np.asarray(got); ref = np.asarray(ref); D = np.asarray(D, np.float64)
    assert got.shape == ref.shape, f"{what}: shape {got.shape} vs {ref.shape}"
    if got.size == 0:
        return 0.0, 0.0
    assert np.isfinite(ref).all(), f"{what}: oracle result is not finite"
    assert np.isfinite(got).all(), f"{what}: GPU result has {np.count_nonzero(~np.isfinite(got))} non-finite values"
    diff = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    scale = float(np.max(np.abs(ref)))
    normwise = float(diff.max() / scale) if scale > 0 else float(diff.max())
    zero = D == 0
    assert np.array_equal(got[zero], ref[zero]), f"{what}: differs where the condition denominator is 0"
    cond = float(np.max(diff[~zero] / D[~zero])) if (~zero).any() else 0.0
    tol = min(tolerance(ref.dtype, n_red), tight_tolerance(ref.dtype, n_red))
    assert normwise <= tol and cond <= tol, (
        f"{what}: norm-wise {normwise:.3e}, condition-aware {cond:.3e} exceed {tol:.3e} "
        f"(acceptance bound {tolerance(ref.dtype, n_red):.3e})")
    return normwise, cond


def bits_equal(a, b) -> bool:
    """Bitwise equality after mapping -0 to +0."""
    a = np.asarray(a) + 0; b = np.asarray(b) + 0
    a = np.where(a == 0, 0, a); b = np.where(b == 0, 0, b)
    return a.tobytes() == b.tobytes()


def to_dev(a: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_host(t) -> np.ndarray:
    return t.detach().cpu().numpy()


def prefix_of(dtype) -> str:
    return "s" if np.dtype(dtype) == np.float32 else "d"
