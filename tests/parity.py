"""Tolerance and comparison helpers shared by the parity tests (no method arithmetic here).

Bar (fp32 math, one rounding to storage):
  f32 storage : |gpu - ref| <= max(2e-6, ulp_f32(ref))      (2e-6 flat wherever |ref| < 16)
  f16 / bf16  : |gpu - ref| <= max(ulp_T(ref), 2e-6)
with ulp_T(v) = 2^(max(floor(log2 |v|), e_min) - p), (p, e_min) = (23,-126) f32, (10,-14) f16,
(7,-126) bf16, and ref the fp64 oracle value on the storage-rounded input.  Every pass of the
method and of the two baselines is gated at exactly this bar (`compare` with no allowance).

Two derived budgets exist, for results the bar was not written for:
  * a gradient computed from a tangent that was itself rounded to storage by the GPU (forward
    feeding backward): the tangent may be off by its own bar, which the upstream gradient
    scales, and the product is rounded once more: |gy| * bar_T(dydx) + bar_T(gx)
    (`two_stage_budget`; `saveall_two_stage_budget` is the same for the save-all baseline, whose
    backward pass consumes several GPU-stored tensors);
  * a composed chain of up to a dozen fp32 primitives: each primitive rounds (2^-24 relative)
    and the hardware exponential's argument rounding grows with |x|, so on top of the bar
    5e-7 * max(1, |x|) * max(1, |ref|) (`chain_allowance`; eight roundings of a value of
    magnitude max(1, |ref|) are 4.8e-7 relative).
"""
from __future__ import annotations

import numpy as np
import torch

P_EMIN = {torch.float32: (23, -126), torch.float16: (10, -14), torch.bfloat16: (7, -126)}
ABS_FLOOR = 2e-6


def ulp_of(ref: torch.Tensor, dtype: torch.dtype) -> torch.Tensor:
    """ulp of `dtype` at the magnitude of the float64 tensor `ref`."""
    p, emin = P_EMIN[dtype]
    _, e = torch.frexp(ref.abs())           # |ref| = m * 2^e, m in [0.5, 1)
    e = torch.clamp(e.to(torch.int32) - 1, min=emin)
    e = torch.where(ref == 0, torch.full_like(e, emin), e)
    return torch.ldexp(torch.ones_like(ref), e - p)


def tolerance(ref: torch.Tensor, dtype: torch.dtype) -> torch.Tensor:
    return torch.clamp(ulp_of(ref, dtype), min=ABS_FLOOR)


def chain_allowance(x64, ref64):
    """Allowance on top of the bar for a composed chain (see the module docstring); numpy float64."""
    return 5e-7 * np.maximum(1.0, np.abs(np.asarray(x64))) * np.maximum(1.0, np.abs(np.asarray(ref64)))


def two_stage_budget(gy64, d_ref64, gx_ref64, dtype: torch.dtype, d_allowance=None):
    """Tolerance (numpy float64) of gx = gy * dydx when dydx is the GPU's own stored tangent:
    |gy| * (bar_T(dydx) [+ allowance of dydx]) for the tangent's error; subtract the plain bar
    that `compare` applies itself, i.e. pass the result as `extra_tol`."""
    tol_d = tolerance(torch.as_tensor(np.asarray(d_ref64), dtype=torch.float64), dtype).numpy()
    if d_allowance is not None:
        tol_d = tol_d + np.asarray(d_allowance)
    return np.abs(np.asarray(gy64)) * tol_d


def saveall_two_stage_budget(kind, gy64, x64, dtype: torch.dtype):
    """The same budget for the save-all baseline when its backward pass consumes the intermediates
    that the GPU forward pass stored: each stored tensor may be off by its own bar, and the
    backward formula passes that on with the sensitivity d gx / d saved_j, taken here from the
    oracle by displacing one stored tensor at a time by its bar (both signs, the larger effect);
    numpy float64, to be passed as `extra_tol`."""
    import oracle
    x64 = np.asarray(x64, dtype=np.float64)
    one = np.ones_like(x64)
    _, saved = oracle.saveall_fwd(kind, x64)
    base = oracle.saveall_bwd(kind, one, saved)
    budget = np.zeros_like(x64)
    for j in range(1, len(saved)):
        bar_j = tolerance(torch.as_tensor(saved[j], dtype=torch.float64), dtype).numpy()
        effect = np.zeros_like(x64)
        for sign in (1.0, -1.0):
            moved = list(saved)
            moved[j] = saved[j] + sign * bar_j
            effect = np.maximum(effect, np.abs(oracle.saveall_bwd(kind, one, moved) - base))
        budget += effect
    return np.abs(np.asarray(gy64)) * budget


def compare(got: torch.Tensor, ref64, dtype: torch.dtype, what: str = "", flat_abs: float | None = None,
            extra_tol=None):
    """Element-by-element check of a storage tensor against float64 reference values.
    Returns a dict of statistics; raises AssertionError naming the worst element."""
    dev = got.device
    ref = torch.as_tensor(np.asarray(ref64), dtype=torch.float64).reshape(-1).to(dev)
    g = got.detach().reshape(-1).to(torch.float64)
    assert g.numel() == ref.numel(), (what, g.numel(), ref.numel())
    if g.numel() == 0:
        return {"n": 0, "max_abs": 0.0, "max_ulp": 0.0, "n_over_1ulp": 0}
    finite = torch.isfinite(g)
    assert bool(finite.all()), f"{what}: {int((~finite).sum())} non-finite outputs"
    err = (g - ref).abs()
    tol = tolerance(ref, dtype) if flat_abs is None else torch.full_like(ref, flat_abs)
    if extra_tol is not None:   # per-element allowance on top (float64 array-like)
        tol = tol + torch.as_tensor(np.asarray(extra_tol), dtype=torch.float64).reshape(-1).to(dev)
    bad = err > tol
    ulps = err / ulp_of(ref, dtype)
    bar = tolerance(ref, dtype) if flat_abs is None else torch.full_like(ref, flat_abs)
    stats = {
        "n": int(g.numel()),
        "max_abs": float(err.max()),
        "max_ulp": float(ulps.max()),                 # strict statistic, reported not gated
        "n_over_1ulp": int((ulps > 1.0).sum()),
        "max_over_bar": float((err / bar).max()),     # worst error in units of the stated bar (no allowance)
    }
    if bool(bad.any()):
        i = int(torch.argmax(err / tol))
        raise AssertionError(
            f"{what}: {int(bad.sum())}/{g.numel()} elements out of tolerance; worst at {i}: "
            f"got {float(g[i])!r} ref {float(ref[i])!r} err {float(err[i]):.3e} tol {float(tol[i]):.3e}")
    return stats
