"""ctypes front end of the fp64 CPU oracle (``nfad_oracle.c``).

TEST INFRASTRUCTURE ONLY.  The oracle is the independent yardstick for the GPU
library: only the tests, the smoke check and the benchmark's ``cpu_baseline``
leg may import this package.  It imports nothing from the GPU package and the
GPU package imports nothing from here.

All arrays are contiguous ``numpy.float64``.  Kinds: 0 GELU-tanh, 1 GELU-erf,
2 Swish, 3 Mish (Table I of the paper, plus the textbook erf form of GELU).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nfad_oracle.c")
_SO = os.path.join(_HERE, "libnfad_oracle.so")

GELU_TANH, GELU_ERF, SWISH, MISH = 0, 1, 2, 3
KINDS = (GELU_TANH, GELU_ERF, SWISH, MISH)
KIND_NAMES = {GELU_TANH: "gelu_tanh", GELU_ERF: "gelu_erf", SWISH: "swish", MISH: "mish"}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, OpenMP for the timed leg)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-fno-fast-math",
               "-ffp-contract=off", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        dpp = ctypes.POINTER(dp)
        sz, ci = ctypes.c_size_t, ctypes.c_int
        lib.nfad_oracle_max_threads.restype = ci
        lib.nfad_oracle_num_saved.argtypes = [ci]
        lib.nfad_oracle_fwd.argtypes = [ci, dp, dp, dp, sz, ci]
        lib.nfad_oracle_fwd_dual.argtypes = [ci, dp, dp, dp, sz]
        lib.nfad_oracle_bwd.argtypes = [dp, dp, dp, sz, ci]
        lib.nfad_oracle_recompute_fwd.argtypes = [ci, dp, dp, sz, ci]
        lib.nfad_oracle_recompute_bwd.argtypes = [ci, dp, dp, dp, sz, ci]
        lib.nfad_oracle_saveall_fwd.argtypes = [ci, dp, dp, dpp, sz, ci]
        lib.nfad_oracle_saveall_bwd.argtypes = [ci, dp, dpp, dp, sz, ci]
        _lib = lib
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64).reshape(-1))


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"oracle {what}: bad kind or null pointer (rc={rc})")


def max_threads() -> int:
    return int(_load().nfad_oracle_max_threads())


def num_saved(kind: int) -> int:
    return int(_load().nfad_oracle_num_saved(int(kind)))


def fwd(kind: int, x, threads: int = 0):
    """(y, dydx) = (f(x), f'(x)) by the closed forms."""
    x = _f64(x)
    y, d = np.empty_like(x), np.empty_like(x)
    _check(_load().nfad_oracle_fwd(int(kind), _ptr(x), _ptr(y), _ptr(d), x.size, threads), "fwd")
    return y, d


def fwd_dual(kind: int, x):
    """(y, dydx) by propagating (value, tangent) pairs, seed tangent 1 (serial)."""
    x = _f64(x)
    y, d = np.empty_like(x), np.empty_like(x)
    _check(_load().nfad_oracle_fwd_dual(int(kind), _ptr(x), _ptr(y), _ptr(d), x.size), "fwd_dual")
    return y, d


def bwd(gy, dydx, threads: int = 0):
    gy, dydx = _f64(gy), _f64(dydx)
    assert gy.size == dydx.size
    gx = np.empty_like(gy)
    _check(_load().nfad_oracle_bwd(_ptr(gy), _ptr(dydx), _ptr(gx), gy.size, threads), "bwd")
    return gx


def recompute_fwd(kind: int, x, threads: int = 0):
    x = _f64(x)
    y = np.empty_like(x)
    _check(_load().nfad_oracle_recompute_fwd(int(kind), _ptr(x), _ptr(y), x.size, threads),
           "recompute_fwd")
    return y


def recompute_bwd(kind: int, gy, x, threads: int = 0):
    gy, x = _f64(gy), _f64(x)
    assert gy.size == x.size
    gx = np.empty_like(x)
    _check(_load().nfad_oracle_recompute_bwd(int(kind), _ptr(gy), _ptr(x), _ptr(gx), x.size,
                                             threads), "recompute_bwd")
    return gx


def _ptr_array(arrs):
    dp = ctypes.POINTER(ctypes.c_double)
    return (dp * len(arrs))(*[_ptr(a) for a in arrs])


def saveall_fwd(kind: int, x, threads: int = 0):
    """Returns (y, saved) with saved[0] a copy of x and saved[1:] the new intermediates."""
    x = _f64(x)
    k = num_saved(kind)
    if k < 0:
        raise ValueError("oracle saveall_fwd: bad kind")
    y = np.empty_like(x)
    saved = [np.empty_like(x) for _ in range(k)]
    _check(_load().nfad_oracle_saveall_fwd(int(kind), _ptr(x), _ptr(y), _ptr_array(saved), x.size,
                                           threads), "saveall_fwd")
    return y, saved


def saveall_bwd(kind: int, gy, saved, threads: int = 0):
    gy = _f64(gy)
    saved = [_f64(s) for s in saved]
    if len(saved) != num_saved(kind):
        raise ValueError("oracle saveall_bwd: wrong number of saved tensors")
    gx = np.empty_like(gy)
    _check(_load().nfad_oracle_saveall_bwd(int(kind), _ptr(gy), _ptr_array(saved), _ptr(gx),
                                           gy.size, threads), "saveall_bwd")
    return gx
