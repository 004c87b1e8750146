"""ctypes binding of libnfad.so: same names as the C ABI, argument marshalling only."""
from __future__ import annotations

import ctypes
import os

import torch

GELU_TANH, GELU_ERF, SWISH, MISH = 0, 1, 2, 3
KINDS = (GELU_TANH, GELU_ERF, SWISH, MISH)
KIND_NAMES = {GELU_TANH: "gelu_tanh", GELU_ERF: "gelu_erf", SWISH: "swish", MISH: "mish"}
F32, F16, BF16 = 0, 1, 2
NFAD_CHAIN_JIT_BASE = 1000   # ids of run-time compiled chains start here (include/nfad.h)
_DTYPE_CODE = {torch.float32: F32, torch.float16: F16, torch.bfloat16: BF16}

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libnfad.so")
_lib = None


class NfadError(RuntimeError):
    """A libnfad call returned a non-zero status."""

    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {nfad_status_string(status)} (status {status})")


def lib_path() -> str:
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    """The loaded C library.  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(
                f"{_LIB_PATH} is missing: build it first (python -m paper_2209_10778_amd.build). "
                "libnfad has no CPU or PyTorch fallback.")
        L = ctypes.CDLL(_LIB_PATH)
        vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        vpp = ctypes.POINTER(ctypes.c_void_p)
        L.nfad_fwd.argtypes = [ci, vp, vp, vp, sz, ci, vp]
        L.nfad_bwd.argtypes = [vp, vp, vp, sz, ci, vp]
        L.nfad_recompute_fwd.argtypes = [ci, vp, vp, sz, ci, vp]
        L.nfad_recompute_bwd.argtypes = [ci, vp, vp, vp, sz, ci, vp]
        L.nfad_saveall_num_saved.argtypes = [ci]
        L.nfad_saveall_fwd.argtypes = [ci, vp, vp, vpp, sz, ci, vp]
        L.nfad_saveall_bwd.argtypes = [ci, vp, vpp, vp, sz, ci, vp]
        L.nfad_chain_fwd.argtypes = [ci, vp, vp, vp, sz, ci, vp]
        L.nfad_chain_name.argtypes = [ci]
        L.nfad_chain_name.restype = ctypes.c_char_p
        L.nfad_chain_program.argtypes = [ci]
        L.nfad_chain_program.restype = ctypes.c_char_p
        L.nfad_chain_compile.argtypes = [ctypes.c_char_p, ctypes.POINTER(ci)]
        L.nfad_chain_release.argtypes = [ci]
        L.nfad_chain_kernel.argtypes = [ci]
        L.nfad_chain_compile_multi.argtypes = [ctypes.POINTER(ctypes.c_char_p), ci, ctypes.POINTER(ci)]
        L.nfad_chain_num_outputs.argtypes = [ci]
        L.nfad_chain_fwd_multi.argtypes = [ci, vp, vpp, vpp, sz, ci, vp]
        L.nfad_bwd_multi.argtypes = [vpp, vpp, ci, vp, sz, ci, vp]
        L.nfad_chain_log.restype = ctypes.c_char_p
        L.nfad_status_string.argtypes = [ci]
        L.nfad_status_string.restype = ctypes.c_char_p
        for name in ("nfad_fwd", "nfad_bwd", "nfad_recompute_fwd", "nfad_recompute_bwd",
                     "nfad_saveall_num_saved", "nfad_saveall_fwd", "nfad_saveall_bwd", "nfad_version",
                     "nfad_chain_count", "nfad_chain_fwd", "nfad_chain_compile", "nfad_chain_release",
                     "nfad_chain_compile_multi", "nfad_chain_num_outputs", "nfad_chain_fwd_multi",
                     "nfad_bwd_multi", "nfad_chain_kernel"):
            getattr(L, name).restype = ci
        _lib = L
    return _lib


def _stream(stream) -> int:
    if stream is None:                       # the current device's current stream, without a Stream object
        return torch._C._cuda_getCurrentRawStream(torch._C._cuda_getDevice())
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


def _marshal(*tensors):
    """All tensors: contiguous device tensors of one supported dtype and one size."""
    t0 = tensors[0]
    if t0.dtype not in _DTYPE_CODE:
        raise TypeError(f"unsupported dtype {t0.dtype}")
    for t in tensors:
        if not t.is_cuda:
            raise ValueError("libnfad works on device memory only")
        if t.dtype != t0.dtype or t.numel() != t0.numel():
            raise ValueError("all tensors of one call must share dtype and element count")
        if not t.is_contiguous():
            raise ValueError("tensors must be contiguous")
    return t0.numel(), _DTYPE_CODE[t0.dtype]


def _check(status: int, where: str) -> None:
    if status != 0:
        raise NfadError(status, where)


def nfad_fwd(kind, x, y, dydx, stream=None) -> None:
    n, dt = _marshal(x, y, dydx)
    _check(lib().nfad_fwd(int(kind), x.data_ptr(), y.data_ptr(), dydx.data_ptr(), n, dt,
                          _stream(stream)), "nfad_fwd")


def nfad_bwd(gy, dydx, gx, stream=None) -> None:
    n, dt = _marshal(gy, dydx, gx)
    _check(lib().nfad_bwd(gy.data_ptr(), dydx.data_ptr(), gx.data_ptr(), n, dt, _stream(stream)),
           "nfad_bwd")


def nfad_recompute_fwd(kind, x, y, stream=None) -> None:
    n, dt = _marshal(x, y)
    _check(lib().nfad_recompute_fwd(int(kind), x.data_ptr(), y.data_ptr(), n, dt, _stream(stream)),
           "nfad_recompute_fwd")


def nfad_recompute_bwd(kind, gy, x, gx, stream=None) -> None:
    n, dt = _marshal(gy, x, gx)
    _check(lib().nfad_recompute_bwd(int(kind), gy.data_ptr(), x.data_ptr(), gx.data_ptr(), n, dt,
                                    _stream(stream)), "nfad_recompute_bwd")


def nfad_saveall_num_saved(kind) -> int:
    return int(lib().nfad_saveall_num_saved(int(kind)))


def _ptr_array(tensors):
    arr = (ctypes.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = None if t is None else t.data_ptr()
    return arr


def nfad_saveall_fwd(kind, x, y, saved, stream=None) -> None:
    """saved: list of k tensors; saved[0] stands for x and is not written (may be None)."""
    k = nfad_saveall_num_saved(kind)
    if k < 0:
        raise NfadError(1, "nfad_saveall_fwd")
    if len(saved) != k:
        raise ValueError(f"kind {kind} keeps {k} tensors, got {len(saved)}")
    n, dt = _marshal(x, y, *[s for s in saved[1:]])
    _check(lib().nfad_saveall_fwd(int(kind), x.data_ptr(), y.data_ptr(), _ptr_array(saved), n, dt,
                                  _stream(stream)), "nfad_saveall_fwd")


def nfad_saveall_bwd(kind, gy, saved, gx, stream=None) -> None:
    k = nfad_saveall_num_saved(kind)
    if k < 0:
        raise NfadError(1, "nfad_saveall_bwd")
    if len(saved) != k:
        raise ValueError(f"kind {kind} keeps {k} tensors, got {len(saved)}")
    n, dt = _marshal(gy, gx, *saved)
    _check(lib().nfad_saveall_bwd(int(kind), gy.data_ptr(), _ptr_array(saved), gx.data_ptr(), n, dt,
                                  _stream(stream)), "nfad_saveall_bwd")


def nfad_chain_count() -> int:
    return int(lib().nfad_chain_count())


def nfad_chain_name(chain_id: int):
    r = lib().nfad_chain_name(int(chain_id))
    return None if r is None else r.decode()


def nfad_chain_program(chain_id: int):
    r = lib().nfad_chain_program(int(chain_id))
    return None if r is None else r.decode()


def nfad_chain_fwd(chain_id, x, y, dydx, stream=None) -> None:
    n, dt = _marshal(x, y, dydx)
    _check(lib().nfad_chain_fwd(int(chain_id), x.data_ptr(), y.data_ptr(), dydx.data_ptr(), n, dt,
                                _stream(stream)), "nfad_chain_fwd")


def nfad_chain_compile(program: str) -> int:
    """Compile a postfix chain program into a fused forward kernel; returns its chain id."""
    cid = ctypes.c_int(-1)
    status = lib().nfad_chain_compile(program.encode(), ctypes.byref(cid))
    if status != 0:
        raise NfadError(status, f"nfad_chain_compile({program!r}): {nfad_chain_log()}")
    return int(cid.value)


def nfad_chain_compile_multi(programs) -> int:
    """Compile m chains over the same source into ONE forward kernel; returns the chain id."""
    arr = (ctypes.c_char_p * len(programs))(*[p.encode() for p in programs])
    cid = ctypes.c_int(-1)
    status = lib().nfad_chain_compile_multi(arr, len(programs), ctypes.byref(cid))
    if status != 0:
        raise NfadError(status, f"nfad_chain_compile_multi({list(programs)!r}): {nfad_chain_log()}")
    return int(cid.value)


def nfad_chain_num_outputs(chain_id: int) -> int:
    return int(lib().nfad_chain_num_outputs(int(chain_id)))


def nfad_chain_fwd_multi(chain_id, x, ys, dydxs, stream=None) -> None:
    n, dt = _marshal(x, *ys, *dydxs)
    _check(lib().nfad_chain_fwd_multi(int(chain_id), x.data_ptr(), _ptr_array(ys), _ptr_array(dydxs), n, dt,
                                      _stream(stream)), "nfad_chain_fwd_multi")


def nfad_bwd_multi(gys, dydxs, gx, stream=None) -> None:
    if len(gys) != len(dydxs):
        raise ValueError("one upstream gradient per saved tangent")
    n, dt = _marshal(gx, *gys, *dydxs)
    _check(lib().nfad_bwd_multi(_ptr_array(gys), _ptr_array(dydxs), len(gys), gx.data_ptr(), n, dt,
                                _stream(stream)), "nfad_bwd_multi")


def nfad_chain_kernel(chain_id: int) -> int:
    """Identifier of the compiled kernel behind a run-time chain (shared by chains that differ only
    in constants); -1 for a built-in or dead id."""
    return int(lib().nfad_chain_kernel(int(chain_id)))


def nfad_chain_release(chain_id: int) -> None:
    _check(lib().nfad_chain_release(int(chain_id)), "nfad_chain_release")


def nfad_chain_log() -> str:
    return (lib().nfad_chain_log() or b"").decode(errors="replace")


def nfad_status_string(status: int) -> str:
    return lib().nfad_status_string(int(status)).decode()


def nfad_version() -> int:
    return int(lib().nfad_version())
