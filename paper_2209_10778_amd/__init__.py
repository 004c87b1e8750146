"""libnfad for MI355X: nested forward-mode AD of element-wise activations.

The work is done by hand-written gfx950 kernels in ``libnfad.so`` (C ABI: ``include/nfad.h``).
This package is the thin binding: it marshals torch tensors (device memory and streams
only) into that ABI and raises if the library is missing or a call fails.  There is no
CPU or PyTorch fallback.
"""
from .binding import (  # noqa: F401
    BF16, F16, F32, GELU_ERF, GELU_TANH, KIND_NAMES, KINDS, MISH, SWISH,
    NfadError, lib, lib_path, nfad_bwd, nfad_bwd_multi, nfad_chain_compile, nfad_chain_compile_multi, nfad_chain_count,
    nfad_chain_fwd_multi, nfad_chain_num_outputs, nfad_chain_fwd, nfad_chain_log,
    nfad_chain_kernel, nfad_chain_name, nfad_chain_release,
    nfad_chain_program, nfad_fwd, nfad_recompute_bwd, nfad_recompute_fwd,
    nfad_saveall_bwd, nfad_saveall_fwd, nfad_saveall_num_saved, nfad_status_string, nfad_version,
)
