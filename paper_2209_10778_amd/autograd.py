"""PyTorch autograd front end: activations whose backward pass needs ONE saved tensor.

The paper deploys its method in PyTorch by overriding autograd Functions (Sec. V-A); this is
the same hook for libnfad.  The forward pass runs the fused kernel (y and dydx in one pass
over x), keeps only `dydx` for backward (Sec. II-C eq. 3: the tangent v3' is the one stored value), and the
backward pass is the single multiply gx = gy * dydx (eq. 4).  `x` is not saved, so its
buffer is free as soon as no other operator holds it.

Only argument marshalling happens here; there is no PyTorch fallback.  For comparison the
two baselines are wrapped the same way: `mode="recompute"` keeps x and re-derives f'(x) in
backward, `mode="saveall"` keeps every intermediate of ordinary back-propagation.
"""
from __future__ import annotations

import collections

import torch

from . import binding as B

_KIND_BY_NAME = {"gelu_tanh": B.GELU_TANH, "gelu_erf": B.GELU_ERF, "gelu": B.GELU_ERF,
                 "swish": B.SWISH, "silu": B.SWISH, "mish": B.MISH}


def _flat(t: torch.Tensor) -> torch.Tensor:
    return t.contiguous().view(-1)


class _Fad(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, kind):
        xf = _flat(x)
        y = torch.empty_like(xf)
        dydx = torch.empty_like(xf)
        B.nfad_fwd(kind, xf, y, dydx)
        ctx.save_for_backward(dydx)
        return y.view(x.shape)

    @staticmethod
    def backward(ctx, gy):
        (dydx,) = ctx.saved_tensors
        gyf = _flat(gy)
        gx = torch.empty_like(gyf)
        B.nfad_bwd(gyf, dydx, gx)
        return gx.view(gy.shape), None


class _FadChain(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, chain_id):
        xf = _flat(x)
        y = torch.empty_like(xf)
        dydx = torch.empty_like(xf)
        B.nfad_chain_fwd(chain_id, xf, y, dydx)
        ctx.save_for_backward(dydx)
        return y.view(x.shape)

    @staticmethod
    def backward(ctx, gy):
        (dydx,) = ctx.saved_tensors
        gyf = _flat(gy)
        gx = torch.empty_like(gyf)
        B.nfad_bwd(gyf, dydx, gx)
        return gx.view(gy.shape), None


class _Recompute(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, kind):
        xf = _flat(x)
        y = torch.empty_like(xf)
        B.nfad_recompute_fwd(kind, xf, y)
        ctx.save_for_backward(xf)
        ctx.kind = kind
        return y.view(x.shape)

    @staticmethod
    def backward(ctx, gy):
        (xf,) = ctx.saved_tensors
        gyf = _flat(gy)
        gx = torch.empty_like(gyf)
        B.nfad_recompute_bwd(ctx.kind, gyf, xf, gx)
        return gx.view(gy.shape), None


class _SaveAll(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, kind):
        xf = _flat(x)
        y = torch.empty_like(xf)
        k = B.nfad_saveall_num_saved(kind)
        saved = [xf] + [torch.empty_like(xf) for _ in range(k - 1)]
        B.nfad_saveall_fwd(kind, xf, y, saved)
        ctx.save_for_backward(*saved)
        ctx.kind = kind
        return y.view(x.shape)

    @staticmethod
    def backward(ctx, gy):
        saved = list(ctx.saved_tensors)
        gyf = _flat(gy)
        gx = torch.empty_like(gyf)
        B.nfad_saveall_bwd(ctx.kind, gyf, saved, gx)
        return gx.view(gy.shape), None


_MODES = {"fad": _Fad, "recompute": _Recompute, "saveall": _SaveAll}


def activation(x: torch.Tensor, kind, mode: str = "fad") -> torch.Tensor:
    """kind: one of 'gelu_tanh', 'gelu_erf' ('gelu'), 'swish' ('silu'), 'mish', or the integer code."""
    k = _KIND_BY_NAME[kind] if isinstance(kind, str) else int(kind)
    return _MODES[mode].apply(x, k)


def chain(x: torch.Tensor, chain) -> torch.Tensor:
    """A composed chain: `chain` is a chain id, the name of a built-in chain, or a postfix
    program (compiled at first use and cached for the process)."""
    return _FadChain.apply(x, _chain_id(chain))


class _FadChainMulti(torch.autograd.Function):
    """One source, M chains: one kernel reads x once and writes M values and M tangents;
    backward merges the M upstream gradients at the source."""

    @staticmethod
    def forward(ctx, x, chain_id, m):
        xf = _flat(x)
        ys = [torch.empty_like(xf) for _ in range(m)]
        ds = [torch.empty_like(xf) for _ in range(m)]
        B.nfad_chain_fwd_multi(chain_id, xf, ys, ds)
        ctx.save_for_backward(*ds)
        return tuple(y.view(x.shape) for y in ys)

    @staticmethod
    def backward(ctx, *gys):
        ds = list(ctx.saved_tensors)
        gyf = [_flat(g) for g in gys]
        gx = torch.empty_like(gyf[0])
        B.nfad_bwd_multi(gyf, ds, gx)
        return gx.view(gys[0].shape), None, None


def chain_multi(x: torch.Tensor, programs):
    """Several chains over the same source, fused into one forward kernel (R^1 -> R^M)."""
    key = tuple(programs)
    cid = _remember(key, lambda: B.nfad_chain_compile_multi(list(programs)))
    return _FadChainMulti.apply(x, cid, len(programs))


# program (or tuple of programs) -> chain id, least recently used first.  Bounded: code that bakes a
# changing number into its chains (x * step_size) would otherwise compile, and keep, a kernel per value.
_compiled: "collections.OrderedDict" = collections.OrderedDict()
MAX_COMPILED = 512


def _remember(key, make) -> int:
    if key in _compiled:
        _compiled.move_to_end(key)
        return _compiled[key]
    cid = make()
    _compiled[key] = cid
    while len(_compiled) > MAX_COMPILED:
        _, old = _compiled.popitem(last=False)
        if old >= B.NFAD_CHAIN_JIT_BASE:           # built-in chains are not ours to release
            torch.cuda.synchronize()               # no launch of the evicted kernel may be in flight
            B.nfad_chain_release(old)
    return cid


def _chain_id(chain) -> int:
    if isinstance(chain, int):
        return chain

    def make():
        names = {B.nfad_chain_name(i): i for i in range(B.nfad_chain_count())}
        return names[chain] if chain in names else B.nfad_chain_compile(chain)
    return _remember(chain, make)


def gelu(x, approximate: str = "none", mode: str = "fad"):
    return activation(x, "gelu_tanh" if approximate == "tanh" else "gelu_erf", mode)


def silu(x, mode: str = "fad"):
    return activation(x, "swish", mode)


def mish(x, mode: str = "fad"):
    return activation(x, "mish", mode)


class Activation(torch.nn.Module):
    """Drop-in module: Activation('mish'), Activation('gelu_tanh', mode='recompute'), ..."""

    def __init__(self, kind: str = "gelu_erf", mode: str = "fad"):
        super().__init__()
        self.kind, self.mode = kind, mode

    def forward(self, x):
        return activation(x, self.kind, self.mode)

    def extra_repr(self):
        return f"{self.kind}, mode={self.mode}"
