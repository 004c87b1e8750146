"""Automatic detection and fusion of forward-AD chains in imperative PyTorch code.

The paper finds fad chains in PyTorch's dynamic graph with a finite state machine over
tensor-operator pairs (Sec. IV-A): an input tensor is fad (Y, produced by a fad operator)
or not (N), an operator is fad (Y) or not (N), which gives the four forward states

    NN  ordinary execution            NY  a chain begins
    YY  the chain continues           YN  the chain ends

and the chain between NY and YN is an R^1 -> R^M element-wise function whose backward pass
needs one saved tensor per output (Sec. IV-B).  The paper executes every operator eagerly and
computes tangents beside it; on MI355X the better move is not to execute the chain's
operators at all: inside `with fuse():` a fad operator applied to a tensor returns a LAZY
tensor that only records the chain (as a postfix program over the primitives), each further
fad operator extends the record (YY), and the first non-fad use (YN) compiles the whole chain
into ONE fused forward kernel (nfad_chain_compile, cached per program) that writes y and
dydx; backward is one multiply.  Intermediates never exist, so there is nothing to release.

A binary operator is fad only if both operands derive from the same source tensor, or one
of them is a Python number (Sec. III-A); otherwise it is an nfad operator and ends the chain.
One source, several outputs (R^1 -> R^M, Sec. IV-A/IV-B): when a chain ends, every other chain
over the same source that has been recorded but not yet consumed is fused into the SAME kernel
(x is read once; one value and one saved tangent per output; the backward pass merges the
upstream gradients in one kernel).

Eager semantics under mutation: an in-place operator (or out=) that writes a tensor first
resolves every recorded chain over that tensor, so deferred chains never see a later value of
their source; a tensor that has been resolved counts as an ordinary tensor from then on (an
in-place operator on it cannot leave a stale program behind); and a source changed behind the
detector's back (after the context has closed, or through a view) is caught by its version
counter when the chain is resolved.

A chain of ONE plain primitive (NY directly followed by YN; Sec. IV-B "Efficiency" treats this
case specially too) is not fused: the primitive runs natively, because its own backward keeps
at most its input or its output, both alive anyway, or nothing at all (x * c), whereas a
fused kernel would add a saved tangent.  Single calls of the framework's fused activations
(silu, gelu, mish, ...) ARE replaced: same memory, and the backward becomes one multiply.

    from paper_2209_10778_amd import trace
    with trace.fuse() as t:
        y = x * torch.tanh(torch.nn.functional.softplus(x))     # user-written Mish
        z = torch.relu(y)                                        # non-fad use: chain ends here
    t.states   -> ['NY', 'YY', 'YY', 'YN']
"""
from __future__ import annotations

import math
import weakref
from typing import List, Optional

import torch
import torch.nn.functional as F
from torch.overrides import TorchFunctionMode

from . import autograd as A

SUPPORTED_DTYPES = (torch.float32, torch.float16, torch.bfloat16)


def classify(input_is_fad: bool, op_is_fad: bool) -> str:
    """Forward state of a tensor-operator pair (Sec. IV-A)."""
    return ("Y" if input_is_fad else "N") + ("Y" if op_is_fad else "N")


class Lazy(torch.Tensor):
    """A fad tensor: the not-yet-executed chain `program` applied to `source`."""

    @staticmethod
    def __new__(cls, source: torch.Tensor, program: List[str], tracer: "fuse", nops: int = 2, native=None):
        r = torch.Tensor._make_wrapper_subclass(cls, source.shape, dtype=source.dtype, device=source.device,
                                                requires_grad=source.requires_grad)
        r._source, r._program, r._tracer, r._value = source, list(program), tracer, None
        r._nops, r._native = nops, native      # operators recorded; (func, args, kwargs) of a lone primitive
        r._source_version = source._version    # the chain means f(source as it is NOW)
        r._extended = False                    # True once another recorded chain continues this one
        tracer._register(r)
        return r

    def materialize(self) -> torch.Tensor:
        """YN: run the fused forward kernel of the recorded chain; keeps only dydx for backward.
        A chain of one plain primitive runs that primitive natively instead.  Chains over the same
        source that are waiting to be consumed are resolved by the same kernel."""
        if self._value is None:
            if self._source._version != self._source_version:
                raise RuntimeError(
                    "a tensor was modified in place after a forward-AD chain over it was recorded and before the "
                    "chain was used; resolve the chain first (use its result), or do not modify its source")
            if self._nops == 1 and self._native is not None:
                func, args, kwargs = self._native
                with torch._C.DisableTorchFunction():      # the primitive itself, not another recording
                    self._value = func(*args, **kwargs)
                self._tracer.native_singles += 1
            else:
                group = self._tracer._siblings(self)
                programs = [" ".join(l._program) for l in group]
                if len(group) == 1:
                    self._value = A.chain(self._source, programs[0])
                else:
                    for l, v in zip(group, A.chain_multi(self._source, programs)):
                        l._value, l._native = v, None
                self._tracer.kernels.append(" ; ".join(programs))
            self._native = None
        return self._value

    def __repr__(self):
        return f"Lazy(chain={' '.join(self._program)!r}, shape={tuple(self.shape)})"

    @classmethod
    def __torch_dispatch__(cls, func, types, args=(), kwargs=None):
        # never reached: every operator on a Lazy is resolved at the torch-function level below
        raise RuntimeError(f"{func} reached a lazy chain tensor that was not materialised")

    @classmethod
    def __torch_function__(cls, func, types, args=(), kwargs=None):
        kwargs = kwargs or {}
        for a in args:
            if type(a) is Lazy:
                tracer = a._tracer
                break
        else:
            tracer = [a for a in _flatten(args) + _flatten(tuple(kwargs.values())) if isinstance(a, Lazy)][0]._tracer
        if not kwargs:
            r = tracer._fast(func, args)
            if r is not _MISS:
                return r
        return tracer._dispatch(func, args, kwargs)


def _flatten(xs):
    out = []
    for a in xs:
        if isinstance(a, (list, tuple)):
            out += _flatten(a)
        else:
            out.append(a)
    return out


_F32_MAX = 3.4028234663852886e38


def _const(v) -> Optional[str]:
    """A Python number as a program token; None for anything else, for NaN and for magnitudes fp32 cannot hold."""
    if isinstance(v, bool) or not isinstance(v, (int, float)):
        return None
    return repr(float(v)) if -_F32_MAX <= v <= _F32_MAX else None


# fad operators: name -> (arity, builder over operand programs)
def _un(tok):
    return lambda a: a + [tok]


def _bin(tok):
    return lambda a, b: a + b + [tok]


_SELU_SCALE, _SELU_ALPHA = repr(1.0507009873554804934193349852946), repr(1.6732632423543772848170429916717)

_UNARY = {
    "neg": _un("neg"), "exp": _un("exp"), "log": _un("log"), "tanh": _un("tanh"), "sigmoid": _un("sigmoid"),
    "softplus": _un("softplus"), "erf": _un("erf"), "relu": _un("relu"), "abs": _un("abs"), "sqrt": _un("sqrt"),
    "square": lambda a: a + a + ["*"],
    "relu6": lambda a: a + ["0", "max", "6", "min"],
    "hardswish": lambda a: a + a + ["3", "+", "0", "max", "6", "min", "*", "6", "/"],
    "softsign": lambda a: a + ["1"] + a + ["abs", "+", "/"],
    "logsigmoid": lambda a: a + ["neg", "softplus", "neg"],
    "tanhshrink": lambda a: a + a + ["tanh", "-"],
    "hardsigmoid": lambda a: a + ["6", "/", "0.5", "+", "0", "max", "1", "min"],
    "reciprocal": lambda a: ["1"] + a + ["/"],
    "rsqrt": lambda a: ["1"] + a + ["sqrt", "/"],
    "expm1": lambda a: a + ["exp", "1", "-"],
    "log1p": lambda a: ["1"] + a + ["+", "log"],
    "erfc": lambda a: ["1"] + a + ["erf", "-"],
    "selu": lambda a: [_SELU_SCALE] + a + ["relu", _SELU_ALPHA] + a + ["0", "min", "exp", "1", "-", "*", "+", "*"],
    "silu": lambda a: a + a + ["sigmoid", "*"],
    "mish": lambda a: a + a + ["softplus", "tanh", "*"],
    "gelu_erf": lambda a: ["0.5"] + a + ["*", "1", repr(1.0 / math.sqrt(2.0))] + a + ["*", "erf", "+", "*"],
    "gelu_tanh": lambda a: ["0.5"] + a + ["*", "1", repr(math.sqrt(2.0 / math.pi))] + a + ["0.044715"] + a + a
    + ["*"] + a + ["*", "*", "+", "*", "tanh", "+", "*"],
}
_BINARY = {"add": _bin("+"), "sub": _bin("-"), "mul": _bin("*"), "div": _bin("/")}
# Activations the framework runs as one fused operator that keeps its input: replacing a single
# call by the fused forward-AD kernel costs no memory and makes the backward one multiply.
_FUSED_FUNCTIONALS = {"silu", "mish", "gelu", "elu", "selu", "celu", "hardswish", "hardsigmoid", "softsign",
                      "logsigmoid", "tanhshrink", "softplus", "leaky_relu"}


_OP_TABLE = {
    "add": "add", "__add__": "add", "__radd__": "radd", "sub": "sub", "__sub__": "sub", "__rsub__": "rsub",
    "rsub": "rsub", "mul": "mul", "__mul__": "mul", "__rmul__": "rmul", "multiply": "mul",
    "div": "div", "true_divide": "div", "__truediv__": "div", "__rtruediv__": "rdiv", "__rdiv__": "rdiv", "__div__": "div", "divide": "div",
    "neg": "neg", "negative": "neg", "__neg__": "neg", "exp": "exp", "log": "log", "tanh": "tanh",
    "sigmoid": "sigmoid", "softplus": "softplus", "erf": "erf", "square": "square", "silu": "silu",
    "mish": "mish", "gelu": "gelu", "pow": "pow", "__pow__": "pow", "relu": "relu", "abs": "abs",
    "absolute": "abs", "__abs__": "abs", "sqrt": "sqrt", "relu6": "relu6", "hardswish": "hardswish",
    "softsign": "softsign", "elu": "elu", "clamp": "clamp", "clip": "clamp",
    "logsigmoid": "logsigmoid", "log_sigmoid": "logsigmoid", "tanhshrink": "tanhshrink", "hardsigmoid": "hardsigmoid",
    "reciprocal": "reciprocal", "rsqrt": "rsqrt", "expm1": "expm1", "log1p": "log1p", "erfc": "erfc",
    "selu": "selu", "leaky_relu": "leaky_relu", "celu": "celu", "hardtanh": "hardtanh",
    "clamp_min": "clamp_min", "clamp_max": "clamp_max",
}


def _power(e):
    """The exponent of a power the primitives can spell: an integer 2..8 (also written as a float),
    0.5, -1 or -0.5; None for any other."""
    if isinstance(e, bool) or not isinstance(e, (int, float)):
        return None
    if e in (0.5, -1, -0.5):
        return float(e)
    if float(e).is_integer() and 2 <= e <= 8:
        return int(e)
    return None


def _pow_program(a, k):
    if k == 0.5:
        return a + ["sqrt"]
    if k == -1.0:
        return ["1"] + a + ["/"]
    if k == -0.5:
        return ["1"] + a + ["sqrt", "/"]
    prog = list(a)
    for _ in range(k - 1):
        prog = prog + a + ["*"]
    return prog


def _op_name(func):
    return _OP_TABLE.get(getattr(func, "__name__", ""))


_MISS = object()
_X = ["x"]
# function object -> (kind, token, operands swapped, is a fad operator of any sort, may write in place,
# is an attribute read); kind 1: plain unary primitive, 2: plain binary arithmetic, 3: power, 0: neither
_FUNC_KIND = {}
_PLAIN_UNARY = {"neg": "neg", "exp": "exp", "log": "log", "tanh": "tanh", "sigmoid": "sigmoid", "erf": "erf",
                "relu": "relu", "abs": "abs", "sqrt": "sqrt"}
_PLAIN_BINARY = {"add": ("+", False), "radd": ("+", False), "sub": ("-", False), "rsub": ("-", True),
                 "mul": ("*", False), "rmul": ("*", False), "div": ("/", False), "rdiv": ("/", True)}


def _kind_of(func):
    name = getattr(func, "__name__", "")
    op = _OP_TABLE.get(name)
    writes = (name.endswith("_") and not name.endswith("__")) or name in _INPLACE_DUNDERS
    if op in _PLAIN_UNARY:
        return (1, _PLAIN_UNARY[op], False, True, writes, False)
    if op in _PLAIN_BINARY:
        return (2,) + _PLAIN_BINARY[op] + (True, writes, False)
    if op == "pow":
        return (3, None, False, True, writes, False)
    return (0, None, False, op is not None, writes, name in _PASSIVE)


class fuse(TorchFunctionMode):
    """Context manager: detect fad chains and run each as one fused kernel."""

    def __init__(self, require_cuda: bool = True):
        super().__init__()
        self.require_cuda = require_cuda   # False only lets chains be RECORDED on host tensors (tests)
        self.states: List[str] = []      # forward state of every tensor-operator pair seen
        self.kernels: List[str] = []     # chain programs that were materialised, in order (" ; " joins a fused group)
        self.native_singles = 0          # one-primitive chains that were run natively instead
        self._pending = {}               # id(source) -> weak references to the chains recorded over it

    # ---- chains waiting to be consumed, per source
    def _register(self, lazy):
        key = id(lazy._source)
        refs = self._pending.get(key)
        if refs is None:
            if len(self._pending) >= 64:     # forget sources whose chains are all gone or resolved
                for k in [k for k, v in self._pending.items() if not any(r() is not None and r()._value is None for r in v)]:
                    del self._pending[k]
            refs = self._pending[key] = []
        elif len(refs) >= 16:                # drop references to chains that are gone
            refs[:] = [r for r in refs if r() is not None and r()._value is None]
        refs.append(weakref.ref(lazy))

    def _waiting(self, source):
        """Recorded, unresolved, still referenced chains over `source`."""
        out = []
        for r in self._pending.get(id(source), ()):
            l = r()
            if l is not None and l._value is None and l._source is source:
                out.append(l)
        return out

    def _siblings(self, lazy):
        """The chains one kernel resolves together with `lazy` (first in the list): other chains over
        the same source that nothing has continued yet (a chain that was continued is a shared
        prefix, not an output), at most NFAD_MAX_OUTPUTS distinct programs in all."""
        group, seen = [lazy], {tuple(lazy._program)}
        for l in self._waiting(lazy._source):
            if len(group) == 4:
                break
            if l is lazy or l._extended or (l._nops == 1 and l._native is not None) or tuple(l._program) in seen \
                    or l._source_version != lazy._source_version or l.shape != lazy.shape:
                continue
            seen.add(tuple(l._program))
            group.append(l)
        return group

    def _resolve_chains_over(self, tensor):
        """Before `tensor` is written in place: every chain recorded over it takes its value now."""
        for l in self._waiting(tensor):
            l.materialize()
        self._pending.pop(id(tensor), None)

    # ---- operand analysis
    def _operand(self, a, source):
        """Program of operand `a` relative to `source`, or None if it is not fad there."""
        if isinstance(a, Lazy):
            return a._program if a._source is source else None
        if isinstance(a, torch.Tensor):
            return ["x"] if a is source else None
        c = _const(a)
        return [c] if c is not None else None

    def _eligible(self, t) -> bool:
        return (isinstance(t, torch.Tensor) and not isinstance(t, Lazy) and (t.is_cuda or not self.require_cuda)
                and t.dtype in SUPPORTED_DTYPES and t.dim() > 0)

    def _try_fad(self, func, args, kwargs):
        """Returns a Lazy if (func, args) is a fad tensor-operator pair, else None."""
        op = _op_name(func)
        if op is None:
            return None
        tensors = [a for a in args if isinstance(a, torch.Tensor)]
        if not tensors:
            return None
        lazies = [a for a in tensors if isinstance(a, Lazy)]
        source = lazies[0]._source if lazies else tensors[0]
        if not lazies and not self._eligible(source):
            return None
        prog = None
        if op == "gelu":
            approx = kwargs.get("approximate", "none")
            if len(args) == 1 and set(kwargs) <= {"approximate"}:
                a = self._operand(args[0], source)
                prog = None if a is None else _UNARY["gelu_tanh" if approx == "tanh" else "gelu_erf"](a)
        elif op == "softplus":
            # softplus(v; beta) = softplus(beta v) / beta.  The framework switches to the identity above
            # beta v = threshold, where the two differ by less than exp(-threshold): any threshold >= 15
            # is below fp32 resolution and is treated as exact.
            beta, thr = kwargs.get("beta", 1.0), kwargs.get("threshold", 20.0)
            if len(args) == 1 and set(kwargs) <= {"beta", "threshold"} and _const(beta) is not None \
                    and float(beta) > 0 and _const(thr) is not None and float(thr) >= 15.0:
                a = self._operand(args[0], source)
                if a is not None:
                    prog = _UNARY["softplus"](a) if float(beta) == 1.0 else \
                        a + [_const(beta), "*", "softplus", _const(beta), "/"]
        elif op in ("leaky_relu", "celu", "hardtanh", "clamp_min", "clamp_max"):
            a = self._operand(args[0], source) if args else None
            rest = list(args[1:])
            if a is not None and not kwargs.get("inplace", False):
                def param(name, default):
                    v = rest.pop(0) if rest else kwargs.get(name, default)
                    return _const(v)
                if op == "leaky_relu" and set(kwargs) <= {"negative_slope", "inplace"} and len(args) <= 2:
                    slope = param("negative_slope", 0.01)
                    if slope is not None:       # relu(a) + slope * min(a, 0)
                        prog = a + ["relu", slope] + a + ["0", "min", "*", "+"]
                elif op == "celu" and set(kwargs) <= {"alpha", "inplace"} and len(args) <= 2:
                    alpha = param("alpha", 1.0)
                    if alpha is not None and float(alpha) != 0.0:   # relu(a) + alpha * (exp(min(a, 0) / alpha) - 1)
                        prog = a + ["relu", alpha] + a + ["0", "min", alpha, "/", "exp", "1", "-", "*", "+"]
                elif op == "hardtanh" and set(kwargs) <= {"min_val", "max_val", "inplace"} and len(args) <= 3:
                    lo, hi = param("min_val", -1.0), param("max_val", 1.0)
                    if lo is not None and hi is not None:
                        prog = a + [lo, "max", hi, "min"]
                elif op == "clamp_min" and set(kwargs) <= {"min"} and len(args) <= 2:
                    lo = param("min", None)
                    if lo is not None:
                        prog = a + [lo, "max"]
                elif op == "clamp_max" and set(kwargs) <= {"max"} and len(args) <= 2:
                    hi = param("max", None)
                    if hi is not None:
                        prog = a + [hi, "min"]
        elif op == "elu":
            alpha = kwargs.get("alpha", 1.0)
            if len(args) == 1 and set(kwargs) <= {"alpha", "inplace"} and not kwargs.get("inplace", False) \
                    and _const(alpha) is not None:
                a = self._operand(args[0], source)
                if a is not None:       # relu(a) + alpha * (exp(min(a, 0)) - 1)
                    prog = a + ["relu", _const(alpha)] + a + ["0", "min", "exp", "1", "-", "*", "+"]
        elif op == "clamp":
            lo = args[1] if len(args) > 1 else kwargs.get("min")
            hi = args[2] if len(args) > 2 else kwargs.get("max")
            if set(kwargs) <= {"min", "max"} and len(args) <= 3 and (lo is not None or hi is not None) \
                    and all(v is None or _const(v) is not None for v in (lo, hi)):
                a = self._operand(args[0], source)
                if a is not None:
                    prog = list(a)
                    if lo is not None:
                        prog += [_const(lo), "max"]
                    if hi is not None:
                        prog += [_const(hi), "min"]
        elif op == "pow":
            k = _power(args[1]) if len(args) == 2 and not kwargs else None
            if k is not None:
                a = self._operand(args[0], source)
                if a is not None:
                    prog = _pow_program(a, k)
        elif op in _UNARY:
            if len(args) == 1 and (not kwargs or kwargs == {"inplace": False}):
                a = self._operand(args[0], source)
                prog = None if a is None else _UNARY[op](a)
        else:
            base = {"radd": "add", "rsub": "sub", "rmul": "mul", "rdiv": "div"}.get(op, op)
            if len(args) == 2 and (not kwargs or (base in ("add", "sub") and kwargs == {"alpha": 1})):
                l, r = (args[1], args[0]) if op in ("rsub", "rdiv") else (args[0], args[1])
                a, b = self._operand(l, source), self._operand(r, source)
                same_shape = all(t.shape == source.shape for t in tensors)
                if a is not None and b is not None and same_shape:
                    prog = _BINARY[base](a, b)
        if prog is None or "x" not in prog or len(prog) > 250:
            return None
        nops = 1 + sum(a._nops for a in lazies)
        native = (func, args, dict(kwargs)) if not lazies and op not in _FUSED_FUNCTIONALS else None
        for a in lazies:
            a._extended = True
        return Lazy(source, prog, self, nops, native)

    # ---- the common cases without the general machinery: a primitive applied to a chain or a
    # plain tensor, no keyword arguments.  Classification of the operator is cached per function
    # object.  Returns a Lazy (NY or YY, logged), or _MISS for everything else.
    def _fast(self, func, args):
        info = _FUNC_KIND.get(func)
        if info is None:
            info = _FUNC_KIND[func] = _kind_of(func)
        kind, tok, swap = info[0], info[1], info[2]
        if kind == 1:
            if len(args) != 1:
                return _MISS
            a = args[0]
            ta = type(a)
            if ta is Lazy:
                if a._value is not None:
                    return _MISS
                a._extended = True
                self.states.append("YY")
                return Lazy(a._source, a._program + [tok], self, a._nops + 1, None)
            if (ta is torch.Tensor or ta is torch.nn.Parameter) and self._eligible(a):
                self.states.append("NY")
                return Lazy(a, ["x", tok], self, 1, (func, args, {}))
            return _MISS
        if kind == 2:
            if len(args) != 2:
                return _MISS
            l, r = (args[1], args[0]) if swap else args
            source, lazy_in, progs = None, False, []
            for o in (l, r):
                to = type(o)
                if to is Lazy:
                    if o._value is not None or (source is not None and o._source is not source):
                        return _MISS
                    source, lazy_in = o._source, True
                    progs.append(o._program)
                elif to is torch.Tensor or to is torch.nn.Parameter:
                    if source is not None and o is not source:
                        return _MISS
                    source = o
                    progs.append(_X)
                elif (to is float or to is int) and -_F32_MAX <= o <= _F32_MAX:
                    progs.append([repr(float(o))])
                else:
                    return _MISS
            if source is None:
                return _MISS
            # a plain tensor named before the chain it is the source of: re-check identity
            for o in (l, r):
                if type(o) is not Lazy and isinstance(o, torch.Tensor) and (o is not source or o.shape != source.shape):
                    return _MISS
            if not lazy_in and not self._eligible(source):
                return _MISS
            prog = progs[0] + progs[1] + [tok]
            if len(prog) > 250:
                return _MISS
            nops = 1
            for o in (l, r):
                if type(o) is Lazy:
                    o._extended = True
                    nops += o._nops
            self.states.append("YY" if lazy_in else "NY")
            return Lazy(source, prog, self, nops, None if lazy_in else (func, args, {}))
        if kind == 3:                                 # a power the primitives can spell
            if len(args) != 2:
                return _MISS
            k = _power(args[1])
            if k is None:
                return _MISS
            a = args[0]
            ta = type(a)
            if ta is Lazy:
                if a._value is not None or len(a._program) * 8 + 8 > 250:
                    return _MISS
                a._extended = True
                self.states.append("YY")
                return Lazy(a._source, _pow_program(a._program, k), self, a._nops + 1, None)
            if (ta is torch.Tensor or ta is torch.nn.Parameter) and self._eligible(a):
                self.states.append("NY")
                return Lazy(a, _pow_program(_X, k), self, 1, (func, args, {}))
            return _MISS
        return _MISS

    # ---- the state machine
    def _dispatch(self, func, args, kwargs):
        if getattr(func, "__name__", "") in _PASSIVE:          # attribute reads: not graph operators
            with torch._C.DisableTorchFunctionSubclass():
                return func(*args, **kwargs)
        with torch._C.DisableTorchFunctionSubclass():
            return self._step(func, args, kwargs)

    def _step(self, func, args, kwargs):
        # a chain that has been resolved is an ordinary tensor from here on (its value may since have
        # been written in place: the recorded program no longer describes it)
        if any(isinstance(a, Lazy) and a._value is not None for a in _flatten(args) + _flatten(tuple(kwargs.values()))):
            swap = lambda a: a._value if isinstance(a, Lazy) and a._value is not None else a
            args = _map(args, swap)
            kwargs = {k: _map((v,), swap)[0] for k, v in kwargs.items()}
        written = _written_tensors(func, args, kwargs)
        if written:
            for t in written:
                self._resolve_chains_over(t.materialize() if isinstance(t, Lazy) else t)
        flat = _flatten(args) + _flatten(tuple(kwargs.values()))
        input_is_fad = any(isinstance(a, Lazy) for a in flat)
        has_tensor = any(isinstance(a, torch.Tensor) for a in flat)
        lazy = self._try_fad(func, args, kwargs) if has_tensor and not written else None
        if has_tensor:
            self.states.append(classify(input_is_fad, lazy is not None))
        if lazy is not None:                       # NY or YY: record, execute nothing
            return lazy
        if input_is_fad:                           # YN: the chain ends; fuse it, then run the operator
            args = _map(args, lambda a: a.materialize() if isinstance(a, Lazy) else a)
            kwargs = {k: _map((v,), lambda a: a.materialize() if isinstance(a, Lazy) else a)[0]
                      for k, v in kwargs.items()}
        return func(*args, **kwargs)               # NN (or the operator after YN)

    def __torch_function__(self, func, types, args=(), kwargs=None):
        # Fast paths for the bulk of a model's operators.  What kind of operator `func` is, is looked
        # up once per function object.  (A lazy tensor nested deeper in the arguments than these
        # checks look is still caught: the call then reaches Lazy.__torch_function__.)
        info = _FUNC_KIND.get(func)
        if info is None:
            info = _FUNC_KIND[func] = _kind_of(func)
        if info[0]:                                   # a plain primitive: NY / YY without the general machinery
            if not kwargs:
                r = self._fast(func, args)
                if r is not _MISS:
                    return r
        elif not info[3]:                             # not a fad operator at all: ordinary execution (NN, not logged)
            for a in args:
                if type(a) is Lazy:
                    if a._value is None and not info[4] and not info[5]:
                        # YN, the common way a chain ends: a non-fad operator consumes it
                        if kwargs:
                            if "out" in kwargs:
                                break
                            for v in kwargs.values():
                                if type(v) is Lazy:
                                    break
                            else:
                                self.states.append("YN")
                                return func(*[b.materialize() if type(b) is Lazy else b for b in args], **kwargs)
                            break
                        self.states.append("YN")
                        return func(*[b.materialize() if type(b) is Lazy else b for b in args])
                    break
            else:
                if kwargs:
                    for v in kwargs.values():
                        if type(v) is Lazy:
                            break
                    else:
                        if not (self._pending and (info[4] or "out" in kwargs)):
                            return func(*args, **kwargs)
                elif not (self._pending and info[4]):
                    return func(*args)
        kwargs = kwargs or {}
        if info[3] and len(args) == 2 and not kwargs and type(args[0]) is torch.Tensor and type(args[1]) is torch.Tensor \
                and args[0] is not args[1]:
            return func(*args)                        # two different tensors: never a fad pair (Sec. III-A)
        return self._dispatch(func, args, kwargs)


# attribute reads and bookkeeping calls that are not operators of the graph
_PASSIVE = {"__get__", "__set__", "size", "dim", "stride", "is_contiguous", "numel", "__len__", "__repr__",
            "is_floating_point", "type", "data_ptr", "requires_grad_", "_make_wrapper_subclass", "detach"}


_INPLACE_DUNDERS = {"__iadd__", "__isub__", "__imul__", "__itruediv__", "__idiv__", "__ifloordiv__", "__imod__",
                    "__ipow__", "__iand__", "__ior__", "__ixor__", "__ilshift__", "__irshift__", "__setitem__"}


def _may_write(name, kwargs) -> bool:
    return (name.endswith("_") and not name.endswith("__")) or name in _INPLACE_DUNDERS or "out" in kwargs


def _written_tensors(func, args, kwargs):
    """Tensors an operator writes in place: `self` of a method whose name ends in an underscore (add_,
    copy_, zero_, ...) or of an augmented assignment, and the out= arguments."""
    name = getattr(func, "__name__", "")
    if not _may_write(name, kwargs):
        return []
    out = []
    if name != "" and (name.endswith("_") or name in _INPLACE_DUNDERS) and args and isinstance(args[0], torch.Tensor):
        out.append(args[0])
    o = kwargs.get("out")
    if o is not None:
        out += [t for t in _flatten((o,)) if isinstance(t, torch.Tensor)]
    return out


def _map(xs, f):
    return type(xs)(_map(a, f) if isinstance(a, (list, tuple)) else f(a) for a in xs)
