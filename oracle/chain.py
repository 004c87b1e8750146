"""fp64 oracle for composed forward-AD chains: a postfix interpreter over dual numbers.

TEST INFRASTRUCTURE ONLY (same rules as the rest of this package).

A chain is a postfix program over the paper's primitive operations (Sec. III-A, Sec. V-A):
tokens are `x` (the source element), decimal constants, the binary operators `+ - * / min max`
(both operands derive from the same source, or one is a constant) and the unary primitives
`neg exp log tanh sigmoid softplus erf relu abs sqrt`.  At a kink the tangent of relu and abs is
0 and min/max follow their first operand.  Every stack entry is a pair (v, v') of float64
arrays; `x` pushes (x, 1) and each primitive applies its textbook derivative rule
(Sec. II-D: v' = sum over inputs of dv/du * u').  The result is (y, dydx).

Plain numpy / scipy.special in float64, one primitive at a time, no fusion.
"""
from __future__ import annotations

import numpy as np
from scipy import special as _sp


def _sigmoid(v):
    return _sp.expit(v)


_UNARY = {
    "neg": lambda v, d: (-v, -d),
    "exp": lambda v, d: (np.exp(v), np.exp(v) * d),
    "log": lambda v, d: (np.log(v), d / v),
    # 1 - tanh^2 = 1/cosh^2 (cosh overflows to inf for huge |v|: the tangent is then 0, as it should be)
    "tanh": lambda v, d: (np.tanh(v), d / np.cosh(v) ** 2),
    "sigmoid": lambda v, d: (_sigmoid(v), _sigmoid(v) * _sigmoid(-v) * d),
    "softplus": lambda v, d: (np.logaddexp(0.0, v), _sigmoid(v) * d),
    "erf": lambda v, d: (_sp.erf(v), 2.0 / np.sqrt(np.pi) * np.exp(-v * v) * d),
    "relu": lambda v, d: (np.maximum(v, 0.0), np.where(v > 0.0, d, 0.0)),
    "abs": lambda v, d: (np.abs(v), np.sign(v) * d),
    "sqrt": lambda v, d: (np.sqrt(v), d / (2.0 * np.sqrt(v))),
}

_BINARY = {
    "+": lambda a, da, b, db: (a + b, da + db),
    "-": lambda a, da, b, db: (a - b, da - db),
    "*": lambda a, da, b, db: (a * b, a * db + da * b),
    "/": lambda a, da, b, db: (a / b, (da - (a / b) * db) / b),
    "min": lambda a, da, b, db: (np.where(a <= b, a, b), np.where(a <= b, da, db)),
    "max": lambda a, da, b, db: (np.where(a >= b, a, b), np.where(a >= b, da, db)),
}


def eval_chain(program: str, x):
    """(y, dydx) of the chain at every element of x, float64."""
    x = np.ascontiguousarray(np.asarray(x, dtype=np.float64).reshape(-1))
    stack = []
    with np.errstate(over="ignore", invalid="ignore", divide="ignore"):
        for tok in program.split():
            if tok == "x":
                stack.append((x, np.ones_like(x)))
            elif tok in _UNARY:
                v, d = stack.pop()
                stack.append(_UNARY[tok](v, d))
            elif tok in _BINARY:
                b, db = stack.pop()
                a, da = stack.pop()
                stack.append(_BINARY[tok](a, da, b, db))
            else:
                c = float(tok)          # raises ValueError on an unknown token
                stack.append((np.full_like(x, c), np.zeros_like(x)))
    if len(stack) != 1:
        raise ValueError(f"malformed chain {program!r}: {len(stack)} values left on the stack")
    y, d = stack[0]
    return np.array(y, dtype=np.float64), np.array(d, dtype=np.float64)
