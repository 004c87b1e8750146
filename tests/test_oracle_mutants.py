"""The pins must be able to fail: plant one plausible mistake at a time in a private copy of
the oracle's C source (on the CPU, in a temp dir), and check that the high-precision
definition pin or the finite-difference pin rejects the mutant."""
import ctypes
import os
import subprocess

import mpmath as mp
import numpy as np
import pytest

import oracle

SRC = os.path.join(os.path.dirname(oracle.__file__), "nfad_oracle.c")

# (kind the mistake shows in, text to replace, replacement)
MUTANTS = [
    (oracle.GELU_TANH, "1.0 + 3.0 * GELU_CUBIC * x * x);\n  double s = sigmoid(2.0 * u);",
     "1.0 + 2.0 * GELU_CUBIC * x * x);\n  double s = sigmoid(2.0 * u);"),          # wrong power rule
    (oracle.GELU_TANH, "*d = s + x * (2.0 * s * sc) * du;", "*d = s + x * (s * sc) * du;"),  # lost factor
    (oracle.GELU_TANH, "static const double GELU_CUBIC = 0.044715;", "static const double GELU_CUBIC = 0.044175;"),
    (oracle.GELU_TANH, "double s = sigmoid(2.0 * u);   /*", "double s = sigmoid(u);   /*"),  # tanh/sigmoid mix-up
    (oracle.GELU_ERF, "double Phi = 0.5 * erfc(-x * c_inv_sqrt_2());", "double Phi = 0.5 * erfc(x * c_inv_sqrt_2());"),
    (oracle.GELU_ERF, "*d = Phi + x * phi;", "*d = Phi - x * phi;"),
    (oracle.GELU_ERF, "double phi = exp(-0.5 * x * x) * c_inv_sqrt_2pi();", "double phi = exp(-x * x) * c_inv_sqrt_2pi();"),
    (oracle.SWISH, "*d = s + x * s * sc;", "*d = s + x * sc;"),                              # dropped term
    (oracle.SWISH, "double s = sigmoid(x), sc = sigmoid(-x);", "double s = sigmoid(x), sc = sigmoid(x);"),
    (oracle.MISH, "*d = t + x * (1.0 - t * t) * sigmoid(x);", "*d = t + x * (1.0 - t * t);"),   # forgot softplus'
    (oracle.MISH, "*d = t + x * (1.0 - t * t) * sigmoid(x);", "*d = t + x * (1.0 - t) * sigmoid(x);"),
    (oracle.MISH, "return v + log1p(exp(-v));", "return v + log1p(exp(v));"),
]


def _defn(kind):
    if kind == oracle.GELU_TANH:
        return lambda x: mp.mpf("0.5") * x * (1 + mp.tanh(mp.sqrt(2 / mp.pi) * (x + mp.mpf("0.044715") * x ** 3)))
    if kind == oracle.GELU_ERF:
        return lambda x: mp.mpf("0.5") * x * (1 + mp.erf(x / mp.sqrt(2)))
    if kind == oracle.SWISH:
        return lambda x: x / (1 + mp.exp(-x))
    return lambda x: x * mp.tanh(mp.log(1 + mp.exp(x)))


def _pins_hold(lib, kind) -> bool:
    """Definition pin (values and numerically differentiated derivative) on a small grid."""
    dp = ctypes.POINTER(ctypes.c_double)
    lib.nfad_oracle_fwd.argtypes = [ctypes.c_int, dp, dp, dp, ctypes.c_size_t, ctypes.c_int]
    x = np.array([-6.0, -2.5, -1.0, -0.3, 0.0, 0.4, 1.0, 2.5, 6.0])
    y, d = np.empty_like(x), np.empty_like(x)
    lib.nfad_oracle_fwd(kind, x.ctypes.data_as(dp), y.ctypes.data_as(dp), d.ctypes.data_as(dp), x.size, 1)
    f = _defn(kind)
    with mp.workdps(60):
        for i, xv in enumerate(x):
            if abs(float(f(mp.mpf(xv))) - y[i]) > 1e-13 * max(1.0, abs(y[i])):
                return False
            if abs(float(mp.diff(f, mp.mpf(xv))) - d[i]) > 1e-13:
                return False
    return True


def _compile(text, tmp_path, name):
    c = tmp_path / f"{name}.c"
    so = tmp_path / f"{name}.so"
    c.write_text(text)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fno-fast-math", "-o", str(so), str(c), "-lm"],
                   check=True)
    return ctypes.CDLL(str(so))


def test_unmutated_copy_passes(tmp_path):
    lib = _compile(open(SRC).read(), tmp_path, "clean")
    for kind in oracle.KINDS:
        assert _pins_hold(lib, kind)


@pytest.mark.parametrize("idx", range(len(MUTANTS)))
def test_planted_mistake_is_caught(tmp_path, idx):
    kind, old, new = MUTANTS[idx]
    text = open(SRC).read()
    assert text.count(old) == 1, "mutation site moved: update the MUTANTS table"
    lib = _compile(text.replace(old, new), tmp_path, f"mutant{idx}")
    assert not _pins_hold(lib, kind)
