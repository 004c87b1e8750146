"""Pins for the chain oracle (the fp64 postfix dual-number interpreter): it must agree with the
pinned closed-form oracle on the chains that spell the four activations, and with mpmath
(expression written independently as a Python function, derivative by numerical
differentiation at 50 digits) on every chain the library carries."""
import mpmath as mp
import numpy as np
import pytest

import oracle
from oracle import chain
import paper_2209_10778_amd as nfad

mp.mp.dps = 50

# independent spellings, by chain name
MP = {
    "sigmoid": lambda x: 1 / (1 + mp.exp(-x)),
    "tanh": lambda x: mp.tanh(x),
    "softplus": lambda x: mp.log(1 + mp.exp(x)),
    "exp": lambda x: mp.exp(x),
    "swish_table1": lambda x: x / (1 + mp.exp(-x)),
    "swish_sigmoid": lambda x: x / (1 + mp.exp(-x)),
    "mish_table1": lambda x: x * mp.tanh(mp.log(1 + mp.exp(x))),
    "gelu_tanh_table1": lambda x: mp.mpf("0.5") * x * (1 + mp.tanh(mp.sqrt(2 / mp.pi) * (x + mp.mpf("0.044715") * x ** 3))),
    "gelu_erf": lambda x: mp.mpf("0.5") * x * (1 + mp.erf(x / mp.sqrt(2))),
    "tanhshrink": lambda x: x - mp.tanh(x),
    "logsigmoid": lambda x: -mp.log(1 + mp.exp(-x)),
    "elu": lambda x: x if x > 0 else mp.exp(x) - 1,
    "hardswish": lambda x: x * min(max(x + 3, 0), 6) / 6,
    "softsign": lambda x: x / (1 + abs(x)),
}
KINKS = {"elu": (0.0,), "hardswish": (-3.0, 3.0), "softsign": (0.0,)}
SAME_AS_KIND = {"swish_table1": oracle.SWISH, "swish_sigmoid": oracle.SWISH, "mish_table1": oracle.MISH,
                "gelu_tanh_table1": oracle.GELU_TANH, "gelu_erf": oracle.GELU_ERF}


def library_chains():
    return [(i, nfad.nfad_chain_name(i), nfad.nfad_chain_program(i)) for i in range(nfad.nfad_chain_count())]


def test_every_library_chain_has_an_independent_spelling():
    names = [n for _, n, _ in library_chains()]
    assert sorted(names) == sorted(MP) and len(set(names)) == len(names)
    assert nfad.nfad_chain_name(-1) is None and nfad.nfad_chain_program(len(names)) is None


@pytest.mark.parametrize("cid,name,program", library_chains())
def test_interpreter_matches_mpmath(cid, name, program):
    xs = np.array([-9.5, -4.0, -1.7, -0.6, -0.01, 0.0, 0.02, 0.5, 1.3, 3.0, 7.25])
    xs = np.array([v for v in xs if v not in KINKS.get(name, ())])     # no derivative at a kink
    y, d = chain.eval_chain(program, xs)
    f = MP[name]
    for i, xv in enumerate(xs):
        yr, dr = f(mp.mpf(float(xv))), mp.diff(f, mp.mpf(float(xv)))
        assert abs(float(yr) - y[i]) <= 4e-15 * max(1.0, abs(float(yr))) + 1e-16 * abs(xv), (name, "y", xv)
        assert abs(float(dr) - d[i]) <= 4e-15 * max(1.0, abs(float(dr))) + 1e-15, (name, "d", xv)


@pytest.mark.parametrize("name,kind", sorted(SAME_AS_KIND.items()))
def test_activation_chains_match_the_closed_form_oracle(name, kind):
    program = dict((n, p) for _, n, p in library_chains())[name]
    x = np.linspace(-30.0, 30.0, 6001)
    y, d = chain.eval_chain(program, x)
    yr, dr = oracle.fwd(kind, x)
    # the chains are spelled as printed (1 + tanh, 1 + erf): absolute agreement where those cancel
    assert np.max(np.abs(y - yr)) <= 1e-14 * 30 and np.max(np.abs(d - dr)) <= 1e-13


def test_product_rule_and_quotient_rule_by_hand():
    # d/dx [x * x] = 2x ; d/dx [1/x] = -1/x^2 ; d/dx [exp(2x)] = 2 exp(2x)
    x = np.array([0.5, -1.5, 3.0])
    y, d = chain.eval_chain("x x *", x)
    assert np.array_equal(y, x * x) and np.array_equal(d, 2 * x)
    y, d = chain.eval_chain("1 x /", x)
    assert np.allclose(y, 1 / x, rtol=1e-15) and np.allclose(d, -1 / x ** 2, rtol=1e-15)
    y, d = chain.eval_chain("2 x * exp", x)
    assert np.allclose(d, 2 * np.exp(2 * x), rtol=1e-15)
    y, d = chain.eval_chain("x log", np.array([0.25, 2.0]))
    assert np.allclose(d, [4.0, 0.5])


def test_piecewise_primitives_at_their_kinks():
    x = np.array([-2.0, 0.0, 3.0])
    assert chain.eval_chain("x relu", x)[1].tolist() == [0.0, 0.0, 1.0]
    assert chain.eval_chain("x abs", x)[1].tolist() == [-1.0, 0.0, 1.0]
    assert chain.eval_chain("x 0 max", x)[1].tolist() == [0.0, 1.0, 1.0]       # first operand on a tie
    assert chain.eval_chain("0 x max", x)[1].tolist() == [0.0, 0.0, 1.0]
    assert chain.eval_chain("x 3 min", x)[1].tolist() == [1.0, 1.0, 1.0]
    v, d = chain.eval_chain("x x * sqrt", np.array([-2.0, 3.0]))                 # |x|
    assert np.allclose(v, [2.0, 3.0]) and np.allclose(d, [-1.0, 1.0])


def test_malformed_programs_are_rejected():
    for bad in ("x x", "x +", "x foo", ""):
        with pytest.raises((ValueError, IndexError)):
            chain.eval_chain(bad, [1.0])


def test_saturation_of_symbolic_primitives():
    x = np.array([-800.0, -80.0, 80.0, 800.0])
    for prog in ("x sigmoid", "x tanh", "x softplus", "x sigmoid x *", "x x softplus tanh *"):
        y, d = chain.eval_chain(prog, x)
        assert np.all(np.isfinite(y)) and np.all(np.isfinite(d)), prog


# ------------------------------------------------------------------ random compositions
def mp_eval(program, x):
    """The program's value at the mpmath number x (a second, value-only reading of the postfix
    grammar; the tangent is NOT propagated here: it comes from numerical differentiation)."""
    un = {"neg": lambda a: -a, "exp": mp.exp, "log": mp.log, "tanh": mp.tanh,
          "sigmoid": lambda a: 1 / (1 + mp.exp(-a)), "softplus": lambda a: mp.log(1 + mp.exp(a)),
          "erf": mp.erf, "relu": lambda a: a if a > 0 else mp.mpf(0), "abs": abs, "sqrt": mp.sqrt}
    bi = {"+": lambda a, b: a + b, "-": lambda a, b: a - b, "*": lambda a, b: a * b, "/": lambda a, b: a / b,
          "min": min, "max": max}
    st = []
    for tok in program.split():
        if tok == "x":
            st.append(x)
        elif tok in un:
            st.append(un[tok](st.pop()))
        elif tok in bi:
            b = st.pop()
            a = st.pop()
            st.append(bi[tok](a, b))
        else:
            st.append(mp.mpf(tok))
    assert len(st) == 1
    return st[0]


def test_interpreter_matches_mpmath_on_random_compositions():
    """Forty random chains over all primitives: value against the mpmath evaluation, tangent
    against numerical differentiation at 50 digits; points where the two one-sided derivatives
    differ (a kink of relu/abs/min/max) are skipped."""
    from chain_programs import random_programs
    xs = np.array([-5.43, -4.37, -1.913, -0.577, -0.0731, 0.318, 1.234, 2.718, 5.77])
    checked = 0
    for program in random_programs(40):
        y, d = chain.eval_chain(program, xs)
        f = lambda t: mp_eval(program, t)
        for i, xv in enumerate(xs):
            xm = mp.mpf(float(xv))
            left, right = mp.diff(f, xm, direction=-1, h=mp.mpf(10) ** -20), mp.diff(f, xm, direction=1, h=mp.mpf(10) ** -20)
            if abs(left - right) > mp.mpf(10) ** -12:
                continue
            yr, dr = f(xm), (left + right) / 2
            assert abs(float(yr) - y[i]) <= 2e-14 * max(1.0, abs(float(yr))), (program, "y", xv)
            assert abs(float(dr) - d[i]) <= 2e-13 * max(1.0, abs(float(dr))), (program, "d", xv)
            checked += 1
    assert checked > 300


@pytest.mark.parametrize("token", sorted(chain._UNARY) + sorted(chain._BINARY))
def test_a_planted_tangent_mistake_in_any_rule_is_caught(token, monkeypatch):
    """Each primitive's rule in turn gets its tangent scaled by 1.001 (or, for the selecting
    rules, taken from the other operand); the random-composition pin must then fail."""
    table = chain._UNARY if token in chain._UNARY else chain._BINARY
    good = table[token]
    if token in ("min", "max"):
        bad = lambda a, da, b, db: (good(a, da, b, db)[0], good(a, db, b, da)[1])
    elif token in ("relu", "abs"):
        bad = lambda v, d: (good(v, d)[0], d)
    else:
        bad = lambda *args: (good(*args)[0], 1.001 * good(*args)[1])
    monkeypatch.setitem(table, token, bad)
    with pytest.raises(AssertionError):
        test_interpreter_matches_mpmath_on_random_compositions()
