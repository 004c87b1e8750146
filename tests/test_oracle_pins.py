"""Pins for the fp64 oracle: each test ties it to something other than itself.

Independent sources used here:
  * the unrewritten definitions of Table I (and x*Phi(x)) evaluated at 150 digits with
    mpmath, and their derivatives obtained by mpmath's numerical differentiation (so the
    oracle's hand-derived f' is never retyped);
  * scipy.special / numpy library routines (expit, ndtr, erf, logaddexp, tanh);
  * closed-form fixed points, asymptotes, symmetries, the Swish derivative of Table II,
    central finite differences, and the equality of the three gradients of
    Sec. II-C (eq. 2 = eq. 4).
"""
import os

import mpmath as mp
import numpy as np
import pytest
import scipy.optimize
import scipy.special as sps

import oracle

mp.mp.dps = 150
K = oracle
NAMES = {v: k for k, v in oracle.KIND_NAMES.items()}
SYMMETRIC = (K.GELU_TANH, K.GELU_ERF, K.SWISH)


# ---------------------------------------------------------------- definitions, 150 digits
def _def(kind):
    if kind == K.GELU_TANH:  # Table I
        return lambda x: mp.mpf("0.5") * x * (1 + mp.tanh(mp.sqrt(2 / mp.pi) * (x + mp.mpf("0.044715") * x ** 3)))
    if kind == K.GELU_ERF:  # textbook x*Phi(x)
        return lambda x: mp.mpf("0.5") * x * (1 + mp.erf(x / mp.sqrt(2)))
    if kind == K.SWISH:  # Table I
        return lambda x: x / (1 + mp.exp(-x))
    if kind == K.MISH:  # Table I
        return lambda x: x * mp.tanh(mp.log(1 + mp.exp(x)))
    raise AssertionError


GRID = np.concatenate([
    np.linspace(-12.0, 12.0, 97),
    np.array([-80.0, -60.0, -37.5, -25.0, -20.0, -16.0, 16.0, 20.0, 25.0, 37.5, 60.0, 80.0]),
    np.array([-1e-3, -1e-8, 1e-8, 1e-3, 0.7524614220710163, 1.2784645427610738]),
])


@pytest.mark.parametrize("kind", oracle.KINDS)
def test_matches_unrewritten_definition_at_high_precision(kind):
    f = _def(kind)
    y, d = oracle.fwd(kind, GRID)
    for i, xv in enumerate(GRID):
        xm = mp.mpf(float(xv))
        y_ref = f(xm)
        d_ref = mp.diff(f, xm)
        # relative to the exact value; where 1+tanh / 1+erf cancel below the 150 working
        # digits (GELU for x << -12) the reference itself is only good to 1e-140 absolute.
        for got, ref, what in ((y[i], y_ref, "y"), (d[i], d_ref, "dydx")):
            err = abs(mp.mpf(float(got)) - ref)
            # exp() of an argument of size ~x^2 carries the argument's rounding: allow for it
            tol = mp.mpf("4e-15") * max(1.0, float(xv) ** 2 / 4) * abs(ref) + mp.mpf("1e-140")
            # dydx passes through zero: there the relative bound is on the two terms it is made of
            if what == "dydx":
                tol += mp.mpf("4e-16")
            assert err <= tol, (oracle.KIND_NAMES[kind], what, xv, got, mp.nstr(ref, 20))
    assert np.all(np.isfinite(y)) and np.all(np.isfinite(d))


def test_fixed_points_golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "fixed_points.txt")
    rows = [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 4
    for name, x, y_ref, d_ref in rows:
        y, d = oracle.fwd(NAMES[name], [float(x)])
        assert y[0] == float(y_ref)
        assert abs(d[0] - float(d_ref)) <= 1e-16, (name, d[0])
    # Mish'(0) = tanh(ln 2) = 3/5
    assert abs(np.tanh(np.log(2.0)) - 0.6) < 1e-15


@pytest.mark.parametrize("kind", oracle.KINDS)
def test_central_finite_differences(kind):
    x = np.linspace(-12.0, 12.0, 4801)
    h = 1e-5 * np.maximum(1.0, np.abs(x))
    yp, _ = oracle.fwd(kind, x + h)
    ym, _ = oracle.fwd(kind, x - h)
    _, d = oracle.fwd(kind, x)
    fd = (yp - ym) / ((x + h) - (x - h))
    assert np.max(np.abs(fd - d) / np.maximum(1.0, np.abs(d))) <= 1e-8


@pytest.mark.parametrize("kind", oracle.KINDS)
def test_asymptotes_and_saturation(kind):
    xp = np.array([20.0, 40.0, 80.0, 700.0])
    y, d = oracle.fwd(kind, xp)
    assert np.all(np.isfinite(y)) and np.all(np.isfinite(d))
    assert np.all(np.abs(y - xp) <= 1e-7) and np.all(np.abs(d - 1.0) <= 1e-7)
    assert y[2] == 80.0 and d[2] == 1.0
    xn = -xp
    y, d = oracle.fwd(kind, xn)
    assert np.all(np.isfinite(y)) and np.all(np.isfinite(d))
    assert np.all(y <= 0.0) and np.all(d <= 0.0)       # approaches zero from below
    assert np.all(np.abs(y) <= 1e-7) and np.all(np.abs(d) <= 1e-7)
    # Swish and Mish at -80 are tiny but normal numbers: x*e^x
    if kind in (K.SWISH, K.MISH):
        assert abs(y[2] / (-80.0 * np.exp(-80.0)) - 1.0) < 1e-12


@pytest.mark.parametrize("kind", SYMMETRIC)
def test_symmetry_invariants(kind):
    # f(x) = x*s(x) with s(x) + s(-x) = 1  =>  f(x) - f(-x) = x and f'(x) + f'(-x) = 1
    x = np.linspace(0.0, 30.0, 3001)
    yp, dp = oracle.fwd(kind, x)
    yn, dn = oracle.fwd(kind, -x)
    assert np.max(np.abs((yp - yn) - x) / np.maximum(1.0, x)) <= 4e-16
    assert np.max(np.abs((dp + dn) - 1.0)) <= 4e-16


def test_mish_is_not_symmetric():
    # guards against wiring Mish to a sigmoid-gated form; residuals checked against mpmath
    f = _def(K.MISH)
    x = 1.7
    yp, dp = oracle.fwd(K.MISH, [x])
    yn, dn = oracle.fwd(K.MISH, [-x])
    r_y = float(f(mp.mpf(x)) - f(mp.mpf(-x)) - mp.mpf(x))
    r_d = float(mp.diff(f, mp.mpf(x)) + mp.diff(f, mp.mpf(-x)) - 1)
    assert abs(r_y) > 0.1 and abs(r_d) > 1e-3
    assert abs((yp[0] - yn[0] - x) - r_y) < 1e-15
    assert abs((dp[0] + dn[0] - 1.0) - r_d) < 1e-15


@pytest.mark.parametrize("kind", oracle.KINDS)
def test_dual_number_propagation_agrees_with_closed_form(kind):
    # Sec. II-D: seed tangent 1, product and chain rule node by node
    rng = np.random.default_rng(7)
    x = np.concatenate([rng.normal(0.0, 3.0, 20000), np.linspace(-80, 80, 3201)])
    y, d = oracle.fwd(kind, x)
    y2, d2 = oracle.fwd_dual(kind, x)
    # the two derivations differ in form (1+tanh vs sigmoid etc.), so compare with an
    # absolute floor where 1+tanh / 1+erf cancel (x << 0) and relatively elsewhere
    assert np.max(np.abs(y - y2) / np.maximum(np.abs(y), 1.0)) <= 1e-14
    assert np.max(np.abs(d - d2) / np.maximum(np.abs(d), 1.0)) <= 1e-14
    sel = x > -3.0
    assert np.max(np.abs(y[sel] - y2[sel]) / np.maximum(np.abs(y[sel]), 1e-30)) <= 1e-13


def test_library_special_cases():
    x = np.linspace(-12.0, 12.0, 4801)   # the deep tails are pinned by the mpmath test
    y, d = oracle.fwd(K.SWISH, x)
    s = sps.expit(x)
    assert np.allclose(y, x * s, rtol=1e-14, atol=0)
    # Table II: sigma + x*sigma*(1-sigma); the printed form loses |x|*eps in 1-sigma
    assert np.max(np.abs(d - (s + x * s * (1 - s)))) <= 1e-14
    y, d = oracle.fwd(K.GELU_ERF, x)
    assert np.allclose(y, x * sps.ndtr(x), rtol=1e-13, atol=0)
    assert np.max(np.abs(d - (sps.ndtr(x) + x * np.exp(-x * x / 2) / np.sqrt(2 * np.pi)))) <= 1e-14
    y, _ = oracle.fwd(K.MISH, x)
    assert np.allclose(y, x * np.tanh(np.logaddexp(0.0, x)), rtol=1e-13, atol=0)
    y, _ = oracle.fwd(K.GELU_TANH, x)
    ref = 0.5 * x * (1 + np.tanh(np.sqrt(2 / np.pi) * (x + 0.044715 * x ** 3)))
    assert np.max(np.abs(y - ref)) <= 1e-14


def test_mish_rational_identity():
    # tanh(ln(1+e^x)) = ((1+e^x)^2 - 1) / ((1+e^x)^2 + 1)
    x = np.linspace(-30.0, 15.0, 4501)
    y, _ = oracle.fwd(K.MISH, x)
    q = (1 + np.exp(x)) ** 2
    n = np.exp(x) * (np.exp(x) + 2)          # q - 1 without cancellation
    assert np.allclose(y, x * n / (q + 1), rtol=1e-14, atol=0)


def test_tanh_and_erf_gelu_are_distinct_and_wired_correctly():
    x = np.arange(-6.0, 6.0, 1e-3)
    yt, dt = oracle.fwd(K.GELU_TANH, x)
    ye, de = oracle.fwd(K.GELU_ERF, x)
    ref_t = 0.5 * x * (1 + np.tanh(np.sqrt(2 / np.pi) * (x + 0.044715 * x ** 3)))
    ref_e = x * sps.ndtr(x)
    gap_ref = np.max(np.abs(ref_t - ref_e))
    gap = np.max(np.abs(yt - ye))
    assert 4.5e-4 < gap_ref < 5.0e-4 and abs(gap - gap_ref) < 1e-12
    assert abs(abs(x[np.argmax(np.abs(yt - ye))]) - 2.70) < 0.05
    assert 8e-4 < np.max(np.abs(dt - de)) < 9.5e-4
    assert np.max(np.abs(yt - ref_t)) < 1e-14 and np.max(np.abs(ye - ref_e)) < 1e-14


@pytest.mark.parametrize("kind", oracle.KINDS)
def test_minimum_where_derivative_vanishes(kind):
    dfun = lambda v: oracle.fwd(kind, [v])[1][0]
    xs = scipy.optimize.brentq(dfun, -3.0, -0.1, xtol=1e-15, rtol=1e-15)
    f = _def(kind)
    xs_ref = mp.findroot(lambda v: mp.diff(f, v), mp.mpf(xs))
    assert abs(xs - float(xs_ref)) < 1e-12
    ymin = oracle.fwd(kind, [xs])[0][0]
    assert abs(ymin - float(f(xs_ref))) < 1e-15
    if kind == K.SWISH:  # at the minimum 1 + x(1-sigma) = 0, hence f = x + 1
        assert abs(ymin - (xs + 1.0)) < 1e-12
    # it is a minimum: values either side are larger
    assert oracle.fwd(kind, [xs - 0.1])[0][0] > ymin < oracle.fwd(kind, [xs + 0.1])[0][0]


@pytest.mark.parametrize("kind", oracle.KINDS)
def test_extrema_of_the_derivative(kind):
    """The derivative overshoots 1 on the right and dips below 0 on the left; location and height of
    both extrema against the 150-digit definition (root of the second derivative)."""
    f = _def(kind)
    dfun = lambda v: oracle.fwd(kind, [v])[1][0]
    hi = scipy.optimize.minimize_scalar(lambda v: -dfun(v), bounds=(0.5, 4.0), method="bounded",
                                        options={"xatol": 1e-10})
    lo = scipy.optimize.minimize_scalar(dfun, bounds=(-4.0, -0.5), method="bounded", options={"xatol": 1e-10})
    x_hi = mp.findroot(lambda v: mp.diff(f, v, 2), mp.mpf(hi.x))
    x_lo = mp.findroot(lambda v: mp.diff(f, v, 2), mp.mpf(lo.x))
    assert abs(hi.x - float(x_hi)) < 1e-5 and abs(lo.x - float(x_lo)) < 1e-5
    assert abs(dfun(float(x_hi)) - float(mp.diff(f, x_hi))) < 1e-14
    assert abs(dfun(float(x_lo)) - float(mp.diff(f, x_lo))) < 1e-14
    assert 1.08 < dfun(float(x_hi)) < 1.13 and -0.13 < dfun(float(x_lo)) < -0.09
    if kind in SYMMETRIC:       # f'(x) + f'(-x) = 1: the dip mirrors the overshoot
        assert abs(float(x_hi) + float(x_lo)) < 1e-12
        assert abs(dfun(float(x_hi)) + dfun(float(x_lo)) - 1.0) < 1e-14


def test_bwd_is_plain_product():
    rng = np.random.default_rng(11)
    gy, dd = rng.normal(size=1000), rng.normal(size=1000)
    gx = oracle.bwd(gy, dd)
    for i in range(1000):          # brute force, element by element
        assert gx[i] == gy[i] * dd[i]
    assert oracle.bwd([], []).size == 0


@pytest.mark.parametrize("kind", oracle.KINDS)
def test_three_gradients_agree(kind):
    # Sec. II-C: back-propagation (eq. 2), recomputation and forward-AD (eq. 4) give the
    # same x' up to rounding.
    rng = np.random.default_rng(3)
    x = rng.normal(0.0, 2.0, 50000)
    gy = rng.normal(0.0, 1.0, 50000)
    y, d = oracle.fwd(kind, x)
    g_fad = oracle.bwd(gy, d)
    g_rec = oracle.recompute_bwd(kind, gy, x)
    y_sa, saved = oracle.saveall_fwd(kind, x)
    g_sa = oracle.saveall_bwd(kind, gy, saved)
    assert np.array_equal(g_fad, g_rec)
    assert np.max(np.abs(g_sa - g_fad)) <= 1e-14
    assert np.max(np.abs(y_sa - y)) <= 1e-15
    assert np.array_equal(oracle.recompute_fwd(kind, x), y)
    assert np.array_equal(saved[0], x)


def test_saved_sets_are_the_primitive_outputs():
    x = np.linspace(-9.0, 9.0, 1801)
    assert [oracle.num_saved(k) for k in oracle.KINDS] == [4, 3, 2, 2]
    _, sv = oracle.saveall_fwd(K.SWISH, x)
    assert np.allclose(sv[1], sps.expit(x), rtol=1e-15, atol=0)
    _, sv = oracle.saveall_fwd(K.MISH, x)
    assert np.allclose(sv[1], np.tanh(np.logaddexp(0, x)), rtol=1e-14, atol=0)
    _, sv = oracle.saveall_fwd(K.GELU_ERF, x)
    assert np.array_equal(sv[1], 0.5 * x)
    assert np.max(np.abs(sv[2] - (1 + sps.erf(x / np.sqrt(2))))) <= 9e-16
    _, sv = oracle.saveall_fwd(K.GELU_TANH, x)
    t = np.tanh(np.sqrt(2 / np.pi) * (x + 0.044715 * x ** 3))
    assert np.max(np.abs(sv[1] - t)) <= 9e-16
    assert np.array_equal(sv[2], 0.5 * x)
    assert np.max(np.abs(sv[3] - (1 + t))) <= 9e-16


def test_threads_do_not_change_results():
    rng = np.random.default_rng(5)
    x = rng.normal(0, 3, 100003)
    for kind in oracle.KINDS:
        a = oracle.fwd(kind, x, threads=1)
        b = oracle.fwd(kind, x, threads=0)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert oracle.max_threads() >= 1


def test_bad_kind_is_rejected():
    with pytest.raises(ValueError):
        oracle.fwd(7, [0.0])
    with pytest.raises(ValueError):
        oracle.saveall_fwd(-1, [0.0])
