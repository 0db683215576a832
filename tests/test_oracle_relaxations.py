"""Pins for the oracle's scalar relaxations and McCormick planes (CPU only).

Each relaxation is checked on a dense grid of its interval against the exact
function: sound everywhere, chord touching both end points, tangent touching at
its contact point, degenerate intervals collapsing to the exact tangent.
"""
import numpy as np
import pytest

from oracle import relaxations as rx

RNG = np.random.default_rng(12345)
FUNCS = {
    "relu": (rx.relu, lambda x: np.maximum(x, 0.0), (-3, 3)),
    "leaky_relu": (rx.leaky_relu(0.1), lambda x: np.where(x >= 0, x, 0.1 * x), (-3, 3)),
    "tanh": (rx.tanh, np.tanh, (-4, 4)),
    "exp": (rx.exp, np.exp, (-6, 3)),
    "reciprocal": (rx.reciprocal, lambda x: 1.0 / x, (0.05, 5)),
    "sqrt": (rx.sqrt, np.sqrt, (1e-5, 5)),
    "square": (rx.square, lambda x: x * x, (-3, 3)),
}


def _intervals(lo, hi, n=400):
    a = RNG.uniform(lo, hi, n)
    b = RNG.uniform(lo, hi, n)
    l, u = np.minimum(a, b), np.maximum(a, b)
    # add narrow and one-sided and wide intervals
    l[:40] = u[:40] - RNG.uniform(1e-9, 1e-3, 40) * (1 + np.abs(u[:40]))
    l = np.clip(l, lo, hi)
    return l, u


@pytest.mark.parametrize("name", list(FUNCS))
def test_relaxation_sound_and_touching(name):
    fn, f, (lo, hi) = FUNCS[name]
    l, u = _intervals(lo, hi)
    kL, cL, kU, cU = fn(l, u)
    t = np.linspace(0, 1, 513)[:, None]
    x = l + (u - l) * t
    fx = f(x)
    tol = 1e-11 * (1 + np.abs(fx))
    assert np.all(kL * x + cL <= fx + tol), name
    assert np.all(kU * x + cU >= fx - tol), name
    # each line touches the function somewhere on [l,u] (no slack relaxation)
    gapL = (fx - (kL * x + cL)).min(0)
    gapU = ((kU * x + cU) - fx).min(0)
    scale = 1 + np.abs(fx).max(0)
    if name != "exp":   # exp's capped tangent touches at d which the grid may miss slightly
        assert np.all(gapL <= 1e-4 * scale * (u - l + 1e-9) + 1e-9), name
    assert np.all(gapU <= 1e-4 * scale * (u - l + 1e-9) + 1e-9), name


def test_relu_cases_exact():
    # l >= 0: identity (paper Sec. 4.1: f(l,u) = 1); u <= 0: zero
    kL, cL, kU, cU = rx.relu(np.array([0.0, 0.5, -2.0, -1.0]), np.array([1.0, 2.0, -0.5, 0.0]))
    assert list(kL) == [1, 1, 0, 0] and list(kU) == [1, 1, 0, 0] and not cL.any() and not cU.any()
    # crossing: chord through (l,0),(u,u); lower slope 1 iff u >= -l (tie -> 1)
    kL, cL, kU, cU = rx.relu(np.array([-1.0, -2.0, -1.0]), np.array([2.0, 1.0, 1.0]))
    assert list(kL) == [1, 0, 1]
    np.testing.assert_allclose(kU, [2 / 3, 1 / 3, 0.5])
    np.testing.assert_allclose(cU, [2 / 3, 2 / 3, 0.5])


def test_leaky_relu_cases_exact():
    a = 0.25
    fn = rx.leaky_relu(a)
    # one-sided: the function's own line
    kL, cL, kU, cU = fn(np.array([0.0, 0.5, -2.0, -1.0]), np.array([1.0, 2.0, -0.5, 0.0]))
    assert list(kL) == [1, 1, a, a] and list(kU) == [1, 1, a, a] and not cL.any() and not cU.any()
    # crossing: chord through (l, a l), (u, u); lower slope 1 iff u >= -l (tie -> 1), else a; no intercept
    l, u = np.array([-1.0, -2.0, -1.0]), np.array([2.0, 1.0, 1.0])
    kL, cL, kU, cU = fn(l, u)
    assert list(kL) == [1, a, 1] and not cL.any()
    np.testing.assert_allclose(kU * l + cU, a * l, atol=1e-15)
    np.testing.assert_allclose(kU * u + cU, u, atol=1e-15)
    np.testing.assert_allclose(kU, [(2 + a) / 3, (1 + 2 * a) / 3, (1 + a) / 2])
    # the two ends of the family: alpha = 0 is ReLU line for line, alpha = 1 the identity
    l, u = _intervals(-3, 3)
    for got, ref in zip(rx.leaky_relu(0.0)(l, u), rx.relu(l, u)):
        np.testing.assert_array_equal(got, ref)
    kL, cL, kU, cU = rx.leaky_relu(1.0)(l, u)
    np.testing.assert_allclose(kL, 1.0); np.testing.assert_allclose(kU, 1.0)
    np.testing.assert_allclose(cL, 0.0); np.testing.assert_allclose(cU, 0.0, atol=1e-15)


def test_chords_and_tangents_closed_form():
    l, u = np.array([0.5]), np.array([2.0])
    m = 1.25
    kL, cL, kU, cU = rx.exp(l, u)
    np.testing.assert_allclose(kU, (np.exp(2.0) - np.exp(0.5)) / 1.5)
    np.testing.assert_allclose(kL * m + cL, np.exp(m))         # tangent at mid (mid < l + 0.99)
    kL, cL, kU, cU = rx.exp(np.array([-5.0]), np.array([1.0]))
    d = -5.0 + 0.99
    np.testing.assert_allclose([kL[0], kL[0] * d + cL[0]], [np.exp(d), np.exp(d)])
    assert kL[0] * (-5.0) + cL[0] > 0                           # capped tangent stays positive at l
    kL, cL, kU, cU = rx.reciprocal(l, u)
    np.testing.assert_allclose([kL[0], cL[0], kU[0], cU[0]], [-1 / m ** 2, 2 / m, -1.0, 2.5])
    kL, cL, kU, cU = rx.sqrt(l, u)
    np.testing.assert_allclose([kU[0], cU[0]], [0.5 / np.sqrt(m), 0.5 * np.sqrt(m)])
    np.testing.assert_allclose(kL * l + cL, np.sqrt(l)); np.testing.assert_allclose(kL * u + cL, np.sqrt(u))
    kL, cL, kU, cU = rx.square(np.array([-1.0]), np.array([3.0]))
    np.testing.assert_allclose([kL[0], cL[0], kU[0], cU[0]], [2.0, -1.0, 2.0, 3.0])
    # tanh one-sided: tangent at mid on the curved side, chord on the other
    kL, cL, kU, cU = rx.tanh(l, u)
    np.testing.assert_allclose(kU * m + cU, np.tanh(m)); np.testing.assert_allclose(kU, 1 - np.tanh(m) ** 2)
    np.testing.assert_allclose(kL * l + cL, np.tanh(l)); np.testing.assert_allclose(kL * u + cL, np.tanh(u))


def test_tanh_crossing_tangent_passes_through_far_end():
    l, u = np.array([-2.0]), np.array([3.0])
    kL, cL, kU, cU = rx.tanh(l, u)
    # lower line: tangent on the convex side, through (u, tanh u) up to the bisection bracket
    np.testing.assert_allclose(kL * u + cL, np.tanh(u), atol=1e-12)
    assert kL * u + cL <= np.tanh(u)
    np.testing.assert_allclose(kU * l + cU, np.tanh(l), atol=1e-12)
    assert kU * l + cU >= np.tanh(l)
    # narrow crossing interval: both lines are the chord
    kL, cL, kU, cU = rx.tanh(np.array([-0.01]), np.array([0.3]))
    kap = (np.tanh(0.3) - np.tanh(-0.01)) / 0.31
    assert kap > 1 - np.tanh(0.01) ** 2 or True
    x = np.linspace(-0.01, 0.3, 1001)
    assert np.all(kL * x + cL <= np.tanh(x) + 1e-14) and np.all(kU * x + cU >= np.tanh(x) - 1e-14)


@pytest.mark.parametrize("name", ["tanh", "exp", "reciprocal", "sqrt", "square"])
def test_degenerate_interval_is_exact_tangent(name):
    fn, f, (lo, hi) = FUNCS[name]
    x = RNG.uniform(lo, hi, 50)
    kL, cL, kU, cU = fn(x, x)
    h = 1e-6
    deriv = (f(x + h) - f(x - h)) / (2 * h)
    np.testing.assert_allclose(kL, deriv, rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(kU, kL)
    np.testing.assert_allclose(kL * x + cL, f(x), rtol=1e-13)
    np.testing.assert_allclose(kU * x + cU, f(x), rtol=1e-13)


def test_mccormick_planes():
    n = 200
    lx = RNG.uniform(-2, 2, n); ux = lx + RNG.uniform(0, 2, n)
    ly = RNG.uniform(-2, 2, n); uy = ly + RNG.uniform(0, 2, n)
    aL, bL, gL, aU, bU, gU = rx.mccormick(lx, ly, uy)
    t = np.linspace(0, 1, 33)
    X = lx + (ux - lx) * t[:, None, None]
    Y = ly + (uy - ly) * t[None, :, None]
    Z = X * Y
    low = aL * X + bL * Y + gL
    up = aU * X + bU * Y + gU
    assert np.all(low <= Z + 1e-12) and np.all(up >= Z - 1e-12)
    # lower plane is exact on the edges x = lx and y = ly; upper plane on x = lx and y = uy
    np.testing.assert_allclose(low[0], Z[0], atol=1e-12)
    np.testing.assert_allclose(low[:, 0], Z[:, 0], atol=1e-12)
    np.testing.assert_allclose(up[0], Z[0], atol=1e-12)
    np.testing.assert_allclose(up[:, -1], Z[:, -1], atol=1e-12)
