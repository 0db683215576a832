"""Scalar linear relaxations used by the bound propagation (float64, numpy).

TEST INFRASTRUCTURE: this is the slow reference the HIP path is checked
against.  Nothing in the product path may import it.

Each function takes arrays of concretized bounds l <= u and returns
(kL, cL, kU, cU) with  kL*x + cL <= f(x) <= kU*x + cU  for every x in [l, u].
This is the f(l, u) of the paper's "generalized elementwise multiplication"
pattern (Sec. 4.1, second pattern), extended with intercepts.

What the paper fixes: ReLU has two lower-bound designs chosen by comparing
|l| with |u| (Sec. 2.1, last paragraph) and slope 1 when l >= 0 (Sec. 4.1);
tanh uses tangent/chord lines between the concretized bounds (Sec. 4.1).
The figures with the exact lines are lost; the lines below are the standard
tightest-area choices and are pinned by soundness tests, not by the paper
("parity unpinned" for the tightness choice itself).
"""
import numpy as np

TAU = 1e-12          # relative width under which an interval counts as a point
BISECT_ITERS = 60    # tangent-point search for tanh
EXP_TANGENT_CAP = 0.99   # exp lower tangent at min(mid, l + 0.99): keeps the line positive on [l, u]


def _degenerate(l, u):
    scale = np.maximum(1.0, np.maximum(np.abs(l), np.abs(u)))
    return (u - l) <= TAU * scale


def _tangent_both(f, df, l, u):
    """Degenerate-width rule: slope f'(m) for both lines, intercepts min/max of f(x)-k*x on {l, m, u}."""
    m = 0.5 * (l + u)
    k = df(m)
    r = np.stack([f(l) - k * l, f(m) - k * m, f(u) - k * u])
    return k, r.min(0), k, r.max(0)


def _merge(deg, dk, dcl, dcu, kL, cL, kU, cU):
    return (np.where(deg, dk, kL), np.where(deg, dcl, cL),
            np.where(deg, dk, kU), np.where(deg, dcu, cU))


def relu(l, u):
    """ReLU: identity when l >= 0, zero when u <= 0; crossing: upper = chord through (l,0),(u,u);
    lower = k*x with k = 1 if u >= -l else 0 (the two designs selected by the range)."""
    l = np.asarray(l, np.float64); u = np.asarray(u, np.float64)
    pos = l >= 0
    neg = (u <= 0) & ~pos
    cross = ~pos & ~neg
    den = np.where(cross, u - l, 1.0)
    kU = np.where(pos, 1.0, np.where(neg, 0.0, u / den))
    cU = np.where(cross, -l * u / den, 0.0)
    kL = np.where(pos, 1.0, np.where(neg, 0.0, np.where(u >= -l, 1.0, 0.0)))
    cL = np.zeros_like(kL)
    return kL, cL, kU, cU


def leaky_relu(alpha):
    """Leaky ReLU f(x) = x (x >= 0), alpha x (x < 0) with 0 <= alpha <= 1 (convex; one of the further activations
    the paper's operator list names, Sec. 4.1).  Same design as ReLU: identity when l >= 0, the line alpha x when
    u <= 0; crossing: upper = chord through (l, alpha l), (u, u); lower = k x with k = 1 if u >= -l else alpha
    (both support the function at 0).  alpha = 0 is ReLU."""
    assert 0.0 <= alpha <= 1.0

    def fn(l, u):
        l = np.asarray(l, np.float64); u = np.asarray(u, np.float64)
        pos = l >= 0
        neg = (u <= 0) & ~pos
        cross = ~pos & ~neg
        den = np.where(cross, u - l, 1.0)
        kc = (u - alpha * l) / den
        kU = np.where(pos, 1.0, np.where(neg, alpha, kc))
        cU = np.where(cross, (alpha - 1.0) * l * u / den, 0.0)
        kL = np.where(pos, 1.0, np.where(neg, alpha, np.where(u >= -l, 1.0, alpha)))
        return kL, np.zeros_like(kL), kU, cU
    return fn


def _dtanh(x):
    t = np.tanh(x)
    return 1.0 - t * t


def _tanh_tangent_through(end, lo, hi, sound_lo):
    """Tangent point d in [lo, hi] whose tangent line passes through (end, tanh end).

    g(d) = tanh d + tanh'(d) (end - d) - tanh(end) changes sign once on the bracket.
    Bisection; returns the bracket end on the sound side (sound_lo: the lower end).
    """
    te = np.tanh(end)
    lo = lo.copy(); hi = hi.copy()

    def g(d):
        return np.tanh(d) + _dtanh(d) * (end - d) - te

    glo = g(lo)
    for _ in range(BISECT_ITERS):
        mid = 0.5 * (lo + hi)
        same = np.sign(g(mid)) == np.sign(glo)
        lo = np.where(same, mid, lo)
        hi = np.where(same, hi, mid)
    return lo if sound_lo else hi


def tanh(l, u):
    """tanh: convex on x<=0, concave on x>=0.
    l>=0: upper tangent at mid, lower chord.  u<=0: lower tangent at mid, upper chord.
    crossing: lower = chord if chord slope <= tanh'(l) else tangent at d in [l,0] through (u, tanh u);
              upper = chord if chord slope <= tanh'(u) else tangent at d in [0,u] through (l, tanh l)."""
    l = np.asarray(l, np.float64); u = np.asarray(u, np.float64)
    deg = _degenerate(l, u)
    dk, dcl, _, dcu = _tangent_both(np.tanh, _dtanh, l, u)
    ls = np.where(deg, -1.0, l); us = np.where(deg, 1.0, u)   # safe stand-ins where degenerate
    tl, tu = np.tanh(ls), np.tanh(us)
    m = 0.5 * (ls + us)
    kap = (tu - tl) / (us - ls)
    chord_c = tl - kap * ls
    tan_k = _dtanh(m); tan_c = np.tanh(m) - tan_k * m
    pos = ls >= 0
    neg = (us <= 0) & ~pos
    cross = ~pos & ~neg
    # crossing case, lower line: tangent on the convex side through the upper end point
    lc = np.where(cross, ls, -1.0); uc = np.where(cross, us, 1.0)
    dL = _tanh_tangent_through(uc, lc, np.zeros_like(lc), sound_lo=True)
    dU = _tanh_tangent_through(lc, np.zeros_like(uc), uc, sound_lo=False)
    kapc = (np.tanh(uc) - np.tanh(lc)) / (uc - lc)
    low_chord = kapc <= _dtanh(lc)
    up_chord = kapc <= _dtanh(uc)
    kL_cross = np.where(low_chord, kapc, _dtanh(dL))
    cL_cross = np.where(low_chord, np.tanh(lc) - kapc * lc, np.tanh(dL) - _dtanh(dL) * dL)
    kU_cross = np.where(up_chord, kapc, _dtanh(dU))
    cU_cross = np.where(up_chord, np.tanh(lc) - kapc * lc, np.tanh(dU) - _dtanh(dU) * dU)
    kL = np.where(pos, kap, np.where(neg, tan_k, kL_cross))
    cL = np.where(pos, chord_c, np.where(neg, tan_c, cL_cross))
    kU = np.where(pos, tan_k, np.where(neg, kap, kU_cross))
    cU = np.where(pos, tan_c, np.where(neg, chord_c, cU_cross))
    return _merge(deg, dk, dcl, dcu, kL, cL, kU, cU)


def exp(l, u):
    """exp (convex): upper = chord; lower = tangent at d = min(mid, l + 0.99)."""
    l = np.asarray(l, np.float64); u = np.asarray(u, np.float64)
    deg = _degenerate(l, u)
    dk, dcl, _, dcu = _tangent_both(np.exp, np.exp, l, u)
    us = np.where(deg, l + 1.0, u)
    el, eu = np.exp(l), np.exp(us)
    kU = (eu - el) / (us - l)
    cU = el - kU * l
    d = np.minimum(0.5 * (l + us), l + EXP_TANGENT_CAP)
    kL = np.exp(d)
    cL = kL * (1.0 - d)
    return _merge(deg, dk, dcl, dcu, kL, cL, kU, cU)


def reciprocal(l, u):
    """1/x on 0 < l <= u (convex, decreasing): lower = tangent at mid, upper = chord."""
    l = np.asarray(l, np.float64); u = np.asarray(u, np.float64)
    deg = _degenerate(l, u)
    dk, dcl, _, dcu = _tangent_both(lambda x: 1.0 / x, lambda x: -1.0 / (x * x), l, u)
    m = 0.5 * (l + u)
    kL = -1.0 / (m * m); cL = 2.0 / m
    kU = -1.0 / (l * u); cU = 1.0 / l + 1.0 / u
    return _merge(deg, dk, dcl, dcu, kL, cL, kU, cU)


def sqrt(l, u):
    """sqrt on 0 < l <= u (concave): upper = tangent at mid, lower = chord."""
    l = np.asarray(l, np.float64); u = np.asarray(u, np.float64)
    deg = _degenerate(l, u)
    dk, dcl, _, dcu = _tangent_both(np.sqrt, lambda x: 0.5 / np.sqrt(x), l, u)
    m = 0.5 * (l + u)
    sl, su, sm = np.sqrt(l), np.sqrt(u), np.sqrt(m)
    kU = 0.5 / sm; cU = 0.5 * sm
    kL = 1.0 / (sl + su); cL = sl * su / (sl + su)
    return _merge(deg, dk, dcl, dcu, kL, cL, kU, cU)


def square(l, u):
    """x^2 (convex): lower = tangent at mid, upper = chord."""
    l = np.asarray(l, np.float64); u = np.asarray(u, np.float64)
    deg = _degenerate(l, u)
    dk, dcl, _, dcu = _tangent_both(lambda x: x * x, lambda x: 2.0 * x, l, u)
    m = 0.5 * (l + u)
    kL = 2.0 * m; cL = -m * m
    kU = l + u; cU = -l * u
    return _merge(deg, dk, dcl, dcu, kL, cL, kU, cU)


def mccormick(lx, ly, uy):
    """Planes for z = x*y on the box [lx,ux] x [ly,uy]  (one fixed pair):
         z >= ly*x + lx*y - lx*ly        z <= uy*x + lx*y - lx*uy
    Returns (aL, bL, gL, aU, bU, gU): coefficient on x, on y, and constant, for each plane."""
    return ly, lx, -lx * ly, uy, lx, -lx * uy
