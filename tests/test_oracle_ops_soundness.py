"""Per-operator soundness pins for the oracle (CPU only).

Each bound rule is fed input states whose true values are known functions of
the perturbation: any value between a lower and an upper line in delta (both
lines are attained by samples at every delta).  The rule's
output bounds must then hold pointwise for the exact operator applied to
x(delta), over ball vertices / surface / interior and extreme slack values.
Wide input ranges make every McCormick plane, sign swap and clamp matter, which
whole-network sampling (dominated by loose LayerNorm bounds) does not.
"""
import math

import numpy as np
import pytest

import plain_forward as pf
from oracle import bounds as B
from oracle import relaxations as rx
from oracle import verifier as V
from oracle.verifier import _Ctx

P_, E_ = 2, 3
PE = P_ * E_
N = 6000
TOL = 1e-9


class Sampled:
    """A bound state plus exact samples of neurons it bounds.

    lw, uw, lb, ub are drawn freely subject to lower(delta) <= upper(delta) on the whole ball
    (ub - lb >= eps * N(uw - lw)); any value between the two lines is a legitimate neuron value, so
    samples sit on the lower line, on the upper line, or in between.  Both lines are therefore
    attained exactly at every delta."""

    def __init__(self, rng, shape, eps, p, wscale=1.0, slack=0.2, offset=0.0, bscale=1.0):
        w = rng.standard_normal(shape + (PE,)) * wscale
        dl = rng.standard_normal(shape + (PE,)) * 0.3 * wscale
        du = rng.standard_normal(shape + (PE,)) * 0.3 * wscale
        b = rng.standard_normal(shape) * bscale + offset
        s = np.abs(rng.standard_normal(shape)) * slack
        lw, uw = w + dl, w + du
        gap = eps * B.block_dual_norm(uw - lw, P_, p)
        lb = b - s - 0.5 * gap
        ub = b + s + 0.5 * gap
        self.state = B.Bounds(lw, lb, uw, ub)

    def values(self, rng, delta):
        st = self.state
        lo = st.lb + np.einsum("...c,nc->n...", st.lw, delta)
        up = st.ub + np.einsum("...c,nc->n...", st.uw, delta)
        assert np.all(lo <= up + 1e-12)
        t = rng.uniform(0, 1, lo.shape)
        ext = rng.random(t.shape) < 0.6
        t = np.where(ext, np.round(t), t)
        return lo + t * (up - lo)


def deltas(rng, p, eps):
    return pf.sample_ball(rng, N, P_, E_, p, eps).reshape(N, PE)


def check(out, y, delta, what):
    lo = out.lb + np.einsum("...c,nc->n...", out.lw, delta)
    up = out.ub + np.einsum("...c,nc->n...", out.uw, delta)
    scale = 1.0 + np.abs(y).max()
    assert np.all(lo <= y + TOL * scale), f"{what}: lower bound violated by {np.max(lo - y)}"
    assert np.all(up >= y - TOL * scale), f"{what}: upper bound violated by {np.max(y - up)}"
    # report tightness so a vacuous rule would be seen
    return float(np.mean(up - lo)), float(np.mean(y.max(0) - y.min(0)))


@pytest.mark.parametrize("p", [0, 2, 1])
@pytest.mark.parametrize("name", ["relu", "tanh", "exp", "square"])
def test_elementwise_rules_sound(name, p):
    rng = np.random.default_rng(100 + p)
    eps = 0.4
    X = Sampled(rng, (40,), eps, p)
    d = deltas(rng, p, eps)
    x = X.values(rng, d)
    l, u = B.concretize(X.state, eps, P_, p)
    assert np.all(x >= l - 1e-12) and np.all(x <= u + 1e-12)
    f = {"relu": lambda t: np.maximum(t, 0), "tanh": np.tanh, "exp": np.exp, "square": lambda t: t * t}[name]
    out = B.relax(X.state, getattr(rx, name), l, u)
    check(out, f(x), d, name)


@pytest.mark.parametrize("p", [0, 2])
@pytest.mark.parametrize("name", ["reciprocal", "sqrt"])
def test_positive_domain_rules_sound(name, p):
    rng = np.random.default_rng(200 + p)
    eps = 0.3
    X = Sampled(rng, (40,), eps, p, wscale=0.3, slack=0.1, offset=3.0, bscale=0.3)
    d = deltas(rng, p, eps)
    x = X.values(rng, d)
    l, u = B.concretize(X.state, eps, P_, p)
    assert l.min() > 0
    f = {"reciprocal": lambda t: 1 / t, "sqrt": np.sqrt}[name]
    check(B.relax(X.state, getattr(rx, name), l, u), f(x), d, name)


@pytest.mark.parametrize("p", [0, 2, 1])
def test_scale_shift_and_affine_sound(p):
    rng = np.random.default_rng(300 + p)
    eps = 0.5
    X = Sampled(rng, (5, 7), eps, p)
    d = deltas(rng, p, eps)
    x = X.values(rng, d)
    a = rng.standard_normal(7); c = rng.standard_normal(7)
    check(B.scale_shift(X.state, a, c), a * x + c, d, "scale_shift")
    W = rng.standard_normal((4, 7)); cc = rng.standard_normal(4)
    check(B.affine(X.state, W, cc), x @ W.T + cc, d, "affine")


@pytest.mark.parametrize("p", [0, 2, 1])
def test_bilinear_rules_sound(p):
    rng = np.random.default_rng(400 + p)
    eps = 0.5
    L, dh = 4, 3
    Q = Sampled(rng, (L, dh), eps, p); K = Sampled(rng, (L, dh), eps, p)
    d = deltas(rng, p, eps)
    q, k = Q.values(rng, d), K.values(rng, d)
    lq, uq = B.concretize(Q.state, eps, P_, p)
    lk, uk = B.concretize(K.state, eps, P_, p)
    w1, r1 = check(B.dot_qk(Q.state, K.state, lq, lk, uk), np.einsum("nid,njd->nij", q, k), d, "dot_qk")
    Pm = Sampled(rng, (L, L), eps, p, wscale=0.3, offset=0.2)
    Vv = Sampled(rng, (L, dh), eps, p)
    pm, vv = Pm.values(rng, d), Vv.values(rng, d)
    lp, up = B.concretize(Pm.state, eps, P_, p)
    lv, uv = B.concretize(Vv.state, eps, P_, p)
    check(B.dot_pv(Pm.state, Vv.state, lp, lv, uv), np.einsum("nij,njd->nid", pm, vv), d, "dot_pv")
    x, y = Q.values(rng, d), K.values(rng, d)
    check(B.product(Q.state, K.state, lq, lk, uk), x * y, d, "product")
    assert w1 < 30 * r1


@pytest.mark.parametrize("p", [0, 2, 1])
def test_softmax_rule_sound(p):
    rng = np.random.default_rng(500 + p)
    eps = 0.3
    S = Sampled(rng, (3, 5), eps, p, wscale=0.7, slack=0.3)
    d = deltas(rng, p, eps)
    s = S.values(rng, d)
    Pb, lp, up = V.softmax_bound(S.state, _Ctx(eps, P_, p))
    e = np.exp(s - s.max(-1, keepdims=True)); sm = e / e.sum(-1, keepdims=True)
    wid, rng_ = check(Pb, sm, d, "softmax")
    assert np.all(sm >= lp - 1e-12) and np.all(sm <= up + 1e-12)
    assert wid < 20 * rng_


@pytest.mark.parametrize("p", [0, 2, 1])
@pytest.mark.parametrize("case", ["wide", "narrow", "low_variance"])
def test_layernorm_rule_sound(case, p):
    rng = np.random.default_rng(600 + p)
    eps = 0.2
    kw = {"wide": dict(wscale=0.5, slack=0.2), "narrow": dict(wscale=0.02, slack=0.01),
          "low_variance": dict(wscale=0.003, slack=0.001, bscale=0.004)}[case]
    X = Sampled(rng, (3, 8), eps, p, **kw)
    d = deltas(rng, p, eps)
    x = X.values(rng, d)
    gamma = rng.standard_normal(8); beta = rng.standard_normal(8)
    ln_eps = 1e-5
    out = V.layernorm_bound(X.state, gamma, beta, ln_eps, _Ctx(eps, P_, p))
    mu = x.mean(-1, keepdims=True); xc = x - mu
    y = xc / np.sqrt((xc * xc).mean(-1, keepdims=True) + ln_eps) * gamma + beta
    check(out, y, d, "layernorm/" + case)


@pytest.mark.parametrize("p", [0, 2, 1])
def test_gelu_rule_sound(p):
    rng = np.random.default_rng(700 + p)
    eps = 0.4
    X = Sampled(rng, (60,), eps, p)
    d = deltas(rng, p, eps)
    x = X.values(rng, d)
    out = V.gelu_bound(X.state, _Ctx(eps, P_, p))
    y = 0.5 * x * (1 + np.tanh(math.sqrt(2 / math.pi) * (x + 0.044715 * x ** 3)))
    check(out, y, d, "gelu")


@pytest.mark.parametrize("p", [0, 2, 1])
def test_silu_and_leaky_relu_rules_sound(p):
    rng = np.random.default_rng(750 + p)
    eps = 0.4
    X = Sampled(rng, (60,), eps, p, bscale=2.0)
    d = deltas(rng, p, eps)
    x = X.values(rng, d)
    ctx = _Ctx(eps, P_, p)
    wid_s, rng_s = check(V.silu_bound(X.state, ctx), x / (1 + np.exp(-x)), d, "silu")
    assert wid_s < 20 * rng_s                      # and not vacuous
    out = V.activation_bound(X.state, V.ACT_LEAKY_RELU, ctx, alpha=0.2)
    check(out, np.where(x >= 0, x, 0.2 * x), d, "leaky relu")
    # the chain collapses to the exact tangent of x sigmoid(x) on a point interval (one neuron, eps = 0)
    x0 = np.array([-3.0, -1.2, 0.0, 0.7, 4.0])
    Pt = B.Bounds(np.ones((5, PE)), x0, np.ones((5, PE)), x0)
    Y = V.silu_bound(Pt, _Ctx(0.0, P_, p))
    sg = 1 / (1 + np.exp(-x0))
    np.testing.assert_allclose(Y.lb, x0 * sg, rtol=1e-12, atol=1e-14); np.testing.assert_allclose(Y.ub, Y.lb, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(Y.lw[:, 0], sg + x0 * sg * (1 - sg), rtol=1e-10)
    np.testing.assert_allclose(Y.uw, Y.lw, rtol=1e-10, atol=1e-14)


@pytest.mark.parametrize("p", [0, 2, 1])
def test_bilinear_rules_sound_single_term(p):
    """One contracted index: no slack from other terms hides a wrong plane or a wrong side."""
    rng = np.random.default_rng(800 + p)
    eps = 0.5
    L = 6
    Q = Sampled(rng, (L, 1), eps, p); K = Sampled(rng, (L, 1), eps, p)
    d = deltas(rng, p, eps)
    q, k = Q.values(rng, d), K.values(rng, d)
    lq, uq = B.concretize(Q.state, eps, P_, p)
    lk, uk = B.concretize(K.state, eps, P_, p)
    check(B.dot_qk(Q.state, K.state, lq, lk, uk), np.einsum("nid,njd->nij", q, k), d, "dot_qk")
    Pm = Sampled(rng, (L, 1), eps, p); Vv = Sampled(rng, (1, 4), eps, p)
    pm, vv = Pm.values(rng, d), Vv.values(rng, d)
    lp, up = B.concretize(Pm.state, eps, P_, p)
    lv, uv = B.concretize(Vv.state, eps, P_, p)
    check(B.dot_pv(Pm.state, Vv.state, lp, lv, uv), np.einsum("nij,njd->nid", pm, vv), d, "dot_pv")


@pytest.mark.parametrize("p", [0, 2])
def test_attention_block_sound(p):
    """Whole self-attention sub-layer (projections, per-head dot products, softmax, mixing, output
    projection) against a numpy attention on sampled inputs."""
    from tv_synth import CONFIGS, make_model, scaled
    rng = np.random.default_rng(900 + p)
    eps = 0.1
    L, D, H = 3, 4, 2
    w = scaled(CONFIGS["c1"], n_layers=1, hidden=D, n_heads=H, ffn=4, seq_len=L, vocab=10, max_len=4)
    m = make_model(w, stress=15.0)
    X = Sampled(rng, (L, D), eps, p, wscale=0.6, slack=0.05)
    d = deltas(rng, p, eps)
    x = X.values(rng, d)
    out = V.attention_bound(X.state, m, 0, _Ctx(eps, P_, p))
    g = lambda n: m[f"l0.{n}"].astype(np.float64)
    q = x @ g("Wq").T + g("bq"); k = x @ g("Wk").T + g("bk"); v = x @ g("Wv").T + g("bv")
    dh = D // H
    o = np.zeros_like(x)
    for h in range(H):
        sl = slice(h * dh, (h + 1) * dh)
        sc = np.einsum("nid,njd->nij", q[..., sl], k[..., sl]) / math.sqrt(dh)
        e = np.exp(sc - sc.max(-1, keepdims=True))
        o[..., sl] = np.einsum("nij,njd->nid", e / e.sum(-1, keepdims=True), v[..., sl])
    y = o @ g("Wo").T + g("bo")
    wid, r = check(out, y, d, "attention")
    print('attention width / range', wid / r)
    assert wid < 100 * r
