"""Pins for the oracle's bound propagation (CPU only).

P1 closed form for affine-only networks (tight, all three norms)
P2 eps = 0 collapses every bound to a separately written forward pass
P3 at eps = 0 the bound weights equal the Jacobian (autograd on that forward pass)
P6 sampled perturbations stay inside [lower, upper]
P7 dense enumeration on a tiny model stays inside the bounds
P8 identities: dual norms vs numpy.linalg.norm, softmax shift invariance, sign split = centre/radius
"""
import numpy as np
import pytest
import torch

import plain_forward as pf
from oracle import bounds as B
from oracle import verifier as V
from oracle.verifier import _Ctx
from tv_synth import CONFIGS, make_model, make_positions, make_tokens, scaled
from tv_synth.generate import randomize_layernorm


def tiny(act=0, layers=1, D=16, H=2, F=24, L=5, P=1, stress=6.0, seed=0):
    w = scaled(CONFIGS["c1"], n_layers=layers, hidden=D, n_heads=H, ffn=F, activation=act, seq_len=L,
               n_perturbed=P, vocab=50, max_len=16, act_alpha=0.1)
    m = randomize_layernorm(make_model(w, seed_offset=seed, stress=stress), seed)
    return w, m, make_tokens(w, 2, seed)[0], make_positions(w, 1)[0]


# ---------------------------------------------------------------- P1
@pytest.mark.parametrize("p,q", [(0, 1), (2, 2), (1, np.inf)])
def test_p1_affine_closed_form_tight(p, q):
    rng = np.random.default_rng(7)
    L, E, P, eps = 4, 6, 2, 0.3
    x0 = rng.standard_normal((L, E))
    positions = [1, 3]
    W1, c1 = rng.standard_normal((5, E)), rng.standard_normal(5)
    W2, c2 = rng.standard_normal((3, 5)), rng.standard_normal(3)
    X = B.input_bounds(x0, positions)
    Y = B.affine(B.affine(X, W1, c1), W2, c2)
    l, u = B.concretize(Y, eps, P, p)
    Weff = W2 @ W1
    centre = x0 @ Weff.T + (W2 @ c1 + c2)
    for t in range(L):
        for j in range(3):
            rad = eps * np.linalg.norm(Weff[j], ord=q) if t in positions else 0.0
            assert abs(u[t, j] - (centre[t, j] + rad)) < 1e-12
            assert abs(l[t, j] - (centre[t, j] - rad)) < 1e-12
    # tightness: the maximiser of a linear form over the ball attains u
    w = Weff[1]
    if p == 0:
        d = eps * np.sign(w)
    elif p == 2:
        d = eps * w / np.linalg.norm(w)
    else:
        d = np.zeros(E); i = np.argmax(np.abs(w)); d[i] = eps * np.sign(w[i])
    xp = x0.copy(); xp[1] += d
    assert abs((xp @ Weff.T + (W2 @ c1 + c2))[1, 1] - u[1, 1]) < 1e-12
    # a sum of positions: token 0 reads both perturbed tokens through a mixing matrix (P blocks add)
    mix = rng.standard_normal((1, L))
    Z = B.Bounds(np.einsum("ot,tdc->odc", mix, Y.lw), mix @ Y.lb, np.einsum("ot,tdc->odc", mix, Y.uw), mix @ Y.ub)
    lz, uz = B.concretize(Z, eps, P, p)
    rad = eps * sum(abs(mix[0, t]) * np.linalg.norm(Weff[2], ord=q) for t in positions)
    assert abs(uz[0, 2] - lz[0, 2] - 2 * rad) < 1e-12


def test_p1_sign_split_mixes_bounds():
    """Eq. (2) with distinct lower/upper inputs: brute force over the box of a 3-input neuron."""
    rng = np.random.default_rng(3)
    lb = rng.standard_normal(3); ub = lb + rng.uniform(0.1, 1, 3)
    X = B.Bounds(np.zeros((3, 1)), lb, np.zeros((3, 1)), ub)
    W = np.array([[1.5, -2.0, 0.0], [-1.0, -1.0, 3.0]]); c = np.array([0.5, -0.25])
    Y = B.affine(X, W, c)
    corners = np.array(np.meshgrid(*[[lb[i], ub[i]] for i in range(3)])).reshape(3, -1).T
    vals = corners @ W.T + c
    np.testing.assert_allclose(Y.ub, vals.max(0)); np.testing.assert_allclose(Y.lb, vals.min(0))


# ---------------------------------------------------------------- P2 / P3
@pytest.mark.parametrize("act", [0, 1, 2, 3, 4])
def test_p2_p3_eps0_forward_and_jacobian(act):
    w, m, tokens, _ = tiny(act=act, layers=2, P=2)
    positions = [1, 3]
    trace = {}
    res = V.verify(m, tokens, positions, 2, 0.0, trace=trace)
    x0 = pf.embed(m, tokens)
    ref = pf.logits(m, x0).numpy()
    np.testing.assert_allclose(res["lower"], ref, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(res["upper"], ref, rtol=1e-10, atol=1e-12)
    assert res["status"] == 0 and res["label"] == int(np.argmax(ref))
    oth = 1 - res["label"]
    np.testing.assert_allclose(res["margin_lower"], [ref[res["label"]] - ref[oth]], rtol=1e-9, atol=1e-12)
    # Jacobian of the final hidden state w.r.t. the perturbed embeddings
    def f(xp):
        x = x0.clone()
        x[positions] = xp
        return pf.encoder(m, x)
    J = torch.autograd.functional.jacobian(f, x0[positions].clone()).numpy()   # [L, D, P, E]
    Xf = trace[f"l{w.enc.n_layers - 1}.x2"]
    Jr = J.reshape(Xf.lw.shape)
    np.testing.assert_allclose(Xf.lw, Jr, rtol=1e-8, atol=1e-10)
    np.testing.assert_allclose(Xf.uw, Jr, rtol=1e-8, atol=1e-10)
    np.testing.assert_allclose(Xf.lb, pf.encoder(m, x0).numpy(), rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------------- P6
@pytest.mark.parametrize("act,p,P,eps", [(0, 2, 1, 0.005), (0, 0, 2, 0.0008), (0, 1, 1, 0.008),
                                         (1, 0, 2, 0.0008), (1, 2, 1, 0.005), (2, 0, 2, 0.0008), (2, 2, 1, 0.005),
                                         (3, 2, 1, 0.005), (3, 0, 2, 0.0008), (4, 2, 1, 0.005), (4, 0, 2, 0.0008)])
def test_p6_sampling_soundness(act, p, P, eps):
    w, m, tokens, _ = tiny(act=act, layers=2, P=P)
    positions = [1, 3][:P]
    trace = {}
    res = V.verify(m, tokens, positions, p, eps, trace=trace)
    assert res["status"] == 0
    rng = np.random.default_rng(99)
    d = pf.sample_ball(rng, 4000, P, w.enc.hidden, p, eps)
    x0 = pf.embed(m, tokens)
    x = x0.unsqueeze(0).repeat(len(d), 1, 1)
    x[:, positions] += torch.as_tensor(d)
    hid = pf.encoder(m, x).numpy()
    Xf = trace[f"l{w.enc.n_layers - 1}.x2"]
    lh, uh = B.concretize(Xf, eps, P, p)
    assert np.all(hid >= lh - 1e-9) and np.all(hid <= uh + 1e-9)
    # the linear bounds themselves hold pointwise, not only their concretization
    dd = d.reshape(len(d), -1)
    assert np.all(hid >= Xf.lb + np.einsum("tdc,nc->ntd", Xf.lw, dd) - 1e-9)
    assert np.all(hid <= Xf.ub + np.einsum("tdc,nc->ntd", Xf.uw, dd) + 1e-9)
    y = (torch.as_tensor(hid)[:, 0] @ torch.as_tensor(m["Wc"].astype(np.float64)).T).numpy() + m["bc"]
    assert np.all(y >= res["lower"] - 1e-9) and np.all(y <= res["upper"] + 1e-9)
    lab, oth = res["label"], 1 - res["label"]
    assert np.all(y[:, lab] - y[:, oth] >= res["margin_lower"][0] - 1e-9)
    # bounds are informative: not wider than 1000x the sampled range
    ratio = (res["upper"] - res["lower"]) / (y.max(0) - y.min(0))
    print("bound width / sampled range:", ratio)
    assert np.all(ratio >= 1.0) and np.all(ratio < 1e3)


# ---------------------------------------------------------------- P7
@pytest.mark.parametrize("p,act", [(0, 1), (2, 1), (1, 1), (2, 0), (2, 3), (2, 4), (0, 4)])
def test_p7_bruteforce_tiny(p, act):
    w, m, tokens, _ = tiny(act=act, layers=1, D=3, H=1, F=4, L=3, P=1, stress=20.0, seed=3)
    eps = 0.01
    res = V.verify(m, tokens, [1], p, eps)
    g = np.linspace(-1, 1, 41)
    d = np.array(np.meshgrid(g, g, g)).reshape(3, -1).T
    nrm = {0: np.abs(d).max(1), 2: np.sqrt((d * d).sum(1)), 1: np.abs(d).sum(1)}[p]
    inside = d[nrm <= 1 + 1e-12]
    surf = d / np.maximum(nrm, 1e-30)[:, None]
    pts = np.concatenate([inside, surf[nrm > 0]]) * eps
    x0 = pf.embed(m, tokens)
    x = x0.unsqueeze(0).repeat(len(pts), 1, 1)
    x[:, 1] += torch.as_tensor(pts)
    y = pf.logits(m, x).numpy()
    assert np.all(y.min(0) >= res["lower"] - 1e-10) and np.all(y.max(0) <= res["upper"] + 1e-10)
    true_w = y.max(0) - y.min(0)
    print("bound width / true range:", (res["upper"] - res["lower"]) / true_w)
    assert np.all(res["upper"] - res["lower"] <= 50 * true_w + 1e-9)     # and not vacuous


# ---------------------------------------------------------------- P8
def test_p8_dual_norm_vs_numpy():
    rng = np.random.default_rng(5)
    w = rng.standard_normal((7, 3 * 5))
    for p, q in [(0, 1), (2, 2), (1, np.inf)]:
        ref = sum(np.linalg.norm(w[:, r * 5:(r + 1) * 5], ord=q, axis=1) for r in range(3))
        np.testing.assert_allclose(B.block_dual_norm(w, 3, p), ref, rtol=1e-14)
        # duality: sup over the ball of w.delta equals the dual norm (checked on the maximiser)
    with pytest.raises(ValueError):
        B.block_dual_norm(w, 3, 3)


def test_p8_softmax_shift_invariance_and_row_sum():
    rng = np.random.default_rng(11)
    L, PE = 6, 8
    lw = rng.standard_normal((4, L, PE)) * 0.3
    uw = lw + rng.uniform(0, 0.05, lw.shape)
    lb = rng.standard_normal((4, L)); ub = lb + rng.uniform(0, 0.1, lb.shape)
    S = B.Bounds(lw, lb, uw, ub)
    ctx = _Ctx(0.1, 2, 0)
    P1, l1, u1 = V.softmax_bound(S, ctx)
    S2 = B.Bounds(lw, lb + 3.7, uw, ub + 3.7)
    P2, l2, u2 = V.softmax_bound(S2, ctx)
    np.testing.assert_allclose(P1.lw, P2.lw, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(l1, l2, rtol=1e-9, atol=1e-12); np.testing.assert_allclose(u1, u2, rtol=1e-9, atol=1e-12)
    assert np.all(l1 >= 0) and np.all(u1 <= 1) and np.all(l1 <= u1)
    # at eps=0 with lw==uw, lb==ub the bound is the exact softmax
    S0 = B.Bounds(lw, lb, lw, lb)
    P0, l0, u0 = V.softmax_bound(S0, _Ctx(0.0, 2, 0))
    e = np.exp(lb - lb.max(-1, keepdims=True)); sm = e / e.sum(-1, keepdims=True)
    np.testing.assert_allclose(l0, sm, rtol=1e-12); np.testing.assert_allclose(u0, sm, rtol=1e-12)


def test_p8_sign_split_equals_centre_radius():
    rng = np.random.default_rng(13)
    lw = rng.standard_normal((5, 9, 4)); uw = rng.standard_normal((5, 9, 4))     # unordered on purpose
    lb = rng.standard_normal((5, 9)); ub = rng.standard_normal((5, 9))
    W = rng.standard_normal((6, 9)); c = rng.standard_normal(6)
    Y = B.affine(B.Bounds(lw, lb, uw, ub), W, c)
    S, R = 0.5 * (uw + lw), 0.5 * (uw - lw)
    np.testing.assert_allclose(Y.uw, W @ S + np.abs(W) @ R, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(Y.lw, W @ S - np.abs(W) @ R, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- search
def test_certify_bisection_and_monotone_margin():
    w, m, tokens, _ = tiny(act=0, layers=2, stress=4.0)
    eps_c, label = V.certify(m, tokens, [1], 2, 0.0, 1.0, 10)
    print("certified eps", eps_c)
    assert 0.0 < eps_c < 0.5
    k = round(eps_c * 1024)
    assert abs(eps_c - k / 1024) < 1e-15                       # a dyadic mid-point (or eps_lo)
    if eps_c > 0:
        assert V.is_verified(V.verify(m, tokens, [1], 2, eps_c, label))
    assert not V.is_verified(V.verify(m, tokens, [1], 2, eps_c + 1 / 1024, label))
    # P9 (diagnostic turned into a check on this case): margin lower bound shrinks as eps grows
    ml = [V.verify(m, tokens, [1], 2, e, label)["margin_lower"][0] for e in (0.0, 0.002, 0.01, 0.05)]
    assert all(a >= b - 1e-12 for a, b in zip(ml, ml[1:]))


def test_status_flag_on_blow_up():
    w, m, tokens, _ = tiny(act=0, layers=2, stress=30.0)
    res = V.verify(m, tokens, [1], 0, 50.0)
    if res["status"] == 1:
        assert np.all(np.isinf(res["lower"])) and np.all(np.isinf(res["upper"])) and not V.is_verified(res)
    else:
        assert np.all(np.isfinite(res["lower"]))
