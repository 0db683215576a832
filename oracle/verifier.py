"""verify / certify: forward linear-bound propagation through a transformer encoder (float64).

TEST INFRASTRUCTURE: the reference the HIP path is checked against; only tests,
the smoke check and the benchmark's CPU-baseline leg may call it.

Problem statement (paper Sec. 1 and Sec. 2.1, "Transformer Verification"):
given a sentence, a model and a perturbation ball of radius eps around the
embeddings of P chosen positions, produce lower/upper bounds on the model
outputs that hold for every point of the ball (`verify`), and find the largest
eps for which the predicted class provably cannot change (`certify`).

The paper gives Eq. (1) (concretization) and Eq. (2) (affine rule) and names the
remaining operators; the encoder layout, softmax / LayerNorm / GELU
decompositions, head, decision rule and binary search below are this
implementation's reading (each stated where it is implemented below); they are pinned by
soundness, eps=0 collapse, the Jacobian at eps=0 and closed forms, not by
numbers printed in the paper.

Encoder (post-norm): a = x + Wo.Attn(x) + bo; x' = LN(a); f = x' + W2.act(W1.x' + b1) + b2; x'' = LN(f).
"""
import math

import numpy as np

from . import bounds as B
from . import relaxations as rx

ACT_RELU, ACT_TANH, ACT_GELU, ACT_LEAKY_RELU, ACT_SILU = 0, 1, 2, 3, 4
FLT_MAX = 3.4028234663852886e38
RECIP_MIN = 1e-12        # domain guard of the reciprocal relaxation
GELU_C = 0.044715


class NotFinite(Exception):
    """A concretized bound left the fp32 range or a reciprocal met a non-positive lower bound."""


def _check(*arrays):
    for a in arrays:
        if not np.all(np.abs(a) <= FLT_MAX):    # also False for NaN
            raise NotFinite()


class _Ctx:
    def __init__(self, eps, P, p, trace=None):
        self.eps, self.P, self.p, self.trace = float(eps), P, p, trace

    def conc(self, X):
        l, u = B.concretize(X, self.eps, self.P, self.p)
        _check(l, u)
        return l, u

    def rec(self, name, X):
        if self.trace is not None:
            self.trace[name] = X


def softmax_bound(S, ctx):
    """Softmax over the last neuron axis of S (rows = all leading axes).

    Input-reduction-compute operator (paper Sec. 3.2).  Steps: shift each row by max_j u_ij (a
    constant; exact softmax is invariant), exp relaxation, row sum (affine with ones), reciprocal
    relaxation, product e_ij * r_i.  Returns the bound state of p and its concretized bounds clamped
    to [0, 1] (the true softmax lies there; the linear forms are left unchanged)."""
    l, u = ctx.conc(S)
    shift = u.max(-1, keepdims=True)
    S = B.Bounds(S.lw, S.lb - shift, S.uw, S.ub - shift)
    l, u = l - shift, u - shift
    Eb = B.relax(S, rx.exp, l, u)
    le, ue = ctx.conc(Eb)
    ones = np.ones((1, S.shape[-1]))
    Sig = B.affine(Eb, ones)                       # [..., 1]
    ls, us = ctx.conc(Sig)
    if not np.all(ls >= RECIP_MIN):
        raise NotFinite()
    R = B.relax(Sig, rx.reciprocal, ls, us)
    lr, ur = ctx.conc(R)
    Pb = B.product(Eb, R, le, lr, ur)
    lp, up = ctx.conc(Pb)
    return Pb, np.clip(lp, 0.0, 1.0), np.clip(up, 0.0, 1.0)


def layernorm_bound(X, gamma, beta, ln_eps, ctx):
    """Full LayerNorm over the last neuron axis: y = gamma * (x - mean) / sqrt(var + ln_eps) + beta.

    Not in the paper (demanded by the benchmark configurations).  Steps: centring c = x - mean(x)
    as one affine map (I - 11^T/D); square relaxation; mean (affine); + ln_eps, concretized lower
    bound clamped to >= ln_eps; sqrt relaxation; reciprocal relaxation; product c_d * r; gamma, beta."""
    D = X.shape[-1]
    C = B.affine(X, np.eye(D) - np.full((D, D), 1.0 / D))
    lc, uc = ctx.conc(C)
    Qb = B.relax(C, rx.square, lc, uc)
    V = B.affine(Qb, np.full((1, D), 1.0 / D), np.array([ln_eps]))
    lv, uv = ctx.conc(V)
    lv = np.maximum(lv, ln_eps)
    uv = np.maximum(uv, lv)
    Sd = B.relax(V, rx.sqrt, lv, uv)
    lsd, usd = ctx.conc(Sd)
    lsd = np.maximum(lsd, math.sqrt(ln_eps))
    usd = np.maximum(usd, lsd)
    R = B.relax(Sd, rx.reciprocal, lsd, usd)
    lr, ur = ctx.conc(R)
    Y = B.product(C, R, lc, lr, ur)
    return B.scale_shift(Y, gamma, beta)


def gelu_bound(X, ctx):
    """tanh-form GELU y = 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3))) as a chain of relaxations:
    square -> affine -> product with x -> tanh -> affine -> product with x."""
    lx, ux = ctx.conc(X)
    A = B.relax(X, rx.square, lx, ux)
    k = math.sqrt(2.0 / math.pi)
    Bb = B.scale_shift(A, k * GELU_C, k)
    lb_, ub_ = ctx.conc(Bb)
    G = B.product(X, Bb, lx, lb_, ub_)
    lg, ug = ctx.conc(G)
    T = B.relax(G, rx.tanh, lg, ug)
    Hh = B.scale_shift(T, 0.5, 0.5)
    lh, uh = ctx.conc(Hh)
    return B.product(X, Hh, lx, lh, uh)


def silu_bound(X, ctx):
    """SiLU y = x * sigmoid(x) with sigmoid(x) = 0.5 (1 + tanh(x / 2)), as a chain of relaxations in the manner of
    the GELU chain: affine (x / 2) -> tanh -> affine -> product with x."""
    lx, ux = ctx.conc(X)
    Hx = B.scale_shift(X, 0.5)
    lh, uh = ctx.conc(Hx)
    T = B.relax(Hx, rx.tanh, lh, uh)
    G = B.scale_shift(T, 0.5, 0.5)
    lg, ug = ctx.conc(G)
    return B.product(X, G, lx, lg, ug)


def activation_bound(X, act, ctx, alpha=0.01):
    if act == ACT_GELU:
        return gelu_bound(X, ctx)
    if act == ACT_SILU:
        return silu_bound(X, ctx)
    l, u = ctx.conc(X)
    fn = {ACT_RELU: rx.relu, ACT_TANH: rx.tanh, ACT_LEAKY_RELU: rx.leaky_relu(alpha)}[act]
    return B.relax(X, fn, l, u)


def attention_bound(X, m, layer, ctx):
    cfg = m["cfg"]
    D, H = cfg.hidden, cfg.n_heads
    dh = D // H
    g = lambda n: m[f"l{layer}.{n}"].astype(np.float64)
    Q = B.affine(X, g("Wq"), g("bq"))
    K = B.affine(X, g("Wk"), g("bk"))
    V = B.affine(X, g("Wv"), g("bv"))
    ctx.rec(f"l{layer}.q", Q); ctx.rec(f"l{layer}.k", K); ctx.rec(f"l{layer}.v", V)
    lq, uq = ctx.conc(Q)
    lk, uk = ctx.conc(K)
    lv, uv = ctx.conc(V)
    outs = []
    for h in range(H):
        sl = (slice(None), slice(h * dh, (h + 1) * dh))
        S = B.dot_qk(Q[sl], K[sl], lq[sl], lk[sl], uk[sl])
        S = B.scale_shift(S, 1.0 / math.sqrt(dh))
        ctx.rec(f"l{layer}.s{h}", S)
        Pb, lp, up = softmax_bound(S, ctx)
        ctx.rec(f"l{layer}.p{h}", Pb)
        outs.append(B.dot_pv(Pb, V[sl], lp, lv[sl], uv[sl]))
    O = B.Bounds(np.concatenate([o.lw for o in outs], 1), np.concatenate([o.lb for o in outs], 1),
                 np.concatenate([o.uw for o in outs], 1), np.concatenate([o.ub for o in outs], 1))
    ctx.rec(f"l{layer}.o", O)
    return B.affine(O, g("Wo"), g("bo"))


def encoder_bounds(m, tokens, positions, p, eps, trace=None):
    """Bound state of the final hidden layer [L, D] for one sentence."""
    cfg = m["cfg"]
    L = len(tokens)
    x0 = m["tok_emb"][tokens].astype(np.float64) + m["pos_emb"][:L].astype(np.float64)
    ctx = _Ctx(eps, len(positions), p, trace)
    X = B.input_bounds(x0, positions)
    for layer in range(cfg.n_layers):
        g = lambda n: m[f"l{layer}.{n}"].astype(np.float64)
        A = B.add(attention_bound(X, m, layer, ctx), X)
        ctx.rec(f"l{layer}.a", A)
        X1 = layernorm_bound(A, g("ln1_g"), g("ln1_b"), cfg.ln_eps, ctx)
        ctx.rec(f"l{layer}.x1", X1)
        Hd = B.affine(X1, g("W1"), g("b1"))
        ctx.rec(f"l{layer}.h", Hd)
        Act = activation_bound(Hd, cfg.activation, ctx, getattr(cfg, "act_alpha", 0.01))
        ctx.rec(f"l{layer}.act", Act)
        F = B.add(B.affine(Act, g("W2"), g("b2")), X1)
        X = layernorm_bound(F, g("ln2_g"), g("ln2_b"), cfg.ln_eps, ctx)
        ctx.rec(f"l{layer}.x2", X)
    return X, ctx


def clean_logits(m, tokens):
    """Logits of the unperturbed sentence = the eps = 0 bounds (both sides coincide)."""
    X, ctx = encoder_bounds(m, tokens, [0], 2, 0.0)
    Y = B.affine(X[0], m["Wc"].astype(np.float64), m["bc"].astype(np.float64))
    return 0.5 * (Y.lb + Y.ub)


def verify(m, tokens, positions, p, eps, label=None, trace=None):
    """Bounds on the logits of one sentence over the perturbation set.

    Returns dict(lower [n_cls], upper [n_cls], margin_lower [n_cls-1], status, label).
    The head reads position 0.  Margins y_label - y_j (j != label, increasing j) are bounded as
    linear functions *before* concretization (rows W[label]-W[j] through Eq. (2), then Eq. (1)).
    status 1 = a bound left the fp32 range / a reciprocal domain guard failed: bounds are -inf/+inf.
    """
    cfg = m["cfg"]
    n_cls = cfg.n_classes
    Wc, bc = m["Wc"].astype(np.float64), m["bc"].astype(np.float64)
    if label is None:
        label = int(np.argmax(clean_logits(m, tokens)))
    others = [j for j in range(n_cls) if j != label]
    try:
        X, ctx = encoder_bounds(m, tokens, list(positions), p, eps, trace)
        Y = B.affine(X[0], Wc, bc)
        lo, up = ctx.conc(Y)
        Mg = B.affine(X[0], Wc[label][None, :] - Wc[others], bc[label] - bc[others])
        ml, _ = ctx.conc(Mg)
        status = 0
        # magnitude of the head's terms before cancellation (a scale for comparing bounds near zero)
        lh, uh = ctx.conc(X[0])
        scale = float((np.abs(Wc) @ np.maximum(np.abs(lh), np.abs(uh)) + np.abs(bc)).max())
    except NotFinite:
        lo = np.full(n_cls, -np.inf); up = np.full(n_cls, np.inf)
        ml = np.full(n_cls - 1, -np.inf)
        status = 1
        scale = float("inf")
    return {"lower": lo, "upper": up, "margin_lower": ml, "status": status, "label": label, "head_scale": scale}


def is_verified(res):
    """Robust iff the lower bound of the correct class exceeds every other class for the whole ball:
    every margin lower bound > 0 (paper Sec. 1) and the run stayed finite."""
    return res["status"] == 0 and bool(np.all(res["margin_lower"] > 0.0))


def certify(m, tokens, positions, p, eps_lo, eps_hi, steps, label=None):
    """Largest verified eps by bisection: lo, hi = eps_lo, eps_hi; `steps` times test mid = (lo+hi)/2,
    verified -> lo = mid else hi = mid; return lo (eps_lo if nothing verified)."""
    if label is None:
        label = int(np.argmax(clean_logits(m, tokens)))
    lo, hi = float(eps_lo), float(eps_hi)
    for _ in range(steps):
        mid = 0.5 * (lo + hi)
        if is_verified(verify(m, tokens, positions, p, mid, label)):
            lo = mid
        else:
            hi = mid
    return lo, label
