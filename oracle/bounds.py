"""Linear-bound state and the per-operator bound rules (float64, numpy).

TEST INFRASTRUCTURE: the slow, plain reference that the HIP path is checked
against.  Nothing in the product path may import it; it imports nothing from
the product.

Notation follows the paper's Table 1 and Sec. 2.1: every neuron X[i] carries
    X[i] >= X_lb[i] + X_lw[i] . delta,     X[i] <= X_ub[i] + X_uw[i] . delta
where delta stacks the offsets of the P perturbed embeddings (length P*E).
A `Bounds` object holds lw, uw of shape neuron_shape + (P*E,) and lb, ub of
shape neuron_shape.

Perturbation set (reading; the paper only says "the norm"): every perturbed
position moves independently inside its own l_p ball of radius eps, so the
norm in Eq. (1) is the sum over positions of the dual (l_q, 1/p + 1/q = 1)
norm of that position's block of coefficients.
"""
import numpy as np

from . import relaxations as rx

P_INF = 0   # encoding of p = infinity (matches tv_synth.configs.NORM_LINF)


class Bounds:
    __slots__ = ("lw", "lb", "uw", "ub")

    def __init__(self, lw, lb, uw, ub):
        self.lw, self.lb, self.uw, self.ub = lw, lb, uw, ub

    @property
    def shape(self):
        return self.lb.shape

    def __getitem__(self, idx):
        return Bounds(self.lw[idx], self.lb[idx], self.uw[idx], self.ub[idx])


def pos(a):
    return np.maximum(a, 0.0)


def neg(a):
    return np.minimum(a, 0.0)


def input_bounds(x0, positions):
    """Sec. 2.1 (input neurons): bias = clean value; weight = one-hot at the neuron's own coordinate.

    x0: [L, E] clean embeddings; positions: the P perturbed token positions.
    Coordinate (r, e) of delta is the offset of embedding entry e of position positions[r].
    """
    L, E = x0.shape
    P = len(positions)
    w = np.zeros((L, E, P, E))
    for r, t in enumerate(positions):
        w[t, np.arange(E), r, np.arange(E)] = 1.0
    w = w.reshape(L, E, P * E)
    return Bounds(w.copy(), x0.astype(np.float64).copy(), w.copy(), x0.astype(np.float64).copy())


def block_dual_norm(w, n_blocks, p):
    """sum over the P blocks of the l_q norm of each block; w: [..., P*E]."""
    blk = w.reshape(w.shape[:-1] + (n_blocks, -1))
    if p == P_INF:        # q = 1
        n = np.abs(blk).sum(-1)
    elif p == 2:          # q = 2
        n = np.sqrt((blk * blk).sum(-1))
    elif p == 1:          # q = infinity
        n = np.abs(blk).max(-1)
    else:
        raise ValueError("p must be 1, 2 or 0 (infinity)")
    return n.sum(-1)


def concretize(X, eps, n_blocks, p):
    """Eq. (1): X_l = X_lb - eps * ||X_lw||,  X_u = X_ub + eps * ||X_uw||."""
    return (X.lb - eps * block_dual_norm(X.lw, n_blocks, p),
            X.ub + eps * block_dual_norm(X.uw, n_blocks, p))


def affine(X, W, c=None):
    """Eq. (2): Y[j] = sum_i W[j,i] X[i] + c[j] along the last neuron axis, split by the sign of W:
    the upper bound takes X's upper where W >= 0 and X's lower where W < 0; the lower the other way."""
    Wp, Wn = pos(W), neg(W)
    uw = Wp @ X.uw + Wn @ X.lw            # [..., out, PE]
    lw = Wp @ X.lw + Wn @ X.uw
    ub = X.ub @ Wp.T + X.lb @ Wn.T
    lb = X.lb @ Wp.T + X.ub @ Wn.T
    if c is not None:
        ub = ub + c
        lb = lb + c
    return Bounds(lw, lb, uw, ub)


def add(X, Y):
    """Sum of two tensors (strict-elementwise in the paper's operator typing): lower with lower, upper with upper."""
    return Bounds(X.lw + Y.lw, X.lb + Y.lb, X.uw + Y.uw, X.ub + Y.ub)


def scale_shift(X, a, c=0.0):
    """Elementwise y = a*x + c with per-neuron constants a (any sign), c: Eq. (2) with a diagonal W."""
    a = np.broadcast_to(np.asarray(a, np.float64), X.shape)
    return substitute(X, a, c, a, c)


def substitute(X, kL, cL, kU, cU):
    """Given kL*x + cL <= f(x) <= kU*x + cU on the concretized range of x, bound f(X):
    each line takes X's own-side bound where its slope is >= 0 and the other side where it is < 0
    (the sign rule of Eq. (2) applied to a per-neuron scalar; Eq. (4) with intercepts)."""
    kLp, kLn, kUp, kUn = pos(kL)[..., None], neg(kL)[..., None], pos(kU)[..., None], neg(kU)[..., None]
    lw = kLp * X.lw + kLn * X.uw
    uw = kUp * X.uw + kUn * X.lw
    lb = pos(kL) * X.lb + neg(kL) * X.ub + cL
    ub = pos(kU) * X.ub + neg(kU) * X.lb + cU
    return Bounds(lw, lb, uw, ub)


def relax(X, fn, l, u):
    """Bound an elementwise function given its relaxation `fn` and the concretized range [l, u] of X."""
    return substitute(X, *fn(l, u))


def _bilinear(X, Y, lx, ly, uy, sx, sy, so):
    """z[so] = sum over the contracted index of x[sx] * y[sy]  (einsum subscripts without the
    coefficient axis), with the McCormick planes of relaxations.mccormick per scalar product and the
    sign rule of `substitute` for both operands, summed over the contracted index."""
    # plane slopes only (aL, aU shaped like y; bL = bU shaped like x); the constants -lx*ly and
    # -lx*uy of the planes are formed per scalar product inside the contraction below
    aL, bL, aU, bU = ly, lx, uy, lx

    def w_terms(coef_on_x, coef_on_y, Xown, Xoth, Yown, Yoth):
        # coef on x has y's shape and multiplies X; coef on y has x's shape and multiplies Y
        return (np.einsum(f"{sy},{sx}c->{so}c", pos(coef_on_x), Xown)
                + np.einsum(f"{sy},{sx}c->{so}c", neg(coef_on_x), Xoth)
                + np.einsum(f"{sx},{sy}c->{so}c", pos(coef_on_y), Yown)
                + np.einsum(f"{sx},{sy}c->{so}c", neg(coef_on_y), Yoth))

    def b_terms(coef_on_x, coef_on_y, Xown, Xoth, Yown, Yoth, const_xy):
        return (np.einsum(f"{sy},{sx}->{so}", pos(coef_on_x), Xown)
                + np.einsum(f"{sy},{sx}->{so}", neg(coef_on_x), Xoth)
                + np.einsum(f"{sx},{sy}->{so}", pos(coef_on_y), Yown)
                + np.einsum(f"{sx},{sy}->{so}", neg(coef_on_y), Yoth)
                + const_xy)

    lw = w_terms(aL, bL, X.lw, X.uw, Y.lw, Y.uw)
    uw = w_terms(aU, bU, X.uw, X.lw, Y.uw, Y.lw)
    lb = b_terms(aL, bL, X.lb, X.ub, Y.lb, Y.ub, np.einsum(f"{sx},{sy}->{so}", -lx, ly))
    ub = b_terms(aU, bU, X.ub, X.lb, Y.ub, Y.lb, np.einsum(f"{sx},{sy}->{so}", -lx, uy))
    return Bounds(lw, lb, uw, ub)


def dot_qk(Q, K, lq, lk, uk):
    """Dot-product operator of one head: s[i,j] = sum_d q[i,d] k[j,d]; both operands carry bounds
    (Sec. 2.3, first observation).  x = q[i,d], y = k[j,d]."""
    return _bilinear(Q, K, lq, lk, uk, "id", "jd", "ij")


def dot_pv(Pb, V, lp, lv, uv):
    """o[i,d] = sum_j p[i,j] v[j,d];  x = p[i,j], y = v[j,d]."""
    return _bilinear(Pb, V, lp, lv, uv, "ij", "jd", "id")


def product(X, Y, lx, ly, uy):
    """Elementwise z = x*y for same-shaped (or broadcastable) bound states."""
    aL, bL, gL, aU, bU, gU = rx.mccormick(lx, ly, uy)
    lw = (pos(aL)[..., None] * X.lw + neg(aL)[..., None] * X.uw
          + pos(bL)[..., None] * Y.lw + neg(bL)[..., None] * Y.uw)
    uw = (pos(aU)[..., None] * X.uw + neg(aU)[..., None] * X.lw
          + pos(bU)[..., None] * Y.uw + neg(bU)[..., None] * Y.lw)
    lb = pos(aL) * X.lb + neg(aL) * X.ub + pos(bL) * Y.lb + neg(bL) * Y.ub + gL
    ub = pos(aU) * X.ub + neg(aU) * X.lb + pos(bU) * Y.ub + neg(bU) * Y.lb + gU
    return Bounds(lw, lb, uw, ub)
