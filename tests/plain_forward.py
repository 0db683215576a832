"""A textbook post-norm transformer encoder forward pass in torch float64.

Written separately from the oracle (it knows nothing about bounds): used to pin
the oracle at eps = 0, to take Jacobians with autograd, and to evaluate sampled
perturbed inputs for soundness checks.
"""
import math

import numpy as np
import torch

ACT_RELU, ACT_TANH, ACT_GELU, ACT_LEAKY_RELU, ACT_SILU = 0, 1, 2, 3, 4


def _t(a):
    return torch.as_tensor(np.asarray(a), dtype=torch.float64)


def embed(m, tokens):
    L = len(tokens)
    return _t(m["tok_emb"])[torch.as_tensor(np.asarray(tokens), dtype=torch.long)] + _t(m["pos_emb"])[:L]


def _ln(x, g, b, eps):
    mu = x.mean(-1, keepdim=True)
    xc = x - mu
    var = (xc * xc).mean(-1, keepdim=True)
    return xc / torch.sqrt(var + eps) * g + b


def _act(x, kind, alpha=0.01):
    if kind == ACT_RELU:
        return torch.relu(x)
    if kind == ACT_TANH:
        return torch.tanh(x)
    if kind == ACT_LEAKY_RELU:
        return torch.where(x >= 0, x, alpha * x)
    if kind == ACT_SILU:
        return x / (1.0 + torch.exp(-x))
    return 0.5 * x * (1.0 + torch.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))


def encoder(m, x):
    """x: [..., L, D] embeddings (already perturbed) -> final hidden [..., L, D]."""
    cfg = m["cfg"]
    H, D = cfg.n_heads, cfg.hidden
    dh = D // H
    for l in range(cfg.n_layers):
        w = lambda n: _t(m[f"l{l}.{n}"])
        q = x @ w("Wq").T + w("bq")
        k = x @ w("Wk").T + w("bk")
        v = x @ w("Wv").T + w("bv")
        sh = x.shape[:-1] + (H, dh)
        q, k, v = (z.reshape(sh).transpose(-2, -3) for z in (q, k, v))     # [..., H, L, dh]
        s = q @ k.transpose(-1, -2) / math.sqrt(dh)
        p = torch.softmax(s, -1)
        o = (p @ v).transpose(-2, -3).reshape(x.shape)
        a = x + o @ w("Wo").T + w("bo")
        x1 = _ln(a, w("ln1_g"), w("ln1_b"), cfg.ln_eps)
        h = _act(x1 @ w("W1").T + w("b1"), cfg.activation, cfg.act_alpha)
        f = x1 + h @ w("W2").T + w("b2")
        x = _ln(f, w("ln2_g"), w("ln2_b"), cfg.ln_eps)
    return x


def logits(m, x):
    return encoder(m, x)[..., 0, :] @ _t(m["Wc"]).T + _t(m["bc"])


def sample_ball(rng, n, P, E, p, eps, surface_frac=0.5):
    """n perturbations [n, P, E]: each position's block inside its own l_p ball of radius eps.
    Mix of interior points, surface points and (for l_inf / l_1) vertices."""
    g = rng.standard_normal((n, P, E))
    if p == 0:      # l_inf
        d = rng.uniform(-1, 1, (n, P, E))
        nv = int(n * surface_frac)
        d[:nv] = np.sign(g[:nv])
    elif p == 2:
        d = g / np.linalg.norm(g, axis=-1, keepdims=True)
        r = rng.uniform(0, 1, (n, P, 1)) ** (1.0 / E)
        r[: int(n * surface_frac)] = 1.0
        d = d * r
    else:           # l_1: exponential trick for the surface, vertices for a share
        e = rng.exponential(size=(n, P, E))
        d = np.sign(g) * e / e.sum(-1, keepdims=True)
        nv = int(n * surface_frac)
        idx = rng.integers(0, E, (nv, P))
        v = np.zeros((nv, P, E))
        np.put_along_axis(v, idx[..., None], 1.0, -1)
        d[:nv] = v * np.sign(g[:nv, :, :1])
        r = rng.uniform(0, 1, (n, P, 1))
        r[: n // 2] = 1.0
        d = d * r
    return d * eps
