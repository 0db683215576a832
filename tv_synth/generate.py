"""Seeded generators: fp32 weights, token ids and perturbed positions.

Recipe: every weight, embedding and bias is drawn N(0, std^2) in float64 from
numpy's default_rng and rounded once to fp32; LayerNorm gamma = 1, beta = 0;
tokens are uniform integers in [0, vocab).  seed = 1000 * config_id + k with
k = 0 for weights and k = 1 for tokens.  `stress` multiplies the std of the
embeddings and of every weight matrix (biases keep std), which drives
pre-activations, attention scores and LayerNorm inputs away from the
almost-linear regime that the plain std-0.02 models stay in.
"""
import numpy as np

from .configs import Workload


def _normal(rng, shape, std):
    return (rng.standard_normal(shape) * std).astype(np.float32)


def make_model(w: Workload, seed_offset: int = 0, stress: float = 1.0) -> dict:
    """Return {'cfg': EncoderConfig, name: fp32 array ...}.

    Linear weights are stored [out, in] (Y[j] = sum_i W[j, i] X[i]).
    """
    enc = w.enc
    rng = np.random.default_rng(1000 * w.config_id + 0 + 7919 * seed_offset)
    D, F, std = enc.hidden, enc.ffn, w.weight_std
    m = {"cfg": enc}
    m["tok_emb"] = _normal(rng, (enc.vocab, D), std * stress)
    m["pos_emb"] = _normal(rng, (enc.max_len, D), std * stress)
    wstd = std * stress
    for l in range(enc.n_layers):
        for nm in ("q", "k", "v", "o"):
            m[f"l{l}.W{nm}"] = _normal(rng, (D, D), wstd)
            m[f"l{l}.b{nm}"] = _normal(rng, (D,), std)
        m[f"l{l}.ln1_g"] = np.ones(D, np.float32)
        m[f"l{l}.ln1_b"] = np.zeros(D, np.float32)
        m[f"l{l}.W1"] = _normal(rng, (F, D), wstd)
        m[f"l{l}.b1"] = _normal(rng, (F,), std)
        m[f"l{l}.W2"] = _normal(rng, (D, F), wstd)
        m[f"l{l}.b2"] = _normal(rng, (D,), std)
        m[f"l{l}.ln2_g"] = np.ones(D, np.float32)
        m[f"l{l}.ln2_b"] = np.zeros(D, np.float32)
    m["Wc"] = _normal(rng, (enc.n_classes, D), wstd)
    m["bc"] = _normal(rng, (enc.n_classes,), std)
    return m


def randomize_layernorm(m: dict, seed: int = 0) -> dict:
    """Test helper: non-trivial gamma (both signs) and beta, so the scale/shift step is exercised."""
    enc = m["cfg"]
    rng = np.random.default_rng(424242 + seed)
    out = dict(m)
    for l in range(enc.n_layers):
        for nm in ("ln1", "ln2"):
            g = rng.standard_normal(enc.hidden) * 0.5 + 0.8
            out[f"l{l}.{nm}_g"] = g.astype(np.float32)
            out[f"l{l}.{nm}_b"] = (rng.standard_normal(enc.hidden) * 0.1).astype(np.float32)
    return out


def make_tokens(w: Workload, batch: int = None, seed_offset: int = 0) -> np.ndarray:
    rng = np.random.default_rng(1000 * w.config_id + 1 + 7919 * seed_offset)
    b = w.batch if batch is None else batch
    return rng.integers(0, w.enc.vocab, size=(b, w.seq_len), dtype=np.int32)


def make_positions(w: Workload, batch: int = None) -> np.ndarray:
    """Deterministic perturbed positions: P=1 -> {1}; P=2 -> {1, L/2}; sorted, distinct."""
    b = w.batch if batch is None else batch
    L, P = w.seq_len, w.n_perturbed
    if P == 1:
        pos = [min(1, L - 1)]
    elif P == 2:
        pos = [1, max(2, L // 2)]
    else:
        pos = list(np.linspace(0, L - 1, P).astype(int))
    assert len(set(pos)) == P and max(pos) < L
    return np.tile(np.asarray(pos, np.int32), (b, 1))
