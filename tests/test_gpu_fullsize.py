"""Full-size runs of the three large configurations (c3, c4, c5), where the float64 oracle needs minutes to
hours per sentence.  Properties that hold at any size stand in for an element-by-element comparison:

* eps = 0: every radius is exactly zero, so lower == upper == the clean logits of a plain float64 forward pass
  (this exercises every contraction, the relaxations at point intervals, LayerNorm, softmax and the head at the
  full launch shapes: VEC = 2 / 3 LayerNorm, 64- and 128-token softmax rows, K up to 3072);
* eps > 0: either status 1 with infinite bounds, or bounds that contain sampled perturbed forward passes.

Tolerance as in the parity tests: |g - o| <= 1e-4 |o| + 4e-6 T, T = sum_d |Wc[c,d]| |h_d| + |bc| (the head's terms).
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import plain_forward as pf  # noqa: E402
from tv_synth import CONFIGS, make_model, make_positions, make_tokens  # noqa: E402


@pytest.fixture(scope="module")
def tv():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (run with -m 'not gpu' on CPU boxes)")
    from paper_2209_12708_amd import binding
    binding.lib()
    return binding


def dev(a):
    return torch.as_tensor(np.ascontiguousarray(a), device="cuda:0")


@pytest.mark.parametrize("name,n,eps_pos", [("c3", 2, 1e-8), ("c4", 2, 1e-6), ("c5", 1, 1e-8)])
def test_full_size_properties(tv, name, n, eps_pos):
    w = CONFIGS[name]
    m = make_model(w)
    tokens, positions = make_tokens(w, n), make_positions(w, n)
    p = w.p_norms[0]
    model = tv.Model(m)
    tok_d, pos_d = dev(tokens), dev(positions)

    out = model.verify(tok_d, pos_d, p, torch.zeros(n, dtype=torch.float32, device="cuda:0"))
    lo, up = out["lower"].cpu().numpy().astype(np.float64), out["upper"].cpu().numpy().astype(np.float64)
    assert np.all(out["status"].cpu().numpy() == 0), "eps = 0 must not overflow"
    Wc, bc = np.asarray(m["Wc"], np.float64), np.asarray(m["bc"], np.float64)
    for b in range(n):
        h = pf.encoder(m, pf.embed(m, tokens[b]))[0].numpy()
        clean = Wc @ h + bc
        T = np.max(np.abs(Wc) @ np.abs(h) + np.abs(bc))
        tol = 1e-4 * np.abs(clean) + 4e-6 * T
        assert np.all(np.abs(lo[b] - clean) <= tol) and np.all(np.abs(up[b] - clean) <= tol), (name, b, lo[b], up[b], clean)
        assert int(out["labels"][b]) == int(np.argmax(clean))

    out = model.verify(tok_d, pos_d, p, torch.full((n,), eps_pos, dtype=torch.float32, device="cuda:0"))
    lo, up, st = out["lower"].cpu().numpy(), out["upper"].cpu().numpy(), out["status"].cpu().numpy()
    rng = np.random.default_rng(1)
    for b in range(n):
        if st[b] != 0:
            assert np.all(np.isinf(lo[b])) and np.all(np.isinf(up[b]))
            continue
        d = pf.sample_ball(rng, 16, w.n_perturbed, w.enc.hidden, p, eps_pos)
        x = pf.embed(m, tokens[b]).unsqueeze(0).repeat(len(d), 1, 1)
        x[:, positions[b]] += torch.as_tensor(d)
        y = pf.logits(m, x).numpy()
        tol = 1e-5 * (1 + np.abs(y).max())
        assert np.all(y >= lo[b] - tol) and np.all(y <= up[b] + tol)
    model.close()
    torch.cuda.empty_cache()
