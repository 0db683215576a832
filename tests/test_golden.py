"""Stored oracle outputs (tests/golden/c1_bounds.json, written by tests/golden/make_golden.py from oracle/ only).

CPU: the oracle still reproduces the file (a change of its arithmetic must regenerate the file on purpose).
GPU: the library, through the C ABI, matches the stored values to the parity bar.
"""
import json
import os

import numpy as np
import pytest

from oracle import verifier as V
from tv_synth import CONFIGS, make_model, make_positions, make_tokens

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "c1_bounds.json")


@pytest.fixture(scope="module")
def gold():
    with open(GOLD) as f:
        return json.load(f)


def test_oracle_reproduces_golden(gold):
    w = CONFIGS["c1"]
    m = make_model(w)
    tokens, positions = make_tokens(w), make_positions(w)
    for c in gold["verify"]:
        r = V.verify(m, tokens[c["sentence"]], positions[c["sentence"]], c["p"], float(np.float32(c["eps"])))
        assert r["status"] == c["status"] and r["label"] == c["label"]
        for k in ("lower", "upper", "margin_lower"):
            np.testing.assert_allclose(r[k], c[k], rtol=1e-11, atol=1e-13)
    c = gold["certify"][0]
    e, lab = V.certify(m, tokens[0], positions[0], c["p"], c["eps_lo"], c["eps_hi"], c["steps"])
    assert e == c["eps"] and lab == c["label"]


@pytest.mark.gpu
def test_gpu_matches_golden(gold):
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (run with -m 'not gpu' on CPU boxes)")
    from paper_2209_12708_amd import binding as tv
    w = CONFIGS["c1"]
    m = make_model(w)
    tokens, positions = make_tokens(w, 2), make_positions(w, 2)
    model = tv.Model(m)
    tok_d = torch.as_tensor(tokens, device="cuda:0")
    pos_d = torch.as_tensor(positions, device="cuda:0")
    outs = {}
    for c in gold["verify"]:
        key = (c["p"], c["eps"])
        if key not in outs:
            o = model.verify(tok_d, pos_d, c["p"], torch.full((2,), c["eps"], dtype=torch.float32, device="cuda:0"))
            outs[key] = {k: v.cpu().numpy() for k, v in o.items()}
        o, b = outs[key], c["sentence"]
        assert int(o["status"][b]) == c["status"] and int(o["labels"][b]) == c["label"]
        for k, g in (("lower", o["lower"][b]), ("upper", o["upper"][b]), ("margin_lower", o["margin_lower"][b])):
            ref = np.asarray(c[k])
            assert np.all(np.abs(g - ref) <= 1e-4 * np.abs(ref) + 4e-6 * c["head_scale"]), (c["p"], c["eps"], b, k, g, ref)
    cert = model.certify(tok_d, pos_d, 2, w.eps_lo, w.eps_hi, w.steps)
    for c in gold["certify"]:
        assert abs(float(cert["eps"][c["sentence"]]) - c["eps"]) <= (c["eps_hi"] - c["eps_lo"]) / 2 ** c["steps"] * 1.0001
        assert int(cert["labels"][c["sentence"]]) == c["label"]
    model.close()
