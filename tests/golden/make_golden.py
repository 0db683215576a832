#!/usr/bin/env python3
"""Writes tests/golden/c1_bounds.json: logit bounds, margins and certified radii of the float64 oracle on the
smallest configuration (c1).  The paper prints no worked numerical example of a bound, so these are not the
paper's numbers: they freeze the oracle's present output so that a later change to its arithmetic shows up as a
diff of this file (and has to be justified against the paper in the commit that regenerates it).

Calls only `oracle/` and the seeded input generators.  Run from the repository root:
    python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import verifier as V  # noqa: E402
from tv_synth import CONFIGS, make_model, make_positions, make_tokens  # noqa: E402


def main():
    w = CONFIGS["c1"]
    m = make_model(w)
    tokens, positions = make_tokens(w), make_positions(w)
    cases = []
    for p in (1, 2, 0):
        for eps in (0.0, 1e-3, 0.02):
            for b in range(2):
                r = V.verify(m, tokens[b], positions[b], p, float(np.float32(eps)))
                cases.append({"p": p, "eps": eps, "sentence": b, "lower": [float(x) for x in r["lower"]],
                              "upper": [float(x) for x in r["upper"]],
                              "margin_lower": [float(x) for x in r["margin_lower"]], "status": int(r["status"]),
                              "label": int(r["label"]), "head_scale": float(r["head_scale"])})
    cert = []
    for b in range(2):
        e, lab = V.certify(m, tokens[b], positions[b], 2, w.eps_lo, w.eps_hi, w.steps)
        cert.append({"p": 2, "sentence": b, "eps": float(e), "label": int(lab), "steps": w.steps,
                     "eps_lo": w.eps_lo, "eps_hi": w.eps_hi})
    out = {"config": "c1", "source": "oracle/verifier.py (float64)", "verify": cases, "certify": cert}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c1_bounds.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
    print("wrote", path, len(cases), "verify cases,", len(cert), "certify cases")


if __name__ == "__main__":
    main()
