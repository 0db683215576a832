"""Float64 CPU oracle for transformer-verification bound propagation.

TEST INFRASTRUCTURE ONLY.  A plain, slow implementation of the method, written
from the paper, against which the HIP library is checked.  Only tests, the
smoke check and the benchmark's cpu_baseline leg may import this package; the
product package never does, and this package imports nothing from it.

Pins (tests/test_oracle_*.py, tests/test_golden.py): closed forms of Eq. (1) and Eq. (2), eps = 0 against a
plain forward pass and its Jacobian, sampled soundness of every operator and of the whole encoder, brute force
on tiny models, identities between the operators.  Parity unpinned: which of several sound lines the paper's
own relaxations pick for ReLU / tanh / exp / reciprocal / sqrt / products (its figures for them are not in the
text); the choices made here are stated in the docstrings of relaxations.py and verifier.py and are pinned for
soundness only.
"""
from . import bounds, relaxations, verifier  # noqa: F401
from .verifier import certify, is_verified, verify  # noqa: F401
