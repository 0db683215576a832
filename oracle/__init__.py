"""Float64 CPU oracle for transformer-verification bound propagation.

TEST INFRASTRUCTURE ONLY.  A plain, slow implementation of the method, written
from the paper, against which the HIP library is checked.  Only tests, the
smoke check and the benchmark's cpu_baseline leg may import this package; the
product package never does, and this package imports nothing from it.
"""
from . import bounds, relaxations, verifier  # noqa: F401
from .verifier import certify, is_verified, verify  # noqa: F401
