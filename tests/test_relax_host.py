"""The library's per-neuron relaxation code (csrc/relax.h, double precision) compiled for the host and compared
with the oracle's relaxations on random intervals: same lines to 1e-11, and sound on a dense grid.  This checks the
device code's scalar algebra - including the Newton search for the tanh tangent point, which differs from the
oracle's bisection - without a GPU."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import relaxations as RX

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(os.path.dirname(HERE), "paper_2209_12708_amd", "csrc")


@pytest.fixture(scope="module")
def harness(tmp_path_factory):
    cxx = shutil.which("g++")
    if cxx is None:
        pytest.skip("no host C++ compiler")
    exe = str(tmp_path_factory.mktemp("relax") / "relax_host")
    cmd = [cxx, "-O2", "-std=c++17", "-ffp-contract=off", "-Wno-unknown-pragmas", "-I", os.path.join(HERE, "host_stub"),
           "-I", CSRC, "-o", exe, os.path.join(HERE, "relax_host.cpp")]
    subprocess.run(cmd, check=True)
    return exe


def intervals(rng, n, kind):
    if kind == "crossing":
        l = -np.abs(rng.standard_normal(n)) * 10.0 ** rng.uniform(-4, 1.3, n)
        u = np.abs(rng.standard_normal(n)) * 10.0 ** rng.uniform(-4, 1.3, n)
    elif kind == "positive":
        l = np.abs(rng.standard_normal(n)) * 10.0 ** rng.uniform(-3, 1, n) + 1e-6
        u = l + np.abs(rng.standard_normal(n)) * 10.0 ** rng.uniform(-9, 1, n)
    else:
        c = rng.standard_normal(n) * 10.0 ** rng.uniform(-2, 0.7, n)
        w = np.abs(rng.standard_normal(n)) * 10.0 ** rng.uniform(-13, 0.5, n)
        l, u = c - w, c + w
    return l, u


def silu_lines(l, u):
    """The oracle's SiLU chain on neurons x = mid + delta, |delta| <= half (one coordinate, l_inf ball), as lines in x."""
    from oracle import bounds as B
    from oracle import verifier as V
    mid, half = 0.5 * (l + u), 0.5 * (u - l)
    out = []
    for m_, h_ in zip(mid, half):       # eps differs per neuron: one call each
        X = B.Bounds(np.ones((1, 1)), np.array([m_]), np.ones((1, 1)), np.array([m_]))
        Y = V.silu_bound(X, V._Ctx(float(h_), 1, 0))
        out.append([Y.lw[0, 0], Y.lb[0] - Y.lw[0, 0] * m_, Y.uw[0, 0], Y.ub[0] - Y.uw[0, 0] * m_])
    return tuple(np.array(out).T)


CASES = [("leaky", RX.leaky_relu(0.1), None, ("crossing", "any")), ("silu", silu_lines, None, ("crossing", "any")),
         ("relu", RX.relu, np.maximum, ("crossing", "any")), ("tanh", RX.tanh, None, ("crossing", "any", "positive")),
         ("exp", RX.exp, None, ("any",)), ("recip", RX.reciprocal, None, ("positive",)),
         ("sqrt", RX.sqrt, None, ("positive",)), ("square", RX.square, None, ("crossing", "any"))]
FUNCS = {"leaky": lambda x: np.where(x >= 0, x, 0.1 * x), "silu": lambda x: x / (1.0 + np.exp(-x)),
         "relu": lambda x: np.maximum(x, 0.0), "tanh": np.tanh, "exp": np.exp, "recip": lambda x: 1.0 / x,
         "sqrt": np.sqrt, "square": lambda x: x * x}


@pytest.mark.parametrize("name,oracle_fn,_unused,kinds", CASES)
def test_device_relaxations_match_oracle_on_host(harness, name, oracle_fn, _unused, kinds):
    rng = np.random.default_rng(len(name))
    for kind in kinds:
        l, u = intervals(rng, 1500, kind)
        if name == "exp":
            l, u = np.clip(l, -30, 30), np.clip(u, -30, 30)
        text = "\n".join(f"{name} {float(a)!r} {float(b)!r}" for a, b in zip(l, u))
        out = subprocess.run([harness], input=text, capture_output=True, text=True, check=True).stdout.split("\n")
        G = np.array([[float(x) for x in line.split()] for line in out if line.strip()])
        O = np.stack(oracle_fn(l, u), 1)
        assert G.shape == O.shape
        err = (np.abs(G - O) / np.maximum(1.0, np.abs(O))).max(1)
        # a chord slope (f(u) - f(l)) / (u - l) carries the rounding of f divided by the width: intervals just
        # above the point-interval threshold are conditioned accordingly, on both sides alike
        allowed = 1e-11 + 8e-16 * np.maximum(1.0, np.maximum(np.abs(l), np.abs(u))) / np.maximum(u - l, 1e-300)
        worst = int(np.argmax(err / allowed))
        assert np.all(err <= allowed), (name, kind, err[worst], allowed[worst], l[worst], u[worst])
        f = FUNCS[name]
        for a, b, g in zip(l[:300], u[:300], G[:300]):
            xs = np.linspace(a, b, 513)
            fx = f(xs)
            tol = 1e-12 * (1.0 + np.abs(fx).max())
            assert np.all(g[0] * xs + g[1] <= fx + tol) and np.all(g[2] * xs + g[3] >= fx - tol), (name, a, b)
