"""Pins of the oracle's SGD-momentum update."""
from fractions import Fraction

import numpy as np

import oracle


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def test_first_step_from_zero_momentum():
    rng = np.random.default_rng(0)
    g = rng.standard_normal(257).astype(np.float32)
    p0 = rng.standard_normal(257).astype(np.float32)
    p, v = p0.copy(), np.zeros_like(p0)
    oracle.sgd_momentum(p, v, g, 0.25, 0.9)
    assert np.array_equal(bits(v), bits(np.float32(0.0) + g))       # 0.9*0 + g
    assert np.array_equal(bits(p), bits(p0 - np.float32(0.25) * g))  # 0.25*g exact


def test_exact_rationals_three_steps():
    """lr, mu powers of two and small-integer data: every intermediate is exact."""
    lr, mu = 0.25, 0.5
    rng = np.random.default_rng(1)
    n = 101
    p = rng.integers(-64, 64, n).astype(np.float32)
    v = np.zeros(n, dtype=np.float32)
    P = [Fraction(int(x)) for x in p]
    V = [Fraction(0)] * n
    for step in range(3):
        g = rng.integers(-16, 16, n).astype(np.float32)
        oracle.sgd_momentum(p, v, g, lr, mu)
        V = [Fraction(1, 2) * V[i] + Fraction(int(g[i])) for i in range(n)]
        P = [P[i] - Fraction(1, 4) * V[i] for i in range(n)]
        assert [Fraction(float(x)) for x in v] == V
        assert [Fraction(float(x)) for x in p] == P


def test_scalar_trace_with_rounding():
    """One element, three steps, lr=0.1 mu=0.9: each operation rounded to fp32 on its own."""
    f = np.float32
    lr, mu = f(0.1), f(0.9)
    p, v = np.array([1.0], dtype=np.float32), np.zeros(1, dtype=np.float32)
    ps, vs = f(1.0), f(0.0)
    for g in (f(0.3), f(-0.7), f(1e-3)):
        oracle.sgd_momentum(p, v, np.array([g], dtype=np.float32), float(lr), float(mu))
        # float64 holds the exact product/sum of two fp32 values (48-bit product; sums
        # here are well inside 53 bits), so rounding it once to fp32 is the IEEE result
        mv = f(np.float64(mu) * np.float64(vs))
        vs = f(np.float64(mv) + np.float64(g))
        st = f(np.float64(lr) * np.float64(vs))
        ps = f(np.float64(ps) - np.float64(st))
        assert bits(v)[0] == bits(np.array([vs]))[0]
        assert bits(p)[0] == bits(np.array([ps]))[0]


def test_no_fma_contraction():
    """Inputs on which fma(mu,v,g) and fma(-lr,v,p) differ from separately rounded ops."""
    e = np.float32(1.0 + 2.0 ** -12)          # e*e = 1 + 2^-11 + 2^-24 -> rounds to 1 + 2^-11
    r = np.float32(1.0 + 2.0 ** -11)
    # momentum line: mu*v + g
    p, v, g = (np.array([x], dtype=np.float32) for x in (0.0, e, -r))
    oracle.sgd_momentum(p, v, g, 0.0, float(e))
    assert bits(v)[0] == 0                     # fused would give 2^-24
    # parameter line: p - lr*v, with v <- 0*v + e
    p, v, g = (np.array([x], dtype=np.float32) for x in (r, 0.0, e))
    oracle.sgd_momentum(p, v, g, float(e), 0.0)
    assert v[0] == e and bits(p)[0] == 0       # fused would give -2^-24
