"""Pins of the oracle's BatchNorm batch statistics (fixed tree) and of the clipped update."""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
from test_oracle_tree import golden_witness, witness_inputs


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def twin_tree(terms):
    """The tree of the golden file over a vector of fp32 terms, from reshapes and slice adds."""
    f = np.float32
    t = np.asarray(terms, dtype=f)
    n = t.size
    nblk = max(-(-n // 4096), 1)
    pad = np.zeros(nblk * 4096, dtype=f)
    pad[:n] = t
    sq = pad.reshape(nblk, 4, 256, 4)
    lane = np.zeros((nblk, 256), dtype=f)
    for q in range(4):
        for c in range(4):
            lane = lane + sq[:, q, :, c]

    def tree(v):
        s = 128
        while s >= 1:
            v = v[..., :s] + v[..., s:2 * s]
            s //= 2
        return v[..., 0]

    part = tree(lane)[:-(-n // 4096)] if n else np.zeros(0, dtype=f)
    rows = max(-(-part.size // 256), 1)
    p2 = np.zeros(rows * 256, dtype=f)
    p2[:part.size] = part
    lane2 = np.zeros(256, dtype=f)
    for k in range(rows):
        lane2 = lane2 + p2.reshape(rows, 256)[k]
    return f(tree(lane2))


def twin_bn(x):
    f = np.float32
    B, C, HW = x.shape
    M = f(B * HW)
    mean, var = np.empty(C, dtype=f), np.empty(C, dtype=f)
    for ch in range(C):
        y = x[:, ch, :].reshape(-1)                      # order (image, position)
        mean[ch] = twin_tree(y) / M
        d = (y - mean[ch]).astype(f)
        var[ch] = twin_tree(d * d) / M
    return mean, var


# ---- BatchNorm statistics ---------------------------------------------------------------
def test_hand_derived_witness_fixes_the_tree_and_the_layout():
    """Witness A of tests/golden/tree_witness.txt with the VALUES 2^24 and 1 (their sum follows the
    same derivation as the squares of 4096 and 1): 2^24+12 over 4096 terms, mean = 4096 + 12/4096.
    The same virtual vector cut into 2 or 4 images, and placed in one channel among others,
    must give the same mean."""
    a = witness_inputs()["A"]
    y = np.where(a == 4096, np.float32(2.0 ** 24), a).astype(np.float32)
    want = np.float32(golden_witness()["A"][1]) / np.float32(4096)
    assert want == np.float32(4096.0029296875)
    for B in (1, 2, 4):
        mean, _ = oracle.bn_batch_stats(y.reshape(B, 1, 4096 // B))
        assert bits(mean)[0] == bits(want)[0], B
    rng = np.random.default_rng(0)
    x = rng.standard_normal((2, 3, 2048)).astype(np.float32)
    x[:, 1, :] = y.reshape(2, 2048)
    mean, _ = oracle.bn_batch_stats(x)
    assert bits(mean)[1] == bits(want)[0]
    # witness B: 515 blocks, the second stage of the tree
    b = witness_inputs()["B"]
    yb = np.where(b == 4096, np.float32(2.0 ** 24), b).astype(np.float32)
    mean, _ = oracle.bn_batch_stats(yb.reshape(5, 1, yb.size // 5))
    assert bits(mean)[0] == bits(np.float32(golden_witness()["B"][1]) / np.float32(yb.size))[0]


def test_exact_cases():
    """Integer data in +/- pairs around a centre of 0 or 0.5, shuffled: every sum, the mean, every
    deviation and every square is exact in fp32 in any order, so the result must equal the float64
    mean and variance exactly (a dropped term, a wrong divisor or a wrong centre shows)."""
    rng = np.random.default_rng(1)
    for B, C, HW, centre in ((4, 5, 256, 0.0), (8, 2, 1024, 0.5), (1, 3, 64, 0.0), (16, 1, 4096, 0.5),
                             (3, 2, 50, 0.0)):
        M = B * HW
        x = np.empty((B, C, HW), dtype=np.float32)
        for ch in range(C):
            half = rng.integers(0, 8, M // 2).astype(np.float32)
            y = np.concatenate([half, -half]) + np.float32(centre)
            x[:, ch, :] = rng.permutation(y).reshape(B, HW)
        mean, var = oracle.bn_batch_stats(x)
        x64 = x.astype(np.float64).transpose(1, 0, 2).reshape(C, -1)
        assert np.all(mean == np.float32(centre))
        if M & (M - 1) == 0:                     # power-of-two count: the final division is exact too
            assert np.array_equal(var.astype(np.float64), x64.var(axis=1))
        else:                                    # else it is the correctly rounded quotient of exact operands
            ssd = ((x64 - centre) ** 2).sum(axis=1)
            assert np.array_equal(var, (ssd.astype(np.float32) / np.float32(M)).astype(np.float32))
    x = np.full((3, 2, 700), 1.5, dtype=np.float32)           # constant: mean exact, variance zero
    mean, var = oracle.bn_batch_stats(x)
    assert np.all(mean == 1.5) and np.all(var == 0.0) and not np.any(np.signbit(var))


@pytest.mark.parametrize("B,C,HW", [(1, 1, 1), (2, 3, 49), (3, 2, 4097), (5, 4, 3136), (32, 2, 196),
                                    (7, 1, 150_001)])
def test_matches_numpy_twin(B, C, HW):
    rng = np.random.default_rng(B * 1000 + HW)
    x = (rng.standard_normal((B, C, HW)) * 3 + rng.standard_normal((1, C, 1)) * 10).astype(np.float32)
    mean, var = oracle.bn_batch_stats(x)
    tm, tv = twin_bn(x)
    assert np.array_equal(bits(mean), bits(tm)) and np.array_equal(bits(var), bits(tv))


def test_error_bound_and_layout_permutations():
    rng = np.random.default_rng(3)
    B, C, HW = 6, 5, 5000
    x = (rng.standard_normal((B, C, HW)) + 4).astype(np.float32)
    mean, var = oracle.bn_batch_stats(x)
    x64 = x.astype(np.float64).transpose(1, 0, 2).reshape(C, -1)
    M = B * HW
    depth = 16 + 8 + 1 + 8 + 2                                 # adds on the longest path, +1 op per term, + division
    u = 2.0 ** -24
    for ch in range(C):
        exact_mean = math.fsum(x64[ch]) / M
        assert abs(float(mean[ch]) - exact_mean) <= depth * u * (math.fsum(np.abs(x64[ch])) / M) * 1.01
        exact_var = math.fsum((x64[ch] - float(mean[ch])) ** 2) / M
        assert abs(float(var[ch]) - exact_var) <= (depth + 3) * u * exact_var * 1.05
    # channels are independent: permuting them permutes the results
    perm = rng.permutation(C)
    pm, pv = oracle.bn_batch_stats(x[:, perm, :])
    assert np.array_equal(bits(pm), bits(mean[perm])) and np.array_equal(bits(pv), bits(var[perm]))
    # the order inside a channel is (image, position): swapping two images changes the tree's
    # operands (and, on this data, bits), swapping it back restores them
    sw = x[[1, 0, 2, 3, 4, 5]]
    sm, _ = oracle.bn_batch_stats(sw)
    assert not np.array_equal(bits(sm), bits(mean))
    assert np.array_equal(bits(oracle.bn_batch_stats(sw[[1, 0, 2, 3, 4, 5]])[0]), bits(mean))
    # empty input
    m0, v0 = oracle.bn_batch_stats(np.zeros((2, 0, 8), dtype=np.float32))
    assert m0.size == 0 and v0.size == 0


# ---- clipped update ----------------------------------------------------------------------
def test_clip_coefficient_is_correctly_rounded():
    rng = np.random.default_rng(4)
    for _ in range(2000):
        norm = np.float32(abs(rng.standard_normal()) * 10.0 ** rng.integers(-3, 4))
        mx = np.float32(abs(rng.standard_normal()) * 10.0 ** rng.integers(-2, 3) + 1e-3)
        eps = np.float32(1e-6)
        d = np.float32(norm + eps)                       # one rounding (numpy fp32 add is IEEE)
        q = Fraction(float(mx)) / Fraction(float(d))     # exact quotient of the two fp32 values
        got = oracle.clip_coef(norm, mx, eps)
        if q >= 1:
            assert got == 1.0
        else:
            lo, hi = np.nextafter(got, np.float32(-np.inf)), np.nextafter(got, np.float32(np.inf))
            assert abs(Fraction(float(got)) - q) <= min(abs(Fraction(float(lo)) - q), abs(Fraction(float(hi)) - q))
    assert oracle.clip_coef(3.0, 2.0, 1.0) == 0.5 and oracle.clip_coef(1.0, 2.0, 0.0) == 1.0
    assert oracle.clip_coef(2.0, 2.0, 0.0) == 1.0


def test_unclipped_step_is_the_plain_update_and_clipped_step_scales_first():
    rng = np.random.default_rng(5)
    n = 10_007
    p0, v0, g = (rng.standard_normal(n).astype(np.float32) for _ in range(3))
    p1, v1 = p0.copy(), v0.copy()
    oracle.sgd_momentum(p1, v1, g, 0.1, 0.9)
    p2, v2 = p0.copy(), v0.copy()
    oracle.sgd_momentum_scaled(p2, v2, g, 0.1, 0.9, 1.0)
    assert np.array_equal(bits(p1), bits(p2)) and np.array_equal(bits(v1), bits(v2))
    # coef = 0.5: the scaled gradient g/2 is exact, so the step equals the plain update on g/2
    p3, v3 = p0.copy(), v0.copy()
    oracle.sgd_momentum_scaled(p3, v3, g, 0.1, 0.9, 0.5)
    p4, v4 = p0.copy(), v0.copy()
    oracle.sgd_momentum(p4, v4, (g * np.float32(0.5)).astype(np.float32), 0.1, 0.9)
    assert np.array_equal(bits(p3), bits(p4)) and np.array_equal(bits(v3), bits(v4))
    # the product is rounded on its own before it enters the momentum (no contraction):
    # coef = 1/3: compare with the same three roundings in numpy
    c = np.float32(1.0) / np.float32(3.0)
    p5, v5 = p0.copy(), v0.copy()
    oracle.sgd_momentum_scaled(p5, v5, g, 0.1, 0.9, c)
    gs = (c * g).astype(np.float32)
    vn = ((np.float32(0.9) * v0).astype(np.float32) + gs).astype(np.float32)
    pn = (p0 - (np.float32(0.1) * vn).astype(np.float32)).astype(np.float32)
    assert np.array_equal(bits(v5), bits(vn)) and np.array_equal(bits(p5), bits(pn))
