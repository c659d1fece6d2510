"""Pins of the oracle's ring all-reduce: what the mathematics fixes, not the oracle itself."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import fold_def
from workloads import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def wide_random(shape, seed):
    """fp32 values spread over ~40 binades, both signs: addition order matters."""
    rng = np.random.default_rng(seed)
    m = rng.standard_normal(shape)
    e = rng.integers(-20, 20, size=shape)
    return (m * np.exp2(e)).astype(np.float32)


# ---- geometry ---------------------------------------------------------------

def test_chunk_bounds_partition_and_alignment():
    for N in (1, 2, 3, 4, 5, 7, 8, 16):
        for A in (1, 4):
            for L in list(range(0, 3 * N + 6)) + [1000, 1001, 4099]:
                prev = 0
                for c in range(N):
                    lo, hi = oracle.chunk_bounds(L, N, A, c)
                    assert lo == prev and lo <= hi <= L
                    if hi < L:
                        assert hi % A == 0
                    prev = hi
                assert prev == L
                # no chunk is longer than the first, and length >= ceil(L/N)
                l0 = oracle.chunk_bounds(L, N, A, 0)
                assert (l0[1] - l0[0]) * N >= L


def test_chunk_bounds_resnet50_bucket0_n32():
    # 7,564,264 elements among 32 ranks, A = 4: chunk length 236,384, last chunk 236,360
    L, N, A = 7564264, 32, 4
    assert oracle.chunk_bounds(L, N, A, 0) == (0, 236384)
    lo, hi = oracle.chunk_bounds(L, N, A, 31)
    assert (lo, hi - lo) == (31 * 236384, 236360)


# ---- pins -------------------------------------------------------------------

def test_n1_is_identity_bitwise():
    g = wide_random((1, 1037), 1)
    g[0, :4] = [-0.0, 0.0, 1e-45, -1e-40]          # signed zero and denormals survive
    out = oracle.ring_order_reduce(g, A=1)
    assert np.array_equal(bits(out), bits(g[0]))


@pytest.mark.parametrize("N", [2, 3, 4, 5, 8, 16, 64])
def test_integer_valued_inputs_give_exact_sums(N):
    L = 4099
    g = np.stack([synth.small_ints(L, 7, 0, r, span=1 << 12).numpy() for r in range(N)])
    exact = g.astype(np.int64).sum(axis=0)
    held = oracle.ring_allreduce(g, A=4)
    for r in range(N):                               # every rank holds the exact sums
        assert np.array_equal(held[r].astype(np.int64), exact)
    avg = oracle.ring_order_reduce(g, A=4)
    for i in range(0, L, 97):                        # division correctly rounded
        want = Fraction(int(exact[i]), N)
        got = Fraction(float(avg[i]))
        assert abs(got - want) <= abs(want) * Fraction(1, 2 ** 24)
    if N & (N - 1) == 0:                             # power of two: exact
        assert np.array_equal(avg.astype(np.float64) * N, exact.astype(np.float64))


def test_all_ranks_hold_the_same_bits_after_all_gather():
    for N in (2, 3, 5, 8):
        g = wide_random((N, 211), 10 + N)
        held = oracle.ring_allreduce(g, A=1)
        for r in range(1, N):
            assert np.array_equal(bits(held[r]), bits(held[0]))


def _brute(vals, start):
    """Explicit parenthesised left fold over ranks start, start+1, ... (scalars)."""
    f = np.float32
    n = len(vals)
    v = [f(vals[(start + k) % n]) for k in range(n)]
    if n == 1:
        s = v[0]
    elif n == 2:
        s = f(v[0] + v[1])
    elif n == 3:
        s = f(f(v[0] + v[1]) + v[2])
    else:
        s = f(f(f(v[0] + v[1]) + v[2]) + v[3])
    return f(s / f(n))


@pytest.mark.parametrize("N", [1, 2, 3, 4])
def test_brute_force_small_n(N):
    for A in (1, 4):
        for L in range(0, 3 * N + 6):
            g = wide_random((N, L), 100 * N + L)
            out = oracle.ring_order_reduce(g, A=A)
            cl = -(-(-(-L // N)) // A) * A           # roundup(ceil(L/N), A)
            for i in range(L):
                want = _brute(g[:, i], i // cl)
                assert bits(out[i:i + 1])[0] == bits(np.array([want]))[0], (N, A, L, i)


def test_matches_closed_form_fold():
    for N in range(1, 9):
        for A in (1, 4):
            for L in range(0, 3 * N + 6):
                g = wide_random((N, L), 1000 * N + 10 * L + A)
                assert np.array_equal(bits(oracle.ring_order_reduce(g, A=A)),
                                      bits(fold_def.fold_reduce(g, A=A))), (N, A, L)
                assert np.array_equal(bits(oracle.ring_order_reduce(g, A=A)),
                                      bits(fold_def.fold_reduce_gather(g, A=A))), (N, A, L)
    for N, L, A in ((16, 5003, 4), (64, 3001, 4), (7, 1 << 14, 1)):
        g = wide_random((N, L), N + L)
        assert np.array_equal(bits(oracle.ring_order_reduce(g, A=A)),
                              bits(fold_def.fold_reduce(g, A=A)))
        assert np.array_equal(bits(oracle.ring_order_reduce(g, A=A)),
                              bits(fold_def.fold_reduce_gather(g, A=A)))
    # many more ranks than elements: most chunks empty, start ranks far apart
    for N, L, A in ((300, 7, 1), (300, 41, 4), (1000, 1003, 1)):
        g = wide_random((N, L), N + L)
        assert np.array_equal(bits(oracle.ring_order_reduce(g, A=A)),
                              bits(fold_def.fold_reduce_gather(g, A=A)))


def _read_witness():
    rows = []
    with open(os.path.join(GOLDEN, "order_witness.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                c, s, a, h = line.split()
                rows.append((int(c), float(s), float(a), int(h, 16)))
    return rows


def test_order_witness_golden():
    rows = _read_witness()
    m = 5
    vals = np.array([2.0 ** 24, 1.0, -(2.0 ** 24), 1.0], dtype=np.float32)
    g = np.repeat(vals[:, None], 4 * m, axis=1)
    held = oracle.ring_allreduce(g, A=1)[0]
    avg = oracle.ring_order_reduce(g, A=1)
    for c, s, a, h in rows:
        assert np.all(held[c * m:(c + 1) * m] == np.float32(s))
        assert np.all(bits(avg[c * m:(c + 1) * m]) == h)
        assert np.float32(a).view(np.uint32) == h


def test_witness_tells_other_conventions_apart():
    """The witness input separates the ring order from three plausible wrong ones."""
    f = np.float32
    vals = [f(2.0 ** 24), f(1.0), f(-(2.0 ** 24)), f(1.0)]

    def fold(order):
        s = vals[order[0]]
        for r in order[1:]:
            s = f(s + vals[r])
        return float(s)

    ours = [fold([(c + k) % 4 for k in range(4)]) for c in range(4)]
    start_next = [fold([(c + 1 + k) % 4 for k in range(4)]) for c in range(4)]
    descending = [fold([(c - k) % 4 for k in range(4)]) for c in range(4)]
    naive = [fold([0, 1, 2, 3]) for _ in range(4)]
    assert ours == [s for _, s, _, _ in _read_witness()]
    assert start_next == [2.0, 2.0, 0.0, 1.0]
    assert descending == [1.0, 0.0, 2.0, 2.0]
    assert naive == [1.0, 1.0, 1.0, 1.0]
    assert len({tuple(ours), tuple(start_next), tuple(descending), tuple(naive)}) == 4


def test_recursive_summation_error_bound():
    u = 2.0 ** -24
    for N in (3, 8, 64):
        g = wide_random((N, 503), 77 + N)
        held = oracle.ring_allreduce(g, A=1)[0]
        gamma = (N - 1) * u / (1 - (N - 1) * u)
        for i in range(g.shape[1]):
            exact = math.fsum(float(x) for x in g[:, i])
            bound = gamma * math.fsum(abs(float(x)) for x in g[:, i])
            assert abs(float(held[i]) - exact) <= bound * (1 + 1e-9) + 1e-45


@pytest.mark.parametrize("N", [3, 5, 6, 7])
def test_division_is_correctly_rounded(N):
    """x / N against exact rational rounding (N not a power of two: x*(1/N) would differ)."""
    xs = np.arange(1, 4001, dtype=np.float32)
    g = np.zeros((N, xs.size), dtype=np.float32)
    g[0] = xs
    avg = oracle.ring_order_reduce(g, A=1)
    n_mismatch_recip = 0
    recip = np.float32(1.0) / np.float32(N)
    for i, x in enumerate(xs):
        q = Fraction(int(x), N)
        got = Fraction(float(avg[i]))
        lo = Fraction(float(np.nextafter(avg[i], np.float32(-np.inf))))
        hi = Fraction(float(np.nextafter(avg[i], np.float32(np.inf))))
        assert abs(got - q) <= abs(lo - q) and abs(got - q) <= abs(hi - q)
        n_mismatch_recip += int(np.float32(x * recip) != avg[i])
    assert n_mismatch_recip > 0        # the pin can see a reciprocal-multiply shortcut


def test_negative_control_permuted_ranks_change_bits():
    """Permuting virtual ranks changes the result on an order-sensitive input (paper §5.1.1:
    losing the recorded mapping makes runs diverge)."""
    g = wide_random((4, 64), 5)
    a = oracle.ring_order_reduce(g, A=1)
    b = oracle.ring_order_reduce(g[[1, 0, 2, 3]], A=1)
    assert not np.array_equal(bits(a), bits(b))


def test_random_geometries_against_closed_form():
    """Property test: the message-passing simulation equals the rotated left fold for
    arbitrary rank counts, lengths and alignments (hypothesis draws the cases)."""
    from hypothesis import given, settings, strategies as st

    @settings(max_examples=300, deadline=None)
    @given(N=st.integers(1, 13), L=st.integers(0, 260), A=st.sampled_from([1, 2, 3, 4, 8, 64]),
           seed=st.integers(0, 2 ** 31 - 1))
    def prop(N, L, A, seed):
        g = wide_random((N, L), seed)
        got = oracle.ring_order_reduce(g, A=A)
        assert np.array_equal(bits(got), bits(fold_def.fold_reduce(g, A=A)))
        # element i's fold starts at the rank that owns its chunk
        if L:
            cl = fold_def.chunk_len(L, N, A)
            i = seed % L
            c = i // cl
            acc = np.float32(g[c % N, i])
            for k in range(1, N):
                acc = np.float32(acc + g[(c + k) % N, i])
            assert bits(got[i:i + 1])[0] == bits(np.array([acc / np.float32(N)]))[0]

    prop()


def test_all_core_build_of_the_oracle_gives_the_same_bits():
    """bench.py also times es_oracle.c built with -fopenmp (threads over the ring's ranks and over
    elementwise loops).  It must be the same function: compared here with the pinned default
    build on ragged geometries, and switched back afterwards."""
    rng = np.random.default_rng(77)
    cases = [(N, L, A) for N in (1, 2, 3, 5, 8, 17) for L in (0, 1, 7, 64, 1001, 40_003) for A in (1, 4)]
    want = {}
    for N, L, A in cases:
        g = (rng.standard_normal((N, L)) * np.exp2(rng.integers(-20, 20, (N, L)))).astype(np.float32)
        want[(N, L, A)] = (g, oracle.ring_order_reduce(g, A))
    p0 = rng.standard_normal(5003).astype(np.float32)
    v0 = rng.standard_normal(5003).astype(np.float32)
    gr = rng.standard_normal(5003).astype(np.float32)
    p1, v1 = p0.copy(), v0.copy()
    oracle.sgd_momentum(p1, v1, gr, 0.1, 0.9)
    oracle.use_all_cores(True)
    try:
        for key, (g, ref) in want.items():
            got = oracle.ring_order_reduce(g, key[2])
            assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), key
        p2, v2 = p0.copy(), v0.copy()
        oracle.sgd_momentum(p2, v2, gr, 0.1, 0.9)
        assert np.array_equal(p1.view(np.uint32), p2.view(np.uint32))
        assert np.array_equal(v1.view(np.uint32), v2.view(np.uint32))
    finally:
        oracle.use_all_cores(False)
