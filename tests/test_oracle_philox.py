"""Pins of the oracle's Philox4x32-10 and of the dropout mask built on it."""
import ctypes
import os
import subprocess
import sys

import numpy as np
import pytest

import oracle

M0, M1 = 0xD2511F53, 0xCD9E8D57            # round multipliers (Salmon et al., SC'11)
W0, W1 = 0x9E3779B9, 0xBB67AE85            # key schedule (Weyl) increments
MASK = 0xFFFFFFFF


def philox_bigint(ctr, key, rounds=10):
    """Independent implementation with Python integers."""
    c = list(ctr)
    k = list(key)
    for r in range(rounds):
        p0 = M0 * c[0]
        p1 = M1 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & MASK, (p0 >> 32) ^ c[3] ^ k[1], p0 & MASK]
        k = [(k[0] + W0) & MASK, (k[1] + W1) & MASK]
    return tuple(c)


def philox_inverse(out, key, rounds=10):
    """Runs the rounds backwards (the multipliers are odd, hence invertible mod 2^32)."""
    i0, i1 = pow(M0, -1, 1 << 32), pow(M1, -1, 1 << 32)
    keys = [((key[0] + r * W0) & MASK, (key[1] + r * W1) & MASK) for r in range(rounds)]
    c = list(out)
    for r in reversed(range(rounds)):
        c2 = (c[1] * i1) & MASK
        c0 = (c[3] * i0) & MASK
        c1 = c[0] ^ ((M1 * c2) >> 32) ^ keys[r][0]
        c3 = c[2] ^ ((M0 * c0) >> 32) ^ keys[r][1]
        c = [c0, c1, c2, c3]
    return tuple(c)


def _cases(n, seed):
    rng = np.random.default_rng(seed)
    cs = rng.integers(0, 1 << 32, size=(n, 4), dtype=np.uint64)
    ks = rng.integers(0, 1 << 32, size=(n, 2), dtype=np.uint64)
    edge = [((0, 0, 0, 0), (0, 0)), ((MASK,) * 4, (MASK, MASK)), ((1, 0, 0, 0), (0, 0)),
            ((0, 0, 0, 0), (1, 0)), ((MASK, 0, MASK, 0), (0, MASK))]
    return edge + [(tuple(int(x) for x in c), tuple(int(x) for x in k)) for c, k in zip(cs, ks)]


def test_against_big_integer_implementation():
    for ctr, key in _cases(10000, 3):
        assert oracle.philox4x32_10(ctr, key) == philox_bigint(ctr, key)


def test_is_a_bijection_on_counters():
    for ctr, key in _cases(500, 4):
        assert philox_inverse(oracle.philox4x32_10(ctr, key), key) == ctr


@pytest.fixture(scope="module")
def aten_philox(tmp_path_factory):
    import torch
    inc = os.path.join(os.path.dirname(torch.__file__), "include")
    src = os.path.join(os.path.dirname(__file__), "philox_aten_shim.cpp")
    so = str(tmp_path_factory.mktemp("aten") / "libaten_philox.so")
    try:
        subprocess.check_call(["g++", "-O1", "-std=c++17", "-shared", "-fPIC", "-I", inc, src, "-o", so],
                              stderr=subprocess.STDOUT)
    except (subprocess.CalledProcessError, FileNotFoundError) as e:   # pragma: no cover
        pytest.skip(f"cannot build the ATen Philox shim: {e}")
    lib = ctypes.CDLL(so)
    lib.aten_philox_words.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64,
                                      ctypes.c_uint32, ctypes.POINTER(ctypes.c_uint32)]
    lib.aten_philox_words.restype = None
    return lib


def test_against_pytorch_header_engine(aten_philox):
    """The engine in PyTorch's headers: key = seed (lo,hi), counter = (offset lo,hi, subsequence lo,hi);
    it hands out the four words of one counter value in order, then steps the offset."""
    rng = np.random.default_rng(5)
    for _ in range(300):
        seed, sub, off = (int(x) for x in rng.integers(0, 1 << 63, size=3, dtype=np.uint64))
        out = (ctypes.c_uint32 * 8)()
        aten_philox.aten_philox_words(seed, sub, off, 8, out)
        key = (seed & MASK, seed >> 32)
        for blk in range(2):
            o = off + blk
            ctr = (o & MASK, (o >> 32) & MASK, sub & MASK, sub >> 32)
            assert oracle.philox4x32_10(ctr, key) == tuple(out[4 * blk:4 * blk + 4])


def test_dropout_mask_definition_small():
    """Mask bytes against the stated mapping, evaluated with the big-integer Philox."""
    seed, off, n, p = 0x0123456789ABCDEF, (1 << 32) - 2, 23, 0.1
    thr = int(p * 2 ** 32)
    assert oracle.dropout_threshold(p) == thr == 429496729
    st = np.array([seed, off], dtype=np.uint64)
    mask = oracle.dropout_mask(st, n, p)
    key = (seed & MASK, seed >> 32)
    for j in range(n):
        o = off + j // 4                              # crosses the 32-bit carry
        w = philox_bigint((o & MASK, o >> 32, 0, 0), key)[j % 4]
        assert mask[j] == (1 if w >= thr else 0)
    assert int(st[0]) == seed and int(st[1]) == off + 6      # ceil(23/4)


def test_dropout_threshold_edges():
    assert oracle.dropout_threshold(0.0) == 0
    assert oracle.dropout_threshold(1.0) == 1 << 32
    assert oracle.dropout_threshold(0.5) == 1 << 31
    st = np.array([1, 0], dtype=np.uint64)
    assert oracle.dropout_mask(st, 64, 0.0).all()
    assert not oracle.dropout_mask(st, 64, 1.0).any()


def test_keep_rate():
    n, p = 32 * 128 * 768, 0.1
    st = np.array([42, 0], dtype=np.uint64)
    mask = oracle.dropout_mask(st, n, p)
    keep = mask.mean()
    sigma = (p * (1 - p) / n) ** 0.5
    assert abs(keep - (1 - p)) < 4 * sigma
    assert set(np.unique(mask)) <= {0, 1}


def test_stream_splits_at_aligned_boundary():
    p = 0.3
    a = np.array([99, 1000], dtype=np.uint64)
    whole = oracle.dropout_mask(a, 4 * 50 + 4 * 31 + 3, p)
    b = np.array([99, 1000], dtype=np.uint64)
    first = oracle.dropout_mask(b, 4 * 50, p)
    second = oracle.dropout_mask(b, 4 * 31 + 3, p)
    assert np.array_equal(whole, np.concatenate([first, second]))
    assert np.array_equal(a, b)
    # a ragged first call still consumes whole counter values
    c = np.array([99, 1000], dtype=np.uint64)
    oracle.dropout_mask(c, 5, p)
    assert int(c[1]) == 1002
