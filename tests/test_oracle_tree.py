"""Pins of the oracle's fixed-tree sum of squares."""
import math

import numpy as np
import pytest

import oracle


def twin(x):
    """The same tree from reshapes and slice adds (written independently of the C loops)."""
    f = np.float32
    x = np.asarray(x, dtype=f)
    n = x.size
    nblk = -(-n // 4096)
    pad = np.zeros(max(nblk, 1) * 4096, dtype=f)
    pad[:n] = x
    sq = (pad * pad).reshape(max(nblk, 1), 4, 256, 4)         # [block, q, lane, c]
    lane = np.zeros((max(nblk, 1), 256), dtype=f)
    for q in range(4):
        for c in range(4):
            lane = lane + sq[:, q, :, c]

    def tree(v):
        s = 128
        while s >= 1:
            v = v[..., :s] + v[..., s:2 * s]
            s //= 2
        return v[..., 0]

    part = tree(lane)[:nblk]
    rows = -(-max(nblk, 1) // 256)
    p2 = np.zeros(rows * 256, dtype=f)
    p2[:nblk] = part
    p2 = p2.reshape(rows, 256)
    lane2 = np.zeros(256, dtype=f)
    for k in range(rows):
        lane2 = lane2 + p2[k]
    return f(tree(lane2))


@pytest.mark.parametrize("n", [0, 1, 2, 255, 256, 1023, 4095, 4096, 4097, 8191, 3 * 4096 + 37,
                               256 * 4096, 256 * 4096 + 1, 1_300_003])
def test_matches_numpy_twin(n):
    rng = np.random.default_rng(n)
    x = (rng.standard_normal(n) * np.exp2(rng.integers(-12, 12, n))).astype(np.float32)
    got = oracle.tree_sumsq(x)
    assert np.float32(got).view(np.uint32) == twin(x).view(np.uint32)


def test_exact_cases():
    assert oracle.tree_sumsq(np.zeros(0, dtype=np.float32)) == 0.0
    for n in (1, 4096, 4097, 100_003, (1 << 22) + 5):
        assert oracle.tree_sumsq(np.ones(n, dtype=np.float32)) == float(n)       # exact below 2^24
    rng = np.random.default_rng(1)
    x = rng.integers(-15, 16, 50_021).astype(np.float32)                        # squares <= 225: exact sum
    assert oracle.tree_sumsq(x) == float((x.astype(np.int64) ** 2).sum())
    for pos in (0, 1, 4095, 4096, 70_000, 99_999):                               # one element, anywhere
        x = np.zeros(100_000, dtype=np.float32)
        x[pos] = np.float32(1.7)
        assert oracle.tree_sumsq(x) == np.float32(1.7) * np.float32(1.7)


def test_error_bound_and_order_dependence():
    rng = np.random.default_rng(2)
    n = 777_777
    x = rng.standard_normal(n).astype(np.float32)
    exact = math.fsum(float(v) * float(v) for v in x)
    got = float(oracle.tree_sumsq(x))
    depth = 16 + 8 + (-(-n // 4096) // 256 + 1) + 8 + 1          # adds on the longest path, + the square
    assert abs(got - exact) <= depth * 2.0 ** -24 * exact * 1.01
    # the tree is a fixed function of positions: a plain running sum differs in the last bits
    naive = np.float32(0)
    for v in (x[:20000] * x[:20000]):
        naive = np.float32(naive + v)
    assert np.float32(oracle.tree_sumsq(x[:20000])).view(np.uint32) != naive.view(np.uint32)


# ---- hand-derived order witnesses (tests/golden/tree_witness.txt) ----------------------
def witness_inputs():
    """The two input vectors the golden file describes, built from its own wording."""
    def elem(lane, q, c):
        return 4 * (256 * q + lane) + c
    a = np.zeros(4096, dtype=np.float32)
    a[elem(0, 1, 0)] = 4096
    for pos in ((0, 0, 0), (0, 0, 1), (0, 1, 1), (128, 0, 0), (128, 0, 1), (128, 0, 2), (64, 0, 0),
                (192, 0, 0), (192, 2, 3), (1, 0, 0), (2, 3, 3)):
        a[elem(*pos)] = 1
    b = np.zeros(515 * 4096, dtype=np.float32)
    b[0] = 4096
    for blk in (255, 256, 257, 512):
        b[4096 * blk] = 1
    return {"A": a, "B": b}


def golden_witness():
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "tree_witness.txt")
    rows = {}
    for line in open(path):
        if line.strip() and not line.startswith("#"):
            name, n, val, bits_hex = line.split()
            rows[name] = (int(n), np.float32(float(val)), int(bits_hex, 16))
    return rows


def test_hand_derived_tree_witness():
    inputs, gold = witness_inputs(), golden_witness()
    assert set(gold) == {"A", "B"}
    for name, x in inputs.items():
        n, val, want_bits = gold[name]
        assert x.size == n and int(val.view(np.uint32)) == want_bits
        got = np.float32(oracle.tree_sumsq(x))
        assert int(got.view(np.uint32)) == want_bits, (name, float(got))


def test_witness_tells_other_summation_orders_apart():
    """What the golden file says about other conventions, checked: each gives another value on the
    witness, so a tree that is wrong in one of these ways cannot pass it."""
    f = np.float32
    a = witness_inputs()["A"]
    sq = a * a
    base = f(2.0 ** 24)

    def halving(lane):
        s = lane.size // 2
        while s >= 1:
            lane = lane[:s] + lane[s:2 * s]
            s //= 2
        return lane[0]

    running = f(0)
    for v in sq[np.nonzero(sq)[0]]:
        running = f(running + v)
    pairs = sq.copy()
    while pairs.size > 1:
        pairs = pairs[0::2] + pairs[1::2]
    lanes = np.zeros(256, dtype=f)
    for q in range(4):
        for c in range(4):
            lanes = lanes + sq.reshape(4, 256, 4)[q, :, c]
    adjacent = lanes.copy()
    while adjacent.size > 1:
        adjacent = adjacent[0::2] + adjacent[1::2]
    c_outer = np.zeros(256, dtype=f)
    for c in range(4):
        for q in range(4):
            c_outer = c_outer + sq.reshape(4, 256, 4)[q, :, c]
    strided = np.zeros(256, dtype=f)
    for k in range(16):
        strided = strided + sq.reshape(16, 256)[k]
    assert halving(lanes) - base == 12                     # the specified tree, written a second time
    assert running - base == 8 and pairs[0] - base == 10 and adjacent[0] - base == 8
    assert halving(c_outer) - base == 8 and halving(strided) - base == 8

    b = witness_inputs()["B"]
    part = (b[::4096] * b[::4096]).astype(f)
    rows = np.zeros(3 * 256, dtype=f)
    rows[:part.size] = part
    rows = rows.reshape(3, 256)
    assert halving((rows[0] + rows[1]) + rows[2]) - base == 2        # partials t, t+256, t+512 in that order
    assert halving((rows[2] + rows[1]) + rows[0]) - base == 4        # descending instead
    run = f(0)
    for v in part:
        run = f(run + v)
    assert run - base == 0
