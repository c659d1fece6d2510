"""Pins of the oracle-side model of host-swapped gradient contexts: the two-buffer schedule."""
import numpy as np
import pytest

import oracle
from oracle.est_model import SwappedESTModel, run_swap_in, swap_in_schedule


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def problem(seed, n_ranks=5, lens=(37, 0, 4, 1000, 1, 513, 64)):
    rng = np.random.default_rng(seed)
    rows = [rng.standard_normal((n_ranks, L)).astype(np.float32) for L in lens]
    want = [oracle.ring_order_reduce(r, 4) for r in rows]
    return rows, list(lens), want


def test_schedule_shape_by_hand():
    """Four buckets, written out: buffers alternate; fill b waits for reduce b-2, reduce b for fill b."""
    assert swap_in_schedule(4) == [
        ("fill", 0, 0, -1), ("reduce", 0, 0, 0),
        ("fill", 1, 1, -1), ("reduce", 1, 1, 2),
        ("fill", 2, 0, 1), ("reduce", 2, 0, 4),
        ("fill", 3, 1, 3), ("reduce", 3, 1, 6)]
    assert swap_in_schedule(0) == []


def test_every_legal_interleaving_gives_the_plain_reduce():
    rows, lens, want = problem(1)
    ops = swap_in_schedule(len(lens))
    for seed in [None] + list(range(40)):
        rng = None if seed is None else np.random.default_rng(seed)
        got = run_swap_in(ops, lambda b: rows[b], lens, 5, 4, rng)
        for b in range(len(lens)):
            assert np.array_equal(bits(got[b]), bits(want[b])), (seed, b)


def test_at_most_two_buckets_resident_and_in_order():
    """Replays the dependencies with the copy queue running as far ahead as it may: it can never be
    more than two buckets ahead of the reduce."""
    ops = swap_in_schedule(9)
    done, filled, reduced = set(), [], []
    progress = True
    while progress:
        progress = False
        for i, (kind, b, half, w) in enumerate(ops):          # greedy: fills first whenever allowed
            if i in done or (w >= 0 and w not in done):
                continue
            same_queue_before = [j for j in range(i) if ops[j][0] == kind]
            if any(j not in done for j in same_queue_before):
                continue
            if kind == "reduce" and any(ops[j][0] == "fill" and j not in done and
                                        (ops[j][3] < 0 or ops[j][3] in done) and
                                        all(k in done for k in range(j) if ops[k][0] == "fill")
                                        for j in range(len(ops))):
                continue                                        # a fill could still run: let it
            done.add(i)
            (filled if kind == "fill" else reduced).append(b)
            assert len(filled) - len(reduced) <= 2
            progress = True
            break
    assert filled == list(range(9)) and reduced == list(range(9))


def test_wrong_schedules_are_caught():
    rows, lens, want = problem(2)
    good = swap_in_schedule(len(lens))
    # a fill that does not wait for the previous user of its buffer
    bad = [(k, b, h, (-1 if k == "fill" else w)) for k, b, h, w in good]
    caught = 0
    for seed in range(40):
        try:
            got = run_swap_in(bad, lambda b: rows[b], lens, 5, 4, np.random.default_rng(seed))
            if any(not np.array_equal(bits(got[b]), bits(want[b])) for b in range(len(lens))):
                caught += 1
        except AssertionError:
            caught += 1
    assert caught > 0
    # a reduce that does not wait for its fill
    bad = [(k, b, h, (-1 if k == "reduce" else w)) for k, b, h, w in good]
    caught = 0
    for seed in range(40):
        try:
            got = run_swap_in(bad, lambda b: rows[b], lens, 5, 4, np.random.default_rng(seed))
            if any(not np.array_equal(bits(got[b]), bits(want[b])) for b in range(len(lens))):
                caught += 1
        except AssertionError:
            caught += 1
    assert caught > 0
    # one buffer only, filled before its reader is done
    bad = [(k, b, 0, w) for k, b, h, w in good]
    with pytest.raises((AssertionError, RuntimeError)):
        for seed in range(40):
            got = run_swap_in(bad, lambda b: rows[b], lens, 5, 4, np.random.default_rng(seed))
            for b in range(len(lens)):
                assert np.array_equal(bits(got[b]), bits(want[b]))
    # circular waits
    with pytest.raises(RuntimeError):
        run_swap_in([("fill", 0, 0, 1), ("reduce", 0, 0, 0)], lambda b: rows[b], lens, 5, 4)


def test_swapped_model_equals_the_resident_model():
    import scenario as S
    from workloads import buckets, configs
    lay = buckets.custom([3 * 4096 + 37, 0, 3, 1001, 20004], fan_in=9)
    sc = S.Scenario(6, lay, 4, 0x5AB, steps=3, mask_n=99, bn_channels=(5, 16))
    ref = S.run_ddp_reference(sc)
    g = configs.contiguous([2, 4])
    got = S.run_est_model(sc, g, model_cls=SwappedESTModel)
    S.assert_same(got, ref, "swapped model")
