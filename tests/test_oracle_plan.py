"""Pins for the oracle of the scheduler's performance model (paper section 3.4, Eq. 1a-1d):
hand-worked rational examples, closed forms, an exact-arithmetic characterisation of the
optimum, and the case that decides how Eq. 1c has to be read."""
from fractions import Fraction
from itertools import product

import numpy as np
import pytest

from oracle import plan_model as PM


def test_hand_worked_three_types():
    # capabilities 4, 2, 1 mini-batches/s, one GPU each
    C = [4.0, 2.0, 1.0]
    p = PM.evaluate(C, [1, 1, 1], [4, 2, 1], 7)               # perfectly balanced, nothing spare
    assert (p.n_est, p.f_overload, p.waste, p.throughput) == (7, 1.0, 0.0, 7.0)
    # one EST too many on the slowest type: it now needs 2 s per step and holds the others back
    p = PM.evaluate(C, [1, 1, 1], [4, 2, 2], 7)
    assert p.n_est == 8 and p.f_overload == 2.0
    # idle: (4 - 4/2) + (2 - 2/2) + (1 - 2/2) = 3; over-provisioned: (8 - 7)/2 = 0.5
    assert p.waste == 3.5 and p.throughput == 3.5
    # the over-provisioning term alone: balanced but one place more than needed
    p = PM.evaluate(C, [1, 1, 1], [4, 2, 1], 6)
    assert p.waste == 1.0 and p.throughput == 6.0


def test_homogeneous_closed_form():
    # N GPUs of one type, maxP = N * a: no waste, estimate = N * C
    for n, a, c in [(1, 1, 8.0), (4, 2, 16.0), (8, 4, 0.5), (3, 8, 32.0)]:
        p = PM.evaluate([c], [n], [a], n * a)
        assert p.waste == 0.0 and p.throughput == n * c and p.f_overload == a / c


def test_unused_types_do_not_count():
    a = PM.evaluate([4.0, 2.0], [2, 0], [3, 0], 6)
    b = PM.evaluate([4.0], [2], [3], 6)
    assert (a.n_est, a.f_overload, a.waste, a.throughput) == (b.n_est, b.f_overload, b.waste, b.throughput)
    assert a.est_per_gpu == (3, 0)


def exact_throughput(C, N, A, max_p):
    f = max(Fraction(A[i]) / Fraction(C[i]) for i in range(len(C)) if N[i] > 0)
    return Fraction(max_p) / f


def test_estimate_equals_useful_minibatches_per_step_time():
    """With the idle term weighted per GPU, Eq. 1d collapses to maxP / f_overload."""
    rng = np.random.default_rng(7)
    for _ in range(300):
        K = int(rng.integers(1, 5))
        C = [float(rng.integers(1, 64)) / 4 for _ in range(K)]
        N = [int(rng.integers(0, 5)) for _ in range(K)]
        if sum(N) == 0:
            N[0] = 1
        A = [int(rng.integers(1, 9)) if N[i] else 0 for i in range(K)]
        n_est = sum(n * a for n, a in zip(N, A))
        max_p = int(rng.integers(1, n_est + 1))
        p = PM.evaluate(C, N, A, max_p)
        want = exact_throughput(C, N, A, max_p)
        assert abs(p.throughput - float(want)) <= 1e-12 * float(want) * (4 + sum(N))


def test_printed_sum_overestimates_with_several_gpus_of_an_underloaded_type():
    """The case that decides the reading of Eq. 1c.  One fast-loaded GPU (10 ESTs at 10/s: 1 s
    per step) and four GPUs given 5 ESTs each at 10/s.  A step takes 1 s and carries
    10 + 4*5 = 30 mini-batches: 30 per second is all this plan can deliver."""
    C, N, A = [10.0, 10.0], [1, 4], [10, 5]
    per_gpu = PM.evaluate(C, N, A, 30, per_gpu=True)
    printed = PM.evaluate(C, N, A, 30, per_gpu=False)
    assert per_gpu.throughput == 30.0 and per_gpu.waste == 20.0
    assert printed.waste == 5.0 and printed.throughput == 45.0          # > nEST / f_overload = 30
    assert printed.throughput > per_gpu.n_est / per_gpu.f_overload
    # with one GPU per type the two readings are the same formula
    for A1 in ([10, 5], [3, 7]):
        x = PM.evaluate(C, [1, 1], A1, 8, per_gpu=True)
        y = PM.evaluate(C, [1, 1], A1, 8, per_gpu=False)
        assert (x.waste, x.throughput) == (y.waste, y.throughput)


def exact_optimum_f(C, N, max_p):
    """Independent characterisation in exact arithmetic: the smallest step time t of the form
    a / C[i] for which the GPUs can hold maxP ESTs when type i takes floor(t * C[i]) >= 1."""
    used = [i for i in range(len(C)) if N[i] > 0]
    cands = sorted({Fraction(a) / Fraction(C[i]) for i in used for a in range(1, max_p + 1)})
    for t in cands:
        caps = [int(t * Fraction(C[i])) for i in used]
        if min(caps) >= 1 and sum(N[i] * min(c, max_p) for i, c in zip(used, caps)) >= max_p:
            return t
    raise AssertionError("no feasible step time")


def test_best_mapping_hand_cases():
    C = [4.0, 2.0, 1.0]
    p = PM.best_mapping(C, [1, 1, 1], 7)
    assert p.est_per_gpu == (4, 2, 1) and p.throughput == 7.0
    # 8 ESTs do not fit at 1 s per step; the cheapest way out is a fifth EST on the fastest GPU
    p = PM.best_mapping(C, [1, 1, 1], 8)
    assert p.est_per_gpu == (5, 2, 1) and p.f_overload == 1.25 and p.n_est == 8
    assert abs(p.throughput - 6.4) < 1e-12
    # more GPUs than ESTs: no plan
    assert PM.best_mapping(C, [2, 2, 1], 4) is None
    assert PM.best_mapping(C, [0, 0, 0], 4) is None
    # ties in step time are broken towards less over-provisioning, then the smaller vector
    p = PM.best_mapping([2.0, 2.0], [1, 1], 3)
    assert p.est_per_gpu == (1, 2) and p.n_est == 3 and p.f_overload == 1.0


def test_best_mapping_reaches_the_exact_optimum():
    rng = np.random.default_rng(11)
    for _ in range(60):
        K = int(rng.integers(1, 4))
        C = [float(rng.integers(1, 24)) / 2 for _ in range(K)]
        N = [int(rng.integers(0, 3)) for _ in range(K)]
        if sum(N) == 0:
            N[int(rng.integers(0, K))] = 1
        max_p = int(rng.integers(sum(N), 9))
        p = PM.best_mapping(C, N, max_p)
        t = exact_optimum_f(C, N, max_p)
        assert Fraction(p.f_overload) == t or abs(p.f_overload - float(t)) <= 1e-15 * float(t)
        assert p.n_est >= max_p
        # no allocation with the same step time needs fewer places
        used = [i for i in range(K) if N[i] > 0]
        caps = [min(max_p, int(t * Fraction(C[i]))) for i in used]
        sums = {sum(N[i] * a for i, a in zip(used, ch)) for ch in product(*[range(1, c + 1) for c in caps])}
        assert p.n_est == min(s for s in sums if s >= max_p)


def test_plan_database_is_ranked_and_monotone():
    C = [4.0, 2.0, 1.0]
    plans = PM.enumerate_plans(C, [2, 1, 2], 6)
    assert len(plans) == sum(1 for N in product(range(3), range(2), range(3)) if 1 <= sum(N) <= 6)
    keys = [p.key() for p in plans]
    assert keys == sorted(keys)
    # two fast GPUs with 3 ESTs each: 0.75 s per step.  Adding the medium GPU cannot shorten that
    # (at 0.5 s the three hold only 2 + 2 + 1 = 5 < 6); a slow GPU needs 1 s for its single EST
    assert (plans[0].n_used, plans[0].est_per_gpu, plans[0].throughput) == ((2, 0, 0), (3, 0, 0), 8.0)
    assert (plans[1].n_used, plans[1].f_overload) == ((2, 1, 0), 0.75)
    # more GPUs on offer never lower the best estimate; scaling every capability scales it
    best = plans[0].throughput
    assert PM.enumerate_plans(C, [2, 1, 3], 6)[0].throughput >= best
    assert PM.enumerate_plans(C, [1, 1, 2], 6)[0].throughput <= best
    scaled = PM.enumerate_plans([2 * c for c in C], [2, 1, 2], 6)
    assert [p.n_used for p in scaled] == [p.n_used for p in plans]
    assert [p.throughput for p in scaled] == [2 * p.throughput for p in plans]
    assert PM.enumerate_plans(C, [2, 1, 2], 6, top_k=3) == plans[:3]


@pytest.mark.parametrize("N,A,max_p", [((1, 1, 1), (5, 2, 1), 8), ((2, 3), (4, 3), 12), ((2, 3), (4, 3), 5),
                                       ((4,), (2,), 5), ((1, 2, 1), (1, 1, 1), 4)])
def test_grouping_of_a_plan(N, A, max_p):
    plan = PM.evaluate([1.0] * len(N), list(N), list(A), max_p)
    worker_of, slot_of = PM.grouping(plan, max_p)
    n_workers = sum(N)
    assert len(worker_of) == len(slot_of) == max_p
    assert worker_of == sorted(worker_of) and set(worker_of) == set(range(n_workers))
    cap = [a for n, a in zip(N, A) for _ in range(n)]
    for w in range(n_workers):
        slots = [s for ww, s in zip(worker_of, slot_of) if ww == w]
        assert slots == list(range(len(slots))) and 1 <= len(slots) <= cap[w]
    # places are given back from the last GPU backwards, one per pass
    sizes = [worker_of.count(w) for w in range(n_workers)]
    slack = plan.n_est - max_p
    assert sum(cap) - sum(sizes) == slack
    if 0 < slack <= n_workers and min(cap) > 1:
        assert [c - s for c, s in zip(cap, sizes)] == [0] * (n_workers - slack) + [1] * slack
