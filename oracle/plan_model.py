"""The scheduler's analytical performance model and plan search, written out plainly.
TEST INFRASTRUCTURE ONLY.

Paper section 3.4 ("Companion module"), Eq. 1a-1d.  A job may use N[i] GPUs of type
i; one GPU of type i processes C[i] mini-batches per second of this workload and is
given at most A[i] ESTs (one mini-batch per EST per global step):

    1a  nEST       = sum_i N[i] * A[i]                  with nEST >= maxP
    1b  f_overload = max over used types of A[i] / C[i]          (seconds per global step:
                     the most loaded type holds everybody back, training is synchronous)
    1c  waste      = sum over used types of idle capability + (nEST - maxP) / f_overload
    1d  throughput = sum_i N[i] * C[i] - waste

Reading of Eq. 1c (the printed sum carries no factor N[i] although 1a and 1d count every
GPU): ``per_gpu=True`` weights the idle capability C[i] - A[i]/f_overload of a type by its
N[i] GPUs.  Only then is the model consistent with itself: the estimate equals
maxP / f_overload, the useful mini-batches of a global step over the step's duration.
``per_gpu=False`` is the sum as printed; with several GPUs of an under-loaded type it
estimates more than nEST / f_overload, which no plan can deliver (pinned by a test).

Arithmetic is IEEE double in the order written here.  The search is brute force over every
integer allocation; nothing is pruned, so it is for small cases.
"""
from __future__ import annotations

from dataclasses import dataclass
from itertools import product
from typing import List, Optional, Sequence, Tuple


@dataclass(frozen=True)
class Plan:
    n_used: Tuple[int, ...]          # N[i]
    est_per_gpu: Tuple[int, ...]     # A[i], 0 where N[i] == 0
    n_est: int                       # Eq. 1a
    f_overload: float                # Eq. 1b
    waste: float                     # Eq. 1c
    throughput: float                # Eq. 1d

    @property
    def n_gpus(self) -> int:
        return sum(self.n_used)

    def key(self):
        """Ranking: fastest global step first (= highest estimate in exact arithmetic), then
        fewer GPUs, then less over-provisioning, then the smaller vectors."""
        return (self.f_overload, self.n_gpus, self.n_est, self.n_used, self.est_per_gpu)


def evaluate(C: Sequence[float], N: Sequence[int], A: Sequence[int], max_p: int,
             per_gpu: bool = True) -> Plan:
    """Eq. 1a-1d for one EST-to-GPU mapping configuration."""
    K = len(C)
    assert len(N) == K and len(A) == K and max_p >= 1
    used = [i for i in range(K) if N[i] > 0]
    assert used and all(A[i] >= 1 for i in used) and all(C[i] > 0 for i in range(K))
    n_est = 0
    for i in range(K):
        n_est += N[i] * A[i]                                   # 1a
    assert n_est >= max_p
    f = 0.0
    for i in used:
        f = max(f, float(A[i]) / float(C[i]))                  # 1b
    waste = 0.0
    for i in used:
        idle = float(C[i]) - float(A[i]) / f
        waste = waste + (float(N[i]) * idle if per_gpu else idle)
    waste = waste + float(n_est - max_p) / f                   # 1c
    cap = 0.0
    for i in range(K):
        cap = cap + float(N[i]) * float(C[i])
    return Plan(tuple(N), tuple(A[i] if N[i] > 0 else 0 for i in range(K)), n_est, f, waste,
                cap - waste)                                   # 1d


def best_mapping(C: Sequence[float], N: Sequence[int], max_p: int) -> Optional[Plan]:
    """The best allocation A for fixed GPU counts N: every A[i] in 1..maxP on used types,
    nEST >= maxP, smallest key.  None when the GPUs outnumber the ESTs."""
    K = len(C)
    used = [i for i in range(K) if N[i] > 0]
    if not used or sum(N) > max_p:
        return None
    best = None
    for choice in product(range(1, max_p + 1), repeat=len(used)):
        A = [0] * K
        for i, a in zip(used, choice):
            A[i] = a
        if sum(N[i] * A[i] for i in used) < max_p:
            continue
        plan = evaluate(C, N, A, max_p)
        if best is None or plan.key() < best.key():
            best = plan
    return best


def enumerate_plans(C: Sequence[float], available: Sequence[int], max_p: int,
                    top_k: Optional[int] = None) -> List[Plan]:
    """The plan database: for every choice of GPU counts 0 <= N[i] <= available[i] (at least
    one GPU, no more GPUs than ESTs) its best mapping, ranked by key."""
    plans = []
    for N in product(*[range(a + 1) for a in available]):
        p = best_mapping(C, N, max_p)
        if p is not None:
            plans.append(p)
    plans.sort(key=Plan.key)
    return plans if top_k is None else plans[:top_k]


def grouping(plan: Plan, max_p: int) -> Tuple[List[int], List[int]]:
    """EST-to-worker mapping of a plan: GPUs in type order, each with a quota of A[type]
    ESTs; the over-provisioned nEST - maxP places are given back one at a time, going over
    the GPUs from the last to the first again and again and never emptying one; virtual
    ranks are then dealt out contiguously.  Returns (worker_of_est, slot_of_est)."""
    quota = []
    for i, n in enumerate(plan.n_used):
        quota += [plan.est_per_gpu[i]] * n
    slack = plan.n_est - max_p
    assert len(quota) <= max_p
    while slack > 0:
        for g in range(len(quota) - 1, -1, -1):
            if slack > 0 and quota[g] > 1:
                quota[g] -= 1
                slack -= 1
    worker_of, slot_of = [], []
    for g, q in enumerate(quota):
        worker_of += [g] * q
        slot_of += list(range(q))
    assert len(worker_of) == max_p
    return worker_of, slot_of
