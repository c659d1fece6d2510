"""The oracle's own EST model: time-slicing, grouping and context switching change nothing.

Pin: N ranks that never switch (oracle.ddp_reference) are the definition; the
time-sliced model has to reproduce them bit for bit under every grouping
(paper §3.1 / §3.3 D1).  A negative control shows the comparison sees a
context mix-up."""
import numpy as np
import pytest

from scenario import Scenario, assert_same, run_ddp_reference, run_est_model
from workloads import buckets, configs


def small_scenario(N, A=1, seed=1):
    lay = buckets.custom([37, 0, 1024 + 3, 5, 4 * N + 1], fan_in=4)
    return Scenario(N, lay, A, seed, steps=3, mask_n=203, p_drop=0.1, bn_channels=(3, 8, 1))


@pytest.mark.parametrize("N", [1, 2, 5, 8])
def test_grouping_invariance(N):
    sc = small_scenario(N, A=1 if N % 2 else 4, seed=N)
    ref = run_ddp_reference(sc)
    gs = [configs.contiguous([N]), configs.contiguous([1] * N, "1xN")]
    if N == 5:
        gs += [configs.contiguous([2, 3]), configs.round_robin([2, 3])]
    if N == 8:
        gs += [configs.contiguous([4, 4]), configs.round_robin([3, 5]), configs.contiguous([1, 7])]
    gs += [configs.reversed_slots(g) for g in gs]
    for g in gs:
        assert_same(run_est_model(sc, g), ref, g.name)


def test_state_actually_evolves():
    sc = small_scenario(4)
    ref = run_ddp_reference(sc)
    assert len(ref.masks) == 12 and len(set(ref.masks.values())) == 12
    assert np.all(ref.philox[:, 1] == 3 * ((203 + 3) // 4))
    assert len({r.tobytes() for r in ref.bn}) == 4
    assert np.any(ref.v != 0) and np.any(ref.avg != 0)


def test_negative_control_swapped_contexts_are_seen():
    """Restoring a neighbour's context (a slot mix-up) must change the outcome."""
    from oracle.est_model import ESTModel
    sc = small_scenario(4)
    ref = run_ddp_reference(sc)

    class Broken(ESTModel):
        def ctx_restore(self, e):
            super().ctx_restore(e ^ 1 if self.worker_of_est[e] == self.worker_of_est[e ^ 1] else e)

    import oracle.est_model as em
    orig = em.ESTModel
    em.ESTModel = Broken
    try:
        got = run_est_model(sc, configs.contiguous([4]))
    finally:
        em.ESTModel = orig
    with pytest.raises(AssertionError):
        assert_same(got, ref, "broken")


def test_checkpoint_and_redistribution_change_nothing():
    """Paper section 3.2/5.1.1: scale 1 worker -> 3 workers -> 2 workers through on-demand
    checkpoints; the result equals the uninterrupted N-rank run."""
    sc = small_scenario(6, A=4, seed=9)
    sc = Scenario(sc.n_logical, sc.layout, sc.chunk_align, sc.seed, 4, sc.lr, sc.momentum,
                  sc.mask_n, sc.p_drop, sc.bn_channels)
    ref = run_ddp_reference(sc)
    got = run_est_model(sc, configs.contiguous([6]),
                        regroup_at={1: configs.round_robin([1, 2, 3]), 3: configs.contiguous([4, 2])})
    assert_same(got, ref, "checkpointed")
