"""A whole global step captured into a HIP graph on the job's single stream and replayed:
every library call of the step only launches kernels on the given stream (no allocation,
no memset, no host synchronisation), so the caller may capture it.  Each replay is checked
against the CPU oracle, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import scenario as S
from workloads import buckets, configs

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import gpu_harness as G
    from paper_2208_14228_amd import binding as B


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


@pytest.mark.parametrize("flow", ["separate calls", "one launch per EST boundary"])
def test_captured_step_replays_bit_exactly(flow):
    N, steps = 6, 4
    lay = buckets.custom([3 * 4096 + 37, 0, 3, 1001, 4 * N + 1, 40000], fan_in=9)
    sc = S.Scenario(N, lay, 4, 0x6A9, steps=steps, mask_n=517, bn_channels=(3, 64, 5))
    ref_by_step = [S.run_ddp_reference(S.Scenario(N, lay, 4, sc.seed, t + 1, sc.lr, sc.momentum,
                                                  sc.mask_n, sc.p_drop, sc.bn_channels))
                   for t in range(steps)]
    g = configs.contiguous([2, 4])
    sched = g.schedule()
    job = G.make_job(sc, g, use_streams="one")
    try:
        G.init_contexts(sc, job)
        # persistent buffers the graph reads: per-EST flat gradients, BN deltas; and writes: masks
        flat = [torch.zeros(lay.n_params, device=G.DEV) for _ in range(N)]
        delta = [torch.zeros(sc.bn_len, device=G.DEV) for _ in range(N)]
        masks = [torch.zeros(sc.mask_n, dtype=torch.uint8, device=G.DEV) for _ in range(N)]
        all_b = list(range(lay.n_buckets))

        def fill(t):
            for e in range(N):
                flat[e].copy_(torch.cat([S.grad(sc, t, e, b, G.DEV) for b in all_b]))
                delta[e].copy_(S.bn_delta(sc, t, e, G.DEV))
            torch.cuda.synchronize()

        def one_step_boundary():                          # what bench.py captures
            for k, e in enumerate(sched):
                prev = sched[k - 1] if k else None
                nxt = sched[k + 1] if k + 1 < len(sched) else None
                if nxt is not None and g.worker_of_est[nxt] != g.worker_of_est[e]:
                    nxt = None
                if prev is None or g.worker_of_est[prev] != g.worker_of_est[e]:
                    job.ctx_restore(e)
                job.dropout_mask(e, 0, masks[e], sc.p_drop)
                G.bn_add_live(sc, job, e, delta[e])
                B.check(B.es_est_boundary(job.h, e, nxt, all_b, [flat[e].data_ptr() + 4 * o for o, _ in lay.buckets]),
                        "es_est_boundary", job.h)
            job.reduce_sgd_step(sc.lr, sc.momentum)

        def one_step():
            if flow != "separate calls":
                return one_step_boundary()
            for k, e in enumerate(sched):
                prev = sched[k - 1] if k else None
                if prev is not None and g.worker_of_est[prev] == g.worker_of_est[e]:
                    job.ctx_switch(prev, e)
                else:
                    if prev is not None:
                        job.ctx_save(prev)
                    job.ctx_restore(e)
                job.dropout_mask(e, 0, masks[e], sc.p_drop)
                G.bn_add_live(sc, job, e, delta[e])
                job.accumulate_batch(e, all_b, [flat[e][o:o + l] for o, l in lay.buckets])
            job.ctx_save(sched[-1])
            job.reduce_sgd_step(sc.lr, sc.momentum)

        fill(0)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=job.main):
            one_step()
        torch.cuda.synchronize()
        # capture executes nothing: state is still the initial one
        for t in range(steps):
            fill(t)                                      # eager work between replays
            graph.replay()
            torch.cuda.synchronize()
            ref = ref_by_step[t]
            what = f"replay {t}"
            assert np.array_equal(bits(job.p.cpu().numpy()), bits(ref.p)), what
            assert np.array_equal(bits(job.v.cpu().numpy()), bits(ref.v)), what
            assert np.array_equal(bits(job.avg.cpu().numpy()), bits(ref.avg)), what
            for e in range(N):
                assert S.digest(masks[e].cpu().numpy()) == ref.masks[(t, e)], (what, e)
        got = G.collect(sc, job, ref_by_step[-1].masks)
        S.assert_same(got, ref_by_step[-1], "after graph replays")
    finally:
        job.close()
