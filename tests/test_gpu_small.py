"""HIP path vs. CPU oracle, bit for bit, at sizes the oracle finishes in seconds:
several tiles, ragged tails, empty buckets, every launch shape, every edge case."""
import itertools

import numpy as np
import pytest
import torch

import oracle
from oracle import fold_def
import scenario as S
from workloads import buckets, configs, synth

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import gpu_harness as G
    from paper_2208_14228_amd import binding as B
    from paper_2208_14228_amd.job import ESTJob


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def ragged_scenario(N, A, seed, **kw):
    # bucket lengths: several tiles + ragged tail, empty, shorter than N, odd, exactly one tile
    lay = buckets.custom([3 * 4096 + 37, 0, 3, 4096, 1001, 4 * N + 1, 20000 + N], fan_in=9)
    return S.Scenario(N, lay, A, seed, **kw)


@pytest.mark.parametrize("N,A", [(1, 1), (2, 4), (3, 1), (4, 4), (5, 4), (7, 1), (8, 4), (16, 4), (33, 1), (64, 4)])
def test_ragged_parity_with_context(N, A):
    sc = ragged_scenario(N, A, 100 + N, steps=2, mask_n=1003, bn_channels=(3, 64, 5))
    ref = S.run_ddp_reference(sc)
    g = configs.contiguous([N])
    S.assert_same(G.run_gpu(sc, g), ref, f"N={N} unfused")
    S.assert_same(G.run_gpu(sc, g, fused=True, use_streams=False), ref, f"N={N} fused")


def test_every_launch_shape_gives_the_same_bits():
    """Tile size, unroll, rank batch and the streaming hint are launch shape only."""
    N = 12
    sc = ragged_scenario(N, 4, 7, steps=1)
    ref = S.run_ddp_reference(sc)
    g = configs.contiguous([N])
    job = G.make_job(sc, g)
    try:
        G.init_contexts(sc, job)
        p0, v0 = job.p.clone(), job.v.clone()
        for tile, u, nb, nt, fused in itertools.product((256, 1024, 4096, 16384), (1, 2, 4),
                                                        (1, 2, 4, 8, 16), (0, 1), (False, True)):
            for k, v in (("reduce_tile_elems", tile), ("reduce_unroll", u),
                         ("reduce_rank_batch", nb), ("nontemporal", nt), ("nontemporal_pv", (u + nb) % 2)):
                job.set_option(k, v)
            job.p.copy_(p0); job.v.copy_(v0); job.avg.fill_(float("nan"))
            torch.cuda.synchronize()
            G.run_steps(sc, job, g, fused=fused)
            what = f"tile={tile} unroll={u} batch={nb} nt={nt} fused={fused}"
            assert np.array_equal(bits(job.avg.cpu().numpy()), bits(ref.avg)), what
            assert np.array_equal(bits(job.p.cpu().numpy()), bits(ref.p)), what
            assert np.array_equal(bits(job.v.cpu().numpy()), bits(ref.v)), what
        # big tiles (long contiguous reads per stream) mixed with small remainder tiles
        for ub, nbb, nt, fused in itertools.product((8, 16, 32), (1, 2, 4), (0, 1), (False, True)):
            if ub * nbb > 32:
                continue
            job.set_option("reduce_tile_elems", 2048)
            job.set_option("reduce_big_unroll", 0)
            job.set_option("reduce_big_rank_batch", nbb)
            job.set_option("reduce_big_unroll", ub)
            job.set_option("nontemporal", nt)
            job.set_option("nontemporal_pv", 1 - nt)
            job.p.copy_(p0); job.v.copy_(v0); job.avg.fill_(float("nan"))
            torch.cuda.synchronize()
            G.run_steps(sc, job, g, fused=fused)
            what = f"big unroll={ub} batch={nbb} nt={nt} fused={fused}"
            assert np.array_equal(bits(job.avg.cpu().numpy()), bits(ref.avg)), what
            assert np.array_equal(bits(job.p.cpu().numpy()), bits(ref.p)), what
            assert np.array_equal(bits(job.v.cpu().numpy()), bits(ref.v)), what
    finally:
        job.close()


def test_big_tiles_cover_large_chunks():
    """Chunks long enough to hold several big tiles plus a ragged remainder, N = 2 and 5."""
    for N, A in ((2, 4), (5, 1)):
        lay = buckets.custom([N * (2 * 32768 + 8192 + 13) + 3, 7, N * 8192], fan_in=3)
        sc = S.Scenario(N, lay, A, 31 + N, steps=2)
        ref = S.run_ddp_reference(sc)
        for ub in (8, 32):
            got = G.run_gpu(sc, configs.contiguous([N]), fused=(ub == 8),
                            options={"reduce_big_unroll": ub})
            S.assert_same(got, ref, f"N={N} big={ub}")


def _reduce_only(rank_grads: np.ndarray, A: int, fused=False):
    """One bucket, one step through the library; returns the averaged gradient."""
    N, L = rank_grads.shape
    job = ESTJob(N, L, [(0, L)], A)
    try:
        src = torch.from_numpy(np.ascontiguousarray(rank_grads)).to(G.DEV)
        for e in range(N):
            job.accumulate(e, 0, src[e])
        if fused:
            job.reduce_sgd_step(0.0, 0.0)
        else:
            job.ring_order_reduce()
        job.sync()
        return job.avg.cpu().numpy()
    finally:
        job.close()


def test_order_witness_on_gpu():
    m = 1000
    vals = np.array([2.0 ** 24, 1.0, -(2.0 ** 24), 1.0], dtype=np.float32)
    g = np.repeat(vals[:, None], 4 * m, axis=1)
    for fused in (False, True):
        avg = _reduce_only(g, 1, fused)
        want = np.repeat(np.array([0.25, 0.5, 0.5, 0.0], dtype=np.float32), m)
        assert np.array_equal(bits(avg), bits(want))
    assert np.array_equal(bits(_reduce_only(g, 1)), bits(oracle.ring_order_reduce(g, A=1)))


def test_n1_identity_signed_zero_and_denormals():
    rng = np.random.default_rng(0)
    x = rng.standard_normal(5000).astype(np.float32)
    x[:6] = [-0.0, 0.0, 1e-45, -1e-40, 1.1754942e-38, -1.1754942e-38]
    avg = _reduce_only(x[None, :], 4)
    assert np.array_equal(bits(avg), bits(x))


def test_denormal_sums_and_quotients_are_kept():
    N, L = 4, 4099
    rng = np.random.default_rng(1)
    g = (rng.standard_normal((N, L)) * 1e-39).astype(np.float32)      # all denormal
    g[:, 0] = [1e-45, -1e-45, 0.0, -0.0]
    want = oracle.ring_order_reduce(g, A=4)
    assert np.count_nonzero(want) > L // 2 and np.abs(want).max() < 1.2e-38
    assert np.array_equal(bits(_reduce_only(g, 4)), bits(want))
    assert np.array_equal(bits(_reduce_only(g, 4, fused=True)), bits(want))


@pytest.mark.parametrize("N", [3, 5, 6, 7])
def test_true_division_for_non_power_of_two(N):
    xs = np.arange(1, 20001, dtype=np.float32)
    g = np.zeros((N, xs.size), dtype=np.float32)
    g[N - 1] = xs
    want = oracle.ring_order_reduce(g, A=1)
    got = _reduce_only(g, 1)
    assert np.array_equal(bits(got), bits(want))
    assert np.any(got != xs * (np.float32(1) / np.float32(N)))         # a reciprocal multiply would differ


def _sgd_only(p, v, g, lr, mu):
    n = p.size
    job = ESTJob(1, n, [(0, n)], 1)
    try:
        job.p.copy_(torch.from_numpy(p)); job.v.copy_(torch.from_numpy(v)); job.avg.copy_(torch.from_numpy(g))
        torch.cuda.synchronize()
        job.sgd_step(lr, mu)
        job.sync()
        out = job.p.cpu().numpy(), job.v.cpu().numpy()
        # same through the fused kernel (N = 1: averaged gradient = gradient)
        job.p.copy_(torch.from_numpy(p)); job.v.copy_(torch.from_numpy(v))
        src = torch.from_numpy(g).to(G.DEV)
        torch.cuda.synchronize()
        job.accumulate(0, 0, src)
        job.reduce_sgd_step(lr, mu, store_avg=False)
        job.sync()
        fused = job.p.cpu().numpy(), job.v.cpu().numpy()
        return out, fused
    finally:
        job.close()


def test_sgd_is_not_contracted_to_fma():
    e = np.float32(1.0 + 2.0 ** -12)
    r = np.float32(1.0 + 2.0 ** -11)
    n = 1030                                            # vector body + scalar tail
    for p0, v0, g0, lr, mu in ((0.0, e, -r, 0.0, float(e)), (r, 0.0, e, float(e), 0.0)):
        p = np.full(n, p0, dtype=np.float32); v = np.full(n, v0, dtype=np.float32); g = np.full(n, g0, dtype=np.float32)
        pw, vw = p.copy(), v.copy()
        oracle.sgd_momentum(pw, vw, g, lr, mu)
        for got_p, got_v in _sgd_only(p, v, g, lr, mu):
            assert np.array_equal(bits(got_p), bits(pw)) and np.array_equal(bits(got_v), bits(vw))
    assert pw[0] == 0.0


def test_sgd_random_parity():
    rng = np.random.default_rng(3)
    n = 3 * 4096 + 3
    p, v, g = (rng.standard_normal(n).astype(np.float32) for _ in range(3))
    pw, vw = p.copy(), v.copy()
    oracle.sgd_momentum(pw, vw, g, 0.1, 0.9)
    for got_p, got_v in _sgd_only(p, v, g, 0.1, 0.9):
        assert np.array_equal(bits(got_p), bits(pw)) and np.array_equal(bits(got_v), bits(vw))


@pytest.mark.parametrize("n,p_drop,off", [(1, 0.1, 0), (15, 0.5, 3), (16, 0.1, 2 ** 32 - 1), (4099, 0.1, 2 ** 40),
                                           (100003, 0.9, 12345), (64, 0.0, 0), (64, 1.0, 0)])
def test_dropout_mask_parity(n, p_drop, off):
    seed = 0xFEEDFACE12345678
    for misalign in (0, 1):
        job = ESTJob(2, 4, [(0, 4)], 1, [16])
        try:
            st = np.array([seed, off], dtype=np.uint64)
            job.live_of(0)[0].copy_(torch.from_numpy(st.view(np.uint8)))
            torch.cuda.synchronize()
            buf = torch.full((n + 17,), 7, dtype=torch.uint8, device=G.DEV)
            mask = buf[misalign:misalign + n]
            job.dropout_mask(0, 0, mask, p_drop)
            job.sync()
            want_state = st.copy()
            want = oracle.dropout_mask(want_state, n, p_drop)
            assert np.array_equal(mask.cpu().numpy(), want)
            assert np.all(buf[misalign + n:].cpu().numpy() == 7) and np.all(buf[:misalign].cpu().numpy() == 7)
            got_state = job.live_of(0)[0].cpu().numpy().view(np.uint64)
            assert np.array_equal(got_state, want_state)
        finally:
            job.close()


def test_grouping_invariance_with_switch_and_unaligned_live_tensors():
    N = 8
    sc = ragged_scenario(N, 4, 55, steps=3, mask_n=517, bn_channels=(64, 3, 128, 1, 2048))
    ref = S.run_ddp_reference(sc)
    gs = [configs.contiguous([8]), configs.contiguous([4, 4]), configs.contiguous([1] * 8, "1x8"),
          configs.round_robin([3, 5]), configs.reversed_slots(configs.contiguous([2, 6]))]
    for g in gs:
        S.assert_same(G.run_gpu(sc, g), ref, g.name)
        S.assert_same(G.run_gpu(sc, g, fused=True, use_switch=True), ref, g.name + " switch")

    # live tensors at odd addresses: the byte path of the context copy.  (The Philox
    # state has to stay 8-byte aligned for the mask kernel, so only BN moves.)
    def odd_alloc(nb):
        base = torch.full((nb + 32,), 0xCD, dtype=torch.uint8, device=G.DEV)
        return base[16:16 + nb] if nb == 16 else base[1:1 + nb]
    S.assert_same(G.run_gpu(sc, gs[1], live_alloc=odd_alloc), ref, "unaligned live")


def test_regrouping_between_steps_keeps_contexts():
    """An elasticity event (paper §3.2): ESTs move to other workers between global steps."""
    N = 6
    sc = ragged_scenario(N, 1, 77, steps=3, mask_n=99, bn_channels=(5, 16))
    ref = S.run_ddp_reference(sc)
    g0, g1, g2 = configs.contiguous([6]), configs.contiguous([2, 4]), configs.round_robin([1, 2, 3])
    job = G.make_job(sc, g0)
    try:
        G.init_contexts(sc, job)
        masks = {}
        for t, g in enumerate((g0, g1, g2)):
            if t:
                job.set_grouping(g.worker_of_est, g.slot_of_est)
            G.run_steps(sc, job, g, masks=masks, steps=[t])
        S.assert_same(G.collect(sc, job, masks), ref, "regrouped")
    finally:
        job.close()


def test_state_errors_and_argument_checks():
    job = ESTJob(2, 1024, [(0, 512), (512, 512)], 4, [16, 64])
    h = job.h
    try:
        g = torch.zeros(512, device=G.DEV)
        assert B.es_accumulate(h, 2, 0, g.data_ptr()) == B.ES_EINVAL
        assert B.es_accumulate(h, 0, 2, g.data_ptr()) == B.ES_EINVAL
        assert B.es_accumulate(h, 0, 0, 0) == B.ES_EINVAL
        assert B.es_accumulate(h, 0, 0, g.data_ptr() + 2) == B.ES_EINVAL
        assert B.es_accumulate(h, 0, 0, g.data_ptr()) == B.ES_OK
        assert B.es_accumulate(h, 0, 0, g.data_ptr()) == B.ES_ESTATE          # twice
        assert B.es_ring_order_reduce(h, job.avg.data_ptr()) == B.ES_ESTATE   # not all present
        assert B.es_set_grouping(h, [0, 1], [0, 0]) == B.ES_ESTATE            # mid-step
        assert B.es_ring_order_reduce(h, job.avg.data_ptr() + 4) in (B.ES_EINVAL, B.ES_ESTATE)
        for e, b in ((0, 1), (1, 0)):
            assert B.es_accumulate(h, e, b, g.data_ptr()) == B.ES_OK
        # zero-copy production: write into the slot, then only mark it
        slot = B.es_grad_slot(h, 1, 1)
        assert slot and B.es_accumulate(h, 1, 1, slot) == B.ES_OK
        assert B.es_ring_order_reduce(h, job.avg.data_ptr() + 4) == B.ES_EINVAL
        assert B.es_ring_order_reduce(h, job.avg.data_ptr()) == B.ES_OK
        assert B.es_ring_order_reduce(h, job.avg.data_ptr()) == B.ES_ESTATE   # new step started
        assert B.es_ctx_save(h, 2) == B.ES_EINVAL
        assert B.es_ctx_switch(h, 0, 0) == B.ES_EINVAL
        assert B.es_ctx_switch(h, 0, 1) == B.ES_OK
        assert B.es_dropout_mask(h, 0, 1, g.data_ptr(), 4, 0.1) == B.ES_EINVAL   # not a 16-byte segment
        assert B.es_dropout_mask(h, 0, 0, g.data_ptr(), 4, 1.5) == B.ES_EINVAL
        assert B.es_set_option(h, "reduce_tile_elems", 100) == B.ES_EINVAL
        assert B.es_set_option(h, "no_such_option", 1) == B.ES_EINVAL
        assert B.es_set_grouping(h, [0, 0], [0, 0]) == B.ES_EINVAL
        assert B.es_set_grouping(h, [0, 2], [0, 0]) == B.ES_EINVAL
        assert B.es_set_grouping(h, [0, 1], [0, 0]) == B.ES_OK
        assert B.es_ctx_save(h, 0) == B.ES_ESTATE                             # bindings dropped
        assert B.es_ctx_switch(h, 0, 1) == B.ES_EINVAL                        # different workers now
        assert B.es_sync(h) == B.ES_OK
        # parameters, momentum and averaged gradient must be three separate buffers
        pp, vv, aa = job.p.data_ptr(), job.v.data_ptr(), job.avg.data_ptr()
        assert B.es_sgd_step(h, pp, pp, aa, 0.1, 0.9) == B.ES_EINVAL
        assert B.es_sgd_step(h, pp, vv, pp + 16, 0.1, 0.9) == B.ES_EINVAL
        assert B.es_sgd_step(h, pp, vv, aa, 0.1, 0.9) == B.ES_OK
        assert B.es_reduce_sgd_step(h, pp, pp + 64, 0, 0.1, 0.9) == B.ES_EINVAL
        assert B.es_reduce_sgd_step(h, pp, vv, vv, 0.1, 0.9) == B.ES_EINVAL
        assert B.es_reduce_sgd_step(h, pp, vv, 0, 0.1, 0.9) == B.ES_ESTATE     # valid buffers, nothing staged
        assert B.es_sync(h) == B.ES_OK
        st, q = B.es_query(h)
        assert st == 0 and q["n_params"] == 1024 and q["n_buckets"] == 2 and q["ctx_bytes"] == 80 and q["n_workers"] == 2
    finally:
        job.close()


def test_zero_copy_slots_match_copied_staging():
    """A bucket whose gradient already sits in the slot is only marked, not copied."""
    N, L = 4, 10007
    rng = np.random.default_rng(9)
    g = rng.standard_normal((N, L)).astype(np.float32)
    want = oracle.ring_order_reduce(g, A=4)
    job = ESTJob(N, L, [(0, L)], 4)
    try:
        src = torch.from_numpy(g).to(G.DEV)
        for e in range(N):
            job.accumulate(e, 0, src[e])                     # copies into the slots
        job.ring_order_reduce(); job.sync()
        assert np.array_equal(bits(job.avg.cpu().numpy()), bits(want))
        job.avg.zero_(); torch.cuda.synchronize()
        for e in range(N):                                   # next step: slots still hold the data
            B.check(B.es_accumulate(job.h, e, 0, B.es_grad_slot(job.h, e, 0)), "es_accumulate")
        job.ring_order_reduce(); job.sync()
        assert np.array_equal(bits(job.avg.cpu().numpy()), bits(want))
    finally:
        job.close()


def test_input_generator_gives_the_same_bits_on_cpu_and_gpu():
    from workloads import shapes
    lay = buckets.ddp_buckets(shapes.resnet50())
    for b in (0, 3):
        a = synth.gradient(lay, b, 0x5EED0002, 1, 5)
        c = synth.gradient(lay, b, 0x5EED0002, 1, 5, G.DEV).cpu()
        assert torch.equal(a.view(torch.int32), c.view(torch.int32))
    assert torch.equal(synth.params(lay, 9).view(torch.int32), synth.params(lay, 9, G.DEV).cpu().view(torch.int32))


def test_batched_staging_matches_per_bucket_staging():
    """es_accumulate_batch: merged contiguous runs, separate tensors, unaligned sources,
    empty buckets, more runs than one launch holds."""
    N = 3
    lens = [4096 + 8, 0, 12, 1000, 7] + [64] * 40          # 45 buckets, some not multiples of 4
    lay = buckets.custom(lens, fan_in=1)
    rng = np.random.default_rng(4)
    g = rng.standard_normal((N, lay.n_params)).astype(np.float32)
    want = np.concatenate([oracle.ring_order_reduce(np.ascontiguousarray(g[:, o:o + l]), A=1)
                           for o, l in lay.buckets])
    for variant in ("flat", "separate", "shifted"):
        job = ESTJob(N, lay.n_params, lay.buckets, 1)
        try:
            keep = []
            for e in range(N):
                if variant == "flat":                        # one flat source: runs merge
                    flat = torch.from_numpy(g[e]).to(G.DEV)
                    srcs = [flat[o:o + l] for o, l in lay.buckets]
                elif variant == "separate":                  # one allocation per bucket
                    srcs = [torch.from_numpy(g[e, o:o + l].copy()).to(G.DEV) for o, l in lay.buckets]
                else:                                        # sources at 4-byte (not 16-byte) alignment
                    flat = torch.zeros(lay.n_params + 1, device=G.DEV)
                    flat[1:].copy_(torch.from_numpy(g[e]))
                    srcs = [flat[1 + o:1 + o + l] for o, l in lay.buckets]
                keep.append(srcs)
                torch.cuda.synchronize()
                order = list(range(lay.n_buckets))
                if e == 1:
                    order = order[::-1]                      # any order of buckets within a batch
                job.accumulate_batch(e, order, [srcs[b] for b in order])
            job.ring_order_reduce(); job.sync()
            assert np.array_equal(bits(job.avg.cpu().numpy()), bits(want)), variant
        finally:
            job.close()


def test_batched_staging_validates_before_doing_anything():
    job = ESTJob(2, 64, [(0, 32), (32, 32)], 4)
    h = job.h
    try:
        g = torch.zeros(64, device=G.DEV)
        p0, p1 = g.data_ptr(), g.data_ptr() + 128
        assert B.es_accumulate_batch(h, 0, [0, 0], [p0, p0]) == B.ES_ESTATE       # duplicate in batch
        assert B.es_accumulate_batch(h, 0, [0, 2], [p0, p1]) == B.ES_EINVAL       # bad bucket
        assert B.es_accumulate_batch(h, 0, [0, 1], [p0, 0]) == B.ES_EINVAL        # null source
        assert B.es_accumulate_batch(h, 2, [0], [p0]) == B.ES_EINVAL
        # nothing was marked by the failed calls
        assert B.es_accumulate_batch(h, 0, [0, 1], [p0, p1]) == B.ES_OK
        assert B.es_accumulate_batch(h, 0, [1], [p1]) == B.ES_ESTATE              # already present
        assert B.es_accumulate_batch(h, 1, [], []) == B.ES_OK
        assert B.es_ring_order_reduce(h, job.avg.data_ptr()) == B.ES_ESTATE
        assert B.es_accumulate_batch(h, 1, [1, 0], [p1, p0]) == B.ES_OK
        assert B.es_ring_order_reduce(h, job.avg.data_ptr()) == B.ES_OK
        assert B.es_sync(h) == B.ES_OK
    finally:
        job.close()


def test_host_resident_gradient_slots_give_the_same_bits():
    """Memory-pressure mode: slots in pinned host memory (the paper's placement of EST gradients)."""
    N = 5
    sc = ragged_scenario(N, 4, 91, steps=2, mask_n=64, bn_channels=(8,))
    ref = S.run_ddp_reference(sc)
    g = configs.contiguous([2, 3])
    job = G.make_job(sc, configs.contiguous([N]))
    try:
        job.set_option("host_slots", 1)
        job.set_grouping(g.worker_of_est, g.slot_of_est)        # re-allocates the arenas on the host
        G.init_contexts(sc, job)
        masks = {}
        G.run_steps(sc, job, g, fused=True, masks=masks)
        S.assert_same(G.collect(sc, job, masks), ref, "host slots")
    finally:
        job.close()


def test_in_place_gradients_of_each_workers_last_est():
    """The last EST a worker runs is not staged (paper section 5.1.3): same bits, small and big tiles."""
    for N, sizes in ((5, [2, 3]), (16, [1] * 7 + [9]), (3, [3])):
        lay = buckets.custom([N * (32768 + 2048 + 13) + 3, 0, 7, 4 * N + 1, 4096], fan_in=3)
        sc = S.Scenario(N, lay, 4 if N != 3 else 1, 200 + N, steps=2)
        ref = S.run_ddp_reference(sc)
        g = configs.contiguous(sizes)
        sched = g.schedule()
        last = {e for k, e in enumerate(sched)
                if k + 1 == len(sched) or g.worker_of_est[sched[k + 1]] != g.worker_of_est[e]}
        job = G.make_job(sc, g, options={"reduce_big_unroll": 8} if N == 5 else None)
        try:
            G.init_contexts(sc, job)
            for t in range(sc.steps):
                keep = []
                for e in sched:
                    with job.stream_ctx():
                        flat = torch.cat([S.grad(sc, t, e, b, G.DEV) for b in range(lay.n_buckets)])
                    keep.append(flat)
                    if e in last and len(last) <= 8:
                        job.accumulate_in_place(e, flat)
                    else:
                        job.accumulate_batch(e, list(range(lay.n_buckets)),
                                             [flat[o:o + l] for o, l in lay.buckets])
                if t == 0:
                    job.ring_order_reduce(); job.sgd_step(sc.lr, sc.momentum)
                else:
                    job.reduce_sgd_step(sc.lr, sc.momentum)
                job.sync(); torch.cuda.synchronize()
            for name, got, want in (("avg", job.avg, ref.avg), ("p", job.p, ref.p), ("v", job.v, ref.v)):
                assert np.array_equal(bits(got.cpu().numpy()), bits(want)), (N, name)
        finally:
            job.close()


def test_in_place_state_rules():
    job = ESTJob(10, 64, [(0, 32), (32, 32)], 4)
    h = job.h
    try:
        g = torch.zeros(65, device=G.DEV)
        assert B.es_accumulate_in_place(h, 10, g.data_ptr()) == B.ES_EINVAL
        assert B.es_accumulate_in_place(h, 0, g.data_ptr() + 4) == B.ES_EINVAL        # not 16-byte aligned
        assert B.es_accumulate_in_place(h, 0, 0) == B.ES_EINVAL
        assert B.es_accumulate(h, 0, 1, g.data_ptr()) == B.ES_OK
        assert B.es_accumulate_in_place(h, 0, g.data_ptr()) == B.ES_ESTATE            # a bucket already present
        for e in range(1, 9):
            assert B.es_accumulate_in_place(h, e, g.data_ptr()) == B.ES_OK
        assert B.es_accumulate_in_place(h, 8, g.data_ptr()) == B.ES_ESTATE            # already taken in place
        assert B.es_accumulate(h, 1, 0, g.data_ptr()) == B.ES_ESTATE                  # already counted
        assert B.es_accumulate_batch(h, 9, [0, 1], [g.data_ptr(), g.data_ptr() + 128]) == B.ES_OK
        assert B.es_accumulate(h, 0, 0, g.data_ptr()) == B.ES_OK
        assert B.es_ring_order_reduce(h, g.data_ptr()) == B.ES_EINVAL                 # output overlaps an in-place gradient
        assert B.es_ring_order_reduce(h, job.avg.data_ptr()) == B.ES_OK
        assert B.es_accumulate_in_place(h, 0, g.data_ptr()) == B.ES_OK                # new step, table reset
        assert B.es_sync(h) == B.ES_OK
    finally:
        job.close()


def test_handle_lifecycle_and_two_jobs_side_by_side():
    """Create/destroy cycles give the memory back; two handles do not disturb each other."""
    free0 = torch.cuda.mem_get_info()[0]
    for _ in range(20):
        job = ESTJob(8, 1 << 20, [(0, 1 << 19), (1 << 19, 1 << 19)], 4, [16, 4096])
        job.set_grouping([0, 0, 1, 1, 2, 2, 3, 3], [0, 1, 0, 1, 0, 1, 0, 1])
        job.close()
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] >= free0 - (64 << 20)

    rng = np.random.default_rng(12)
    a = rng.standard_normal((3, 5000)).astype(np.float32)
    b = rng.standard_normal((5, 7001)).astype(np.float32)
    ja, jb = ESTJob(3, 5000, [(0, 5000)], 4), ESTJob(5, 7001, [(0, 7001)], 1)
    try:
        sa, sb = torch.from_numpy(a).to(G.DEV), torch.from_numpy(b).to(G.DEV)
        for e in range(5):                               # interleaved calls on the two handles
            if e < 3:
                ja.accumulate(e, 0, sa[e])
            jb.accumulate(e, 0, sb[e])
        jb.ring_order_reduce(); ja.ring_order_reduce()
        ja.sync(); jb.sync()
        assert np.array_equal(bits(ja.avg.cpu().numpy()), bits(oracle.ring_order_reduce(a, A=4)))
        assert np.array_equal(bits(jb.avg.cpu().numpy()), bits(oracle.ring_order_reduce(b, A=1)))
    finally:
        ja.close(); jb.close()


@pytest.mark.parametrize("N,lens", [(257, [100, 3000, 0, 257]), (1024, [5000, 17]), (4096, [4096 * 4 + 3]),
                                    (65535, [4099])])                       # the largest rank count es_init accepts
def test_many_logical_workers(N, lens):
    """More ranks than elements per chunk, most chunks empty, long add chains."""
    lay = buckets.custom(lens)
    rng = np.random.default_rng(N)
    g = (rng.standard_normal((N, lay.n_params)) * np.exp2(rng.integers(-8, 8, (N, lay.n_params)))).astype(np.float32)
    # the ring simulator walks N^2 messages: beyond a few thousand ranks the closed form of the same
    # fold stands in (tests/test_oracle_ring.py holds the two equal)
    reduce_bucket = oracle.ring_order_reduce if N <= 4096 else fold_def.fold_reduce_gather
    want = np.concatenate([reduce_bucket(np.ascontiguousarray(g[:, o:o + l]), A=1)
                           for o, l in lay.buckets if l] or [np.zeros(0, np.float32)])
    job = ESTJob(N, lay.n_params, lay.buckets, 1)
    try:
        src = torch.from_numpy(g).to(G.DEV)
        allb = list(range(lay.n_buckets))
        for e in range(N):
            job.accumulate_batch(e, allb, [src[e, o:o + l] for o, l in lay.buckets])
        job.ring_order_reduce(); job.sync()
        assert np.array_equal(bits(job.avg.cpu().numpy()), bits(want))
    finally:
        job.close()


def test_degenerate_layouts():
    """No parameters at all, and only empty buckets: every call is a valid no-op."""
    for bk in ([], [(0, 0)], [(0, 0), (0, 0)]):
        st, h = B.es_init(3, 0, bk, 4, [])
        assert st == B.ES_OK and h
        try:
            for e in range(3):
                for b in range(len(bk)):
                    assert B.es_accumulate(h, e, b, 0) == B.ES_OK
            assert B.es_ring_order_reduce(h, 0) == B.ES_OK
            assert B.es_reduce_sgd_step(h, 0, 0, 0, 0.1, 0.9) in (B.ES_OK, B.ES_ESTATE)
            assert B.es_sgd_step(h, 0, 0, 0, 0.1, 0.9) == B.ES_OK
            assert B.es_ctx_save(h, 1) == B.ES_OK and B.es_ctx_switch(h, 0, 1) == B.ES_OK
            assert B.es_sync(h) == B.ES_OK
            n = B.es_checkpoint_bytes(h)
            blob = np.zeros(n, dtype=np.uint8)
            assert B.es_checkpoint_export(h, blob.ctypes.data, n, 0, 0, 3) == B.ES_OK
            assert B.es_checkpoint_import(h, blob.ctypes.data, n, 0, 0) == (B.ES_OK, 3)
        finally:
            B.es_destroy(h)


def test_spilling_some_arenas_to_host_keeps_the_bits():
    """HBM budget for gradient slots: workers that no longer fit get host-resident arenas."""
    N = 6
    sc = S.Scenario(N, buckets.custom([300000, 0, 7, 100001], fan_in=5), 4, 93, steps=2)
    ref = S.run_ddp_reference(sc)
    g = configs.contiguous([2, 2, 2])
    job = G.make_job(sc, configs.contiguous([N]))
    try:
        per_worker_mib = 2 * sc.layout.n_params * 4 / 2 ** 20
        job.set_option("hbm_slot_budget_mib", int(per_worker_mib * 2) + 1)      # room for two of three arenas
        job.set_grouping(g.worker_of_est, g.slot_of_est)
        assert B.es_get_option(job.h, "slots_on_host") == (0, 2)
        G.init_contexts(sc, job)
        G.run_steps(sc, job, g, fused=True)
        for name, got, want in (("avg", job.avg, ref.avg), ("p", job.p, ref.p), ("v", job.v, ref.v)):
            assert np.array_equal(bits(got.cpu().numpy()), bits(want)), name
        job.set_option("hbm_slot_budget_mib", -1)
        job.set_grouping(g.worker_of_est, g.slot_of_est)
        assert B.es_get_option(job.h, "slots_on_host") == (0, 0)
        assert B.es_set_option(job.h, "hbm_slot_budget_mib", -2) == B.ES_EINVAL
    finally:
        job.close()


def test_grouping_from_a_scheduler_plan():
    """Paper section 3.4 feeding section 3.2: the best plan for three GPU types becomes the
    EST-to-worker grouping of the step; the bits stay those of 9-worker data parallelism."""
    st, plans = B.es_sched_enumerate([8.0, 4.0, 2.0], [1, 1, 2], 9, top_k=1)
    assert st == B.ES_OK and len(plans) == 1
    st, nw, wo, so = B.es_sched_grouping(plans[0]["n_used"], plans[0]["est_per_gpu"], 9)
    assert st == B.ES_OK and nw == plans[0]["n_gpus"] >= 2
    g = configs.Grouping("plan", tuple(wo), tuple(so))
    sc = ragged_scenario(9, 1, 91, steps=2, mask_n=77, bn_channels=(4, 9))
    ref = S.run_ddp_reference(sc)
    S.assert_same(G.run_gpu(sc, g, fused=True, use_switch=True), ref, "grouping of the best plan")


def test_random_layouts_groupings_and_launch_shapes():
    """Seeded sweep: bucket lengths around tile, chunk and vector boundaries, any N and chunk
    alignment, random EST-to-worker groupings and launch shapes; every case bit-exact."""
    rng = np.random.default_rng(20240607)
    for case in range(36):
        N = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 9, 12, 16, 17, 24, 32, 40]))
        A = int(rng.choice([1, 1, 2, 4, 4, 8, 64]))
        tile = int(rng.choice([256, 512, 2048, 2048, 8192]))
        lens = []
        for _ in range(int(rng.integers(1, 6))):
            kind = int(rng.integers(0, 6))
            if kind == 0:
                lens.append(int(rng.integers(0, 4)))
            elif kind == 1:
                lens.append(int(rng.integers(1, 3 * N + 6)))
            elif kind == 2:                                   # around a multiple of tile * N
                lens.append(max(0, tile * N * int(rng.integers(1, 3)) + int(rng.integers(-5, 6))))
            elif kind == 3:                                   # around a multiple of the tile
                lens.append(max(0, tile * int(rng.integers(1, 9)) + int(rng.integers(-5, 6))))
            elif kind == 4:                                   # long enough for big tiles when N is small
                lens.append(N * 8192 * int(rng.integers(1, 3)) + int(rng.integers(0, 4099)))
            else:
                lens.append(int(rng.integers(1, 60000)))
        # a random grouping: worker sizes, then one of the three placements
        sizes, left = [], N
        while left:
            k = int(rng.integers(1, left + 1))
            sizes.append(k)
            left -= k
        g = (configs.contiguous, configs.round_robin,
             lambda s: configs.reversed_slots(configs.contiguous(s)))[int(rng.integers(0, 3))](sizes)
        options = {"reduce_tile_elems": tile, "reduce_unroll": int(rng.choice([1, 2, 4])),
                   "reduce_rank_batch": int(rng.choice([1, 2, 4, 8, 16])),
                   "nontemporal": int(rng.integers(0, 2)), "nontemporal_pv": int(rng.integers(0, 2)),
                   "reduce_big_unroll": int(rng.choice([0, 0, 8, 16, 32]))}
        fused, switch = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        streams = [True, "two", "one", False][int(rng.integers(0, 4))]
        batched, shift = bool(rng.integers(0, 2)), int(rng.integers(0, 4))
        what = (f"case {case}: N={N} A={A} lens={lens} grouping={g.name} {options} fused={fused} "
                f"streams={streams} batched={batched} src_shift={shift}")
        print("[gpu-case]", what, flush=True)
        sc = S.Scenario(N, buckets.custom(lens, fan_in=5), A, 9000 + case, steps=2,
                        mask_n=int(rng.integers(0, 300)), bn_channels=(3, int(rng.integers(1, 70))))
        ref = S.run_ddp_reference(sc)
        S.assert_same(G.run_gpu(sc, g, fused=fused, use_switch=switch, use_streams=streams, options=options,
                                batched=batched, src_shift=shift), ref, what)


def test_staging_from_sources_off_a_16_byte_boundary():
    """Buckets at odd offsets, flat sources shifted by 0-3 elements: the vector copy with
    leading and trailing single elements (source and slot equally far off a boundary) and the
    element-wise copy (off by different amounts), batched and per bucket, give the same bits."""
    N = 3
    lay = buckets.custom([4097, 3, 8190, 1, 2, 70001, 5], fan_in=2)      # offsets 1, 0, 2, 3, 1, 2 (mod 4)
    sc = S.Scenario(N, lay, 1, 404, steps=1)
    ref = S.run_ddp_reference(sc)
    g = configs.contiguous([N])
    for shift in range(4):
        S.assert_same(G.run_gpu(sc, g, fused=True, batched=True, src_shift=shift, use_streams="one"),
                      ref, f"batched shift {shift}")
    # per bucket through es_accumulate, sources cut out of one shifted flat vector
    job = G.make_job(sc, g, use_streams="one")
    try:
        for shift in range(4):
            keep = []
            for e in range(N):
                flat = torch.empty(lay.n_params + 4, device=G.DEV)[shift:shift + lay.n_params]
                for b, (off, ln) in enumerate(lay.buckets):
                    with job.stream_ctx():
                        synth.gradient(lay, b, sc.seed, 0, e, G.DEV, out=flat[off:off + ln])
                    job.accumulate(e, b, flat[off:off + ln])
                keep.append(flat)
            job.ring_order_reduce()
            job.sync(); torch.cuda.synchronize()
            assert np.array_equal(bits(job.avg.cpu().numpy()), bits(ref.avg)), f"per bucket shift {shift}"
    finally:
        job.close()


def test_est_boundary_in_one_launch_matches_the_separate_calls():
    """es_est_boundary = staging of the outgoing EST + save + restore of the next EST of its worker in
    one kernel launch on one stream; with a stage stream of its own (two or three streams) the copy goes
    there and the switch to the ctx stream.  Same bits as the reference for every grouping."""
    N = 8
    sc = ragged_scenario(N, 4, 91, steps=3, mask_n=517, bn_channels=(64, 3, 128, 2048))
    ref = S.run_ddp_reference(sc)
    for g in (configs.contiguous([8]), configs.contiguous([3, 5]), configs.round_robin([2, 6]),
              configs.contiguous([1] * 8, "1x8")):
        for streams in ("one", "two", True):
            got = G.run_gpu(sc, g, fused=True, boundary=True, use_streams=streams)
            S.assert_same(got, ref, f"boundary {g.name} streams={streams}")
    # a layout without small state: the boundary is the staging copy alone
    sc2 = ragged_scenario(5, 1, 92, steps=2)
    S.assert_same(G.run_gpu(sc2, configs.contiguous([2, 3]), boundary=True), S.run_ddp_reference(sc2),
                  "boundary without state")


def test_est_boundary_state_rules():
    job = ESTJob(4, 64, [(0, 32), (32, 32)], 4, [16, 64], [0, 0, 1, 1], [0, 1, 0, 1])
    h = job.h
    try:
        g = torch.zeros(64, device=G.DEV)
        ptrs = [g.data_ptr(), g.data_ptr() + 128]
        assert B.es_est_boundary(h, 0, 0, [0, 1], ptrs) == B.ES_EINVAL            # switch to itself
        assert B.es_est_boundary(h, 0, 2, [0, 1], ptrs) == B.ES_EINVAL            # other worker
        assert B.es_est_boundary(h, 4, None, [0, 1], ptrs) == B.ES_EINVAL
        assert B.es_est_boundary(h, 0, 7, [0, 1], ptrs) == B.ES_EINVAL
        assert B.es_est_boundary(h, 0, 1, [0, 0], ptrs) == B.ES_ESTATE            # duplicate bucket
        assert B.es_est_boundary(h, 0, 1, [0, 5], ptrs) == B.ES_EINVAL
        assert B.es_est_boundary(h, 0, 1, [0, 1], ptrs) == B.ES_OK
        assert B.es_est_boundary(h, 0, 1, [0], ptrs[:1]) == B.ES_ESTATE           # already staged
        assert B.es_est_boundary(h, 1, None, [0, 1], ptrs) == B.ES_OK
        assert B.es_est_boundary(h, 2, 3, [], []) == B.ES_OK                      # context only
        assert B.es_sync(h) == B.ES_OK
    finally:
        job.close()
    # live state not bound: refused
    st, h2 = B.es_init(2, 64, [(0, 64)], 4, [16])
    assert st == B.ES_OK
    try:
        g = torch.zeros(64, device=G.DEV)
        assert B.es_est_boundary(h2, 0, 1, [0], [g.data_ptr()]) == B.ES_ESTATE
    finally:
        B.es_destroy(h2)


def test_accumulate_many_matches_per_est_staging():
    """Several ESTs' flat gradients staged by one launch (more ESTs than one launch carries, sources
    off a 16-byte boundary, one EST produced in its slot), against the reference."""
    N = 20
    sc = ragged_scenario(N, 4, 93, steps=2, bn_channels=(5, 16))
    ref = S.run_ddp_reference(sc)
    for g, many, shift in ((configs.contiguous([20]), 20, 0), (configs.contiguous([7, 13]), 3, 1),
                           (configs.contiguous([1] * 20, "1x20"), 17, 2)):
        got = G.run_gpu(sc, g, fused=True, many=many, src_shift=shift)
        S.assert_same(got, ref, f"many={many} {g.name}")


def test_accumulate_many_state_rules():
    job = ESTJob(3, 64, [(0, 32), (32, 32)], 4)
    h = job.h
    try:
        g = [torch.full((64,), float(k + 1), device=G.DEV) for k in range(3)]
        p = [t.data_ptr() for t in g]
        torch.cuda.synchronize()
        assert B.es_accumulate_many(h, [0, 0], [p[0], p[1]]) == B.ES_ESTATE       # duplicate EST
        assert B.es_accumulate_many(h, [0, 3], [p[0], p[1]]) == B.ES_EINVAL
        assert B.es_accumulate_many(h, [0, 1], [p[0], 0]) == B.ES_EINVAL          # null source
        assert B.es_accumulate_many(h, [0, 1], [p[0], p[1] + 2]) == B.ES_EINVAL   # not 4-byte aligned
        assert B.es_accumulate(h, 2, 1, p[2] + 128) == B.ES_OK
        assert B.es_accumulate_many(h, [1, 2], [p[1], p[2]]) == B.ES_ESTATE       # EST 2 partly present
        # EST 1 writes its gradient straight into its slot: only marked
        slot1 = B.es_grad_slot(h, 1, 0)
        torch.cuda.synchronize()
        assert B.es_accumulate_many(h, [0], [p[0]]) == B.ES_OK
        assert B.es_accumulate(h, 2, 0, p[2]) == B.ES_OK
        assert B.es_accumulate_many(h, [1], [slot1]) == B.ES_OK
        assert B.es_accumulate_many(h, [], []) == B.ES_OK
        assert B.es_ring_order_reduce(h, job.avg.data_ptr()) == B.ES_OK
        assert B.es_sync(h) == B.ES_OK
    finally:
        job.close()


def test_every_est_taken_in_place():
    """No staging at all: the reduce reads all N gradient vectors where the caller left them
    (more ESTs than one table-patch launch carries), two steps, small and big tiles."""
    for N, opts in ((5, None), (40, {"reduce_big_unroll": 8})):
        sc = ragged_scenario(N, 4, 300 + N, steps=2)
        ref = S.run_ddp_reference(sc)
        job = G.make_job(sc, configs.contiguous([N]), options=opts)
        try:
            G.init_contexts(sc, job)
            for t in range(sc.steps):
                flats = []
                with job.stream_ctx():
                    for e in range(N):
                        flat = torch.empty(sc.layout.n_params, dtype=torch.float32, device=G.DEV)
                        for b, (off, ln) in enumerate(sc.layout.buckets):
                            synth.gradient(sc.layout, b, sc.seed, t, e, G.DEV, out=flat[off:off + ln])
                        flats.append(flat)
                for e in range(N):
                    job.accumulate_in_place(e, flats[e])
                job.reduce_sgd_step(sc.lr, sc.momentum, store_avg=True)
                job.sync()
                torch.cuda.synchronize()
            S.assert_same(G.collect(sc, job, {}), ref, f"all {N} in place")
        finally:
            job.close()


def test_swap_in_of_host_resident_gradient_slots():
    """The paper's placement of EST gradients (section 3.2) with the swap-in reduce: device-to-host
    staging by asynchronous copies, buckets streamed back through two HBM buffers while the previous
    bucket is reduced.  All slots on the host, some on the host, in-place ESTs, every way of staging,
    odd bucket offsets, big tiles, a regrouping between steps: always the reference's bits."""
    N = 6
    lay = buckets.custom([3 * 4096 + 37, 0, 3, 4096, 1001, 4 * N + 1, 20000 + N, 40000, 5], fan_in=9)
    sc = S.Scenario(N, lay, 1, 0x5A1, steps=3, mask_n=64, bn_channels=(8, 3))
    ref = S.run_ddp_reference(sc)
    g = configs.contiguous([2, 4])
    for flow in ("per_bucket", "boundary", "many", "big_tiles"):
        job = G.make_job(sc, configs.contiguous([N]),
                         options={"reduce_big_unroll": 8} if flow == "big_tiles" else None)
        try:
            job.set_option("host_slots", 1)
            job.set_option("swap_in", 1)
            job.set_grouping(g.worker_of_est, g.slot_of_est)
            assert B.es_get_option(job.h, "slots_on_host") == (0, N)
            G.init_contexts(sc, job)
            masks = {}
            G.run_steps(sc, job, g, fused=(flow != "per_bucket"), masks=masks, boundary=(flow == "boundary"),
                        many=(4 if flow == "many" else 0))
            S.assert_same(G.collect(sc, job, masks), ref, f"swap-in {flow}")
        finally:
            job.close()
    # some arenas in HBM, some on the host; regrouped (and the option switched) between steps
    sc2 = S.Scenario(N, lay, 4, 0x5A2, steps=3)
    ref2 = S.run_ddp_reference(sc2)
    g3 = configs.contiguous([2, 2, 2])
    job = G.make_job(sc2, configs.contiguous([N]))
    try:
        per_worker_mib = 2 * lay.n_params * 4 / 2 ** 20
        job.set_option("hbm_slot_budget_mib", int(per_worker_mib) + 1)      # one arena of three fits
        job.set_option("swap_in", 1)
        job.set_grouping(g3.worker_of_est, g3.slot_of_est)
        assert B.es_get_option(job.h, "slots_on_host") == (0, 4)
        G.init_contexts(sc2, job)
        G.run_steps(sc2, job, g3, fused=True, steps=[0])
        assert B.es_set_option(job.h, "swap_in", 0) == B.ES_OK             # direct access over the link
        G.run_steps(sc2, job, g3, fused=False, steps=[1])
        job.set_option("swap_in", 1)
        job.set_grouping(g.worker_of_est, g.slot_of_est)                    # tables follow the new slots
        G.run_steps(sc2, job, g, fused=True, steps=[2])
        S.assert_same(G.collect(sc2, job, {}), ref2, "mixed placement")
    finally:
        job.close()
    # in-place ESTs under swap-in, and the option refused while gradients are staged
    sc3 = S.Scenario(4, lay, 4, 0x5A3, steps=2)
    ref3 = S.run_ddp_reference(sc3)
    job = G.make_job(sc3, configs.contiguous([4]))
    try:
        job.set_option("host_slots", 1)
        job.set_option("swap_in", 1)
        job.set_grouping([0, 0, 1, 1], [0, 1, 0, 1])
        G.init_contexts(sc3, job)
        for t in range(sc3.steps):
            flats = []
            with job.stream_ctx():
                for e in range(4):
                    flat = torch.empty(lay.n_params, dtype=torch.float32, device=G.DEV)
                    for b, (off, ln) in enumerate(lay.buckets):
                        synth.gradient(lay, b, sc3.seed, t, e, G.DEV, out=flat[off:off + ln])
                    flats.append(flat)
            for e in range(4):
                if e % 2:
                    job.accumulate_in_place(e, flats[e])
                else:
                    job.accumulate_batch(e, list(range(lay.n_buckets)), [flats[e][o:o + l] for o, l in lay.buckets])
            assert B.es_set_option(job.h, "swap_in", 0) == B.ES_ESTATE
            job.reduce_sgd_step(sc3.lr, sc3.momentum, store_avg=True)
            job.sync()
            torch.cuda.synchronize()
        S.assert_same(G.collect(sc3, job, {}), ref3, "in place under swap-in")
    finally:
        job.close()


def test_random_flows_placements_and_occupancy_caps():
    """Second seeded sweep, over the ways gradients reach the reduce: one launch per EST boundary,
    several ESTs per staging launch, per-bucket calls; slots in HBM, in host memory read over the
    link, or swapped in through the two buffers, or mixed by an HBM budget; any occupancy cap."""
    rng = np.random.default_rng(20241127)
    for case in range(24):
        N = int(rng.choice([1, 2, 3, 5, 8, 11, 16, 20, 33]))
        A = int(rng.choice([1, 4, 4, 32]))
        lens = []
        for _ in range(int(rng.integers(1, 7))):
            kind = int(rng.integers(0, 4))
            lens.append([int(rng.integers(0, 5)), int(rng.integers(1, 3 * N + 6)),
                         2048 * N + int(rng.integers(-5, 6)), int(rng.integers(1, 90000))][kind])
        sizes, left = [], N
        while left:
            k = int(rng.integers(1, left + 1))
            sizes.append(k)
            left -= k
        g = (configs.contiguous, configs.round_robin)[int(rng.integers(0, 2))](sizes)
        flow = ["boundary", "many", "per_bucket", "batched"][int(rng.integers(0, 4))]
        placement = ["hbm", "host_direct", "host_swap", "mixed_swap"][int(rng.integers(0, 4))]
        options = {"reduce_lds_pad_kib": int(rng.choice([-1, 0, 24, 64, 160])),
                   "reduce_big_unroll": int(rng.choice([0, 8, 32])),
                   "reduce_rank_batch": int(rng.choice([1, 4, 8]))}
        fused = bool(rng.integers(0, 2))
        streams = [True, "one", "two"][int(rng.integers(0, 3))]
        sc = S.Scenario(N, buckets.custom(lens, fan_in=3), A, 7000 + case, steps=2,
                        mask_n=int(rng.integers(0, 200)), bn_channels=(int(rng.integers(1, 40)),))
        what = (f"case {case}: N={N} A={A} lens={lens} grouping={g.name} flow={flow} placement={placement} "
                f"{options} fused={fused} streams={streams}")
        print("[gpu-case]", what, flush=True)
        ref = S.run_ddp_reference(sc)
        job = G.make_job(sc, configs.contiguous([N]), use_streams=streams, options=options)
        try:
            if placement != "hbm":
                if placement == "mixed_swap":
                    job.set_option("hbm_slot_budget_mib", 0 if len(sizes) == 1 else 1)
                else:
                    job.set_option("host_slots", 1)
                job.set_option("swap_in", 0 if placement == "host_direct" else 1)
            job.set_grouping(g.worker_of_est, g.slot_of_est)
            G.init_contexts(sc, job)
            masks = {}
            G.run_steps(sc, job, g, fused=fused, masks=masks, boundary=(flow == "boundary"),
                        many=(int(rng.integers(1, N + 1)) if flow == "many" else 0), batched=(flow == "batched"))
            S.assert_same(G.collect(sc, job, masks), ref, what)
        finally:
            job.close()


def test_large_and_odd_state_segments_through_every_context_path():
    """Context traffic as plain bytes: segments of 3 MiB + 5, 7, 16 and 12 KiB + 4 bytes, live tensors
    16-byte aligned, 4-byte aligned and at odd addresses; save, restore, the fused switch and the
    one-launch EST boundary all have to move exactly the segment's bytes."""
    segs = [(3 << 20) + 5, 7, 16, 12 * 1024 + 4]
    rng = np.random.default_rng(31)
    for shift in (0, 4, 1):
        def alloc(nb, shift=shift):
            base = torch.full((nb + 64,), 0xEE, dtype=torch.uint8, device=G.DEV)
            return base[shift:shift + nb]
        job = ESTJob(3, 64, [(0, 64)], 4, segs, [0, 0, 0], [2, 0, 1], live_alloc=alloc)
        try:
            pat = [[torch.from_numpy(rng.integers(0, 256, nb, dtype=np.uint8)).to(G.DEV) for nb in segs]
                   for _ in range(3)]
            live = job.live_of(0)

            def put(e):
                for t, src in zip(live, pat[e]):
                    t.copy_(src)
                torch.cuda.synchronize()

            def check(e, what):
                job.sync(); torch.cuda.synchronize()
                for j, (t, src) in enumerate(zip(live, pat[e])):
                    assert torch.equal(t, src), (what, shift, e, j)

            print(f"[gpu-case] large odd state segments, live shift {shift}", flush=True)
            put(0); job.ctx_save(0); job.sync()
            put(1); job.ctx_save(1); job.sync()
            job.ctx_restore(0); check(0, "restore")
            put(2)                                  # EST 2's state is live, 0 and 1 are in their slots
            job.ctx_switch(2, 1); check(1, "switch in")
            job.ctx_restore(2); check(2, "switch saved the outgoing EST")
            grad = torch.zeros(64, device=G.DEV)
            B.check(B.es_est_boundary(job.h, 2, 0, [0], [grad.data_ptr()]), "es_est_boundary", job.h)
            check(0, "boundary in")
            put(1)                                  # overwrite live, then bring EST 2 back from its slot
            job.ctx_restore(2); check(2, "boundary saved the outgoing EST")
            # the guard bytes around every live tensor are untouched
            job.sync(); torch.cuda.synchronize()
            for t in live:
                assert t.untyped_storage().nbytes() >= t.numel() + 64
                raw = torch.empty(0, dtype=torch.uint8, device=G.DEV).set_(t.untyped_storage())
                assert bool((raw[:shift] == 0xEE).all()) and bool((raw[shift + t.numel():] == 0xEE).all()), shift
        finally:
            job.close()
