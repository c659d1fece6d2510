"""On-demand checkpoint through the C boundary (paper sections 3.2, 3.3 D1): export between
global steps, a fresh handle with another grouping imports, training continues, and
the outcome equals the uninterrupted N-rank oracle run bit for bit."""
import numpy as np
import pytest
import torch

import scenario as S
from workloads import buckets, configs

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import gpu_harness as G
    from paper_2208_14228_amd import binding as B


def scenario(N=6, steps=4):
    lay = buckets.custom([3 * 4096 + 37, 0, 3, 1001, 4 * N + 1], fan_in=9)
    return S.Scenario(N, lay, 4, 0xC4EC, steps=steps, mask_n=517, bn_channels=(3, 64, 5))


def parse_blob(sc, blob):
    hdr = blob[:64].view(np.uint64)
    nb, ns = int(hdr[3]), int(hdr[5])
    off = 64
    bk = blob[off:off + 16 * nb].view(np.uint64).reshape(nb, 2); off += 16 * nb
    segs = blob[off:off + 8 * ns].view(np.uint64); off += 8 * ns
    ctx_bytes = int(hdr[6])
    ctx = blob[off:off + sc.n_logical * ctx_bytes].reshape(sc.n_logical, ctx_bytes); off += ctx.size
    P = int(hdr[2])
    p = blob[off:off + 4 * P].view(np.float32); off += 4 * P
    v = blob[off:off + 4 * P].view(np.float32); off += 4 * P
    assert off == blob.size
    return hdr, bk, segs, ctx, p, v


def test_checkpoint_resume_with_other_groupings():
    sc = scenario()
    ref = S.run_ddp_reference(sc)
    # the oracle's state after 2 of the 4 steps: what the blob must contain
    mid = S.run_ddp_reference(S.Scenario(sc.n_logical, sc.layout, sc.chunk_align, sc.seed, 2, sc.lr,
                                         sc.momentum, sc.mask_n, sc.p_drop, sc.bn_channels))
    g0, g1 = configs.contiguous([6]), configs.round_robin([1, 2, 3])
    masks = {}
    job = G.make_job(sc, g0)
    try:
        G.init_contexts(sc, job)
        G.run_steps(sc, job, g0, masks=masks, steps=[0, 1])
        blob = job.checkpoint_export(2)
    finally:
        job.close()

    hdr, bk, segs, ctx, p, v = parse_blob(sc, blob)
    assert hdr[0] == 0x3130544B50435345 and bytes(blob[:8]) == b"ESCPKT01"
    assert list(hdr[1:8]) == [6, sc.layout.n_params, sc.layout.n_buckets, 4, len(G.seg_bytes(sc)),
                              sum((b + 15) // 16 * 16 for b in G.seg_bytes(sc)), 2]
    assert [tuple(int(x) for x in r) for r in bk] == list(sc.layout.buckets)
    assert list(segs) == G.seg_bytes(sc)
    assert np.array_equal(p.view(np.uint32), mid.p.view(np.uint32))
    assert np.array_equal(v.view(np.uint32), mid.v.view(np.uint32))
    for e in range(sc.n_logical):                       # contexts by virtual rank, 16-byte padded segments
        assert np.array_equal(ctx[e, :16].view(np.uint64), mid.philox[e])
        off = 16
        for (o, ln) in sc.bn_segments:
            assert np.array_equal(ctx[e, off:off + 4 * ln].view(np.uint32),
                                  mid.bn[e, o:o + ln].view(np.uint32))
            off += (4 * ln + 15) // 16 * 16

    job = G.make_job(sc, g1, use_streams="two")          # fresh handle, other grouping
    try:
        assert job.checkpoint_import(blob) == 2
        G.run_steps(sc, job, g1, fused=True, use_switch=True, masks=masks, steps=[2, 3])
        S.assert_same(G.collect(sc, job, masks), ref, "resumed")
    finally:
        job.close()


def test_checkpoint_argument_and_state_checks():
    sc = scenario(N=2, steps=1)
    job = G.make_job(sc, configs.contiguous([2]))
    other = G.make_job(S.Scenario(2, buckets.custom([3 * 4096 + 37, 0, 3, 1001, 10], fan_in=9), 4, 1,
                                  mask_n=517, bn_channels=(3, 64, 5)), configs.contiguous([2]))
    try:
        G.init_contexts(sc, job)
        n = B.es_checkpoint_bytes(job.h)
        blob = np.zeros(n, dtype=np.uint8)
        pp, vv = job.p.data_ptr(), job.v.data_ptr()
        assert B.es_checkpoint_export(job.h, blob.ctypes.data, n - 1, pp, vv, 0) == B.ES_EINVAL
        assert B.es_checkpoint_export(job.h, 0, n, pp, vv, 0) == B.ES_EINVAL
        assert B.es_checkpoint_export(job.h, blob.ctypes.data, n, 0, vv, 0) == B.ES_EINVAL
        g = torch.zeros(sc.layout.buckets[0][1], device=G.DEV)
        assert B.es_accumulate(job.h, 0, 0, g.data_ptr()) == B.ES_OK
        assert B.es_checkpoint_export(job.h, blob.ctypes.data, n, pp, vv, 0) == B.ES_ESTATE   # mid-step
        for e in range(2):
            for b in range(sc.layout.n_buckets):
                if (e, b) != (0, 0):
                    gb = torch.zeros(sc.layout.buckets[b][1], device=G.DEV)
                    assert B.es_accumulate(job.h, e, b, gb.data_ptr()) == B.ES_OK
        job.ring_order_reduce(); job.sync()
        assert B.es_checkpoint_export(job.h, blob.ctypes.data, n, pp, vv, 7) == B.ES_OK
        assert B.es_checkpoint_import(job.h, blob.ctypes.data, n - 8, pp, vv)[0] == B.ES_EINVAL
        bad = blob.copy(); bad[0] ^= 1
        assert B.es_checkpoint_import(job.h, bad.ctypes.data, n, pp, vv)[0] == B.ES_EINVAL    # magic
        bad = blob.copy(); bad[64 + 8] ^= 1                                                    # bucket 0 length
        assert B.es_checkpoint_import(job.h, bad.ctypes.data, n, pp, vv)[0] == B.ES_EINVAL
        # a job with another bucket mapping refuses the blob (D1: the mapping is reinstated, not rebuilt)
        n2 = B.es_checkpoint_bytes(other.h)
        assert B.es_checkpoint_import(other.h, blob.ctypes.data, n, other.p.data_ptr(), other.v.data_ptr())[0] == B.ES_EINVAL
        assert n2 != n or True
        assert B.es_checkpoint_import(job.h, blob.ctypes.data, n, pp, vv) == (B.ES_OK, 7)
    finally:
        job.close(); other.close()
