"""Host logic of the reduce's work decomposition, checked on the CPU against the
oracle's chunk geometry: tiles partition the parameter space, never cross a ring
chunk, carry the chunk index as start rank, and big tiles are full and aligned."""
import numpy as np
import pytest

import oracle
from paper_2208_14228_amd import binding as B
from workloads import buckets, configs, shapes


def check(N, lay, A, tile, big):
    st, n_big, tiles = B.es_plan_tiles(N, lay.n_params, lay.buckets, A, tile, big)
    assert st == 0
    covered = np.zeros(lay.n_params, dtype=np.int8) if lay.n_params < 5_000_000 else None
    total = 0
    bstart = [o for o, _ in lay.buckets]
    for k, (off, ln, r0) in enumerate(tiles):
        assert ln > 0 and r0 < N
        b = int(np.searchsorted(bstart, off, side="right")) - 1
        while lay.buckets[b][1] == 0 or off >= lay.buckets[b][0] + lay.buckets[b][1]:
            b += 1                                            # skip empty buckets at the same offset
        bo, L = lay.buckets[b]
        lo, hi = oracle.chunk_bounds(L, N, A, r0)             # the oracle's geometry for chunk r0
        assert bo + lo <= off and off + ln <= bo + hi, (k, off, ln, r0, b)
        if k < n_big:
            assert ln == 256 * big * 4 and off % 4 == 0
        else:
            assert ln <= tile
        total += ln
        if covered is not None:
            covered[off:off + ln] += 1
    assert total == lay.n_params
    if covered is not None:
        assert np.all(covered == 1)
    return n_big, len(tiles)


@pytest.mark.parametrize("N,A", [(1, 1), (3, 1), (4, 4), (7, 4), (16, 4), (64, 4)])
def test_ragged_layouts(N, A):
    lay = buckets.custom([3 * 4096 + 37, 0, 3, 4096, 1001, 4 * N + 1, 20000 + N, N * 40000 + 5])
    for tile, big in ((256, 0), (2048, 0), (4096, 8), (2048, 32)):
        check(N, lay, A, tile, big)


def test_benchmark_layouts():
    for cid in (1, 2, 3, 4, 5):
        cfg = configs.config(cid)
        big = 32 if cfg.n_logical >= 11 else 0
        n_big, n = check(cfg.n_logical, cfg.layout, cfg.chunk_align, 2048, big)
        if big:                                               # most of the work is in big tiles
            assert n_big * 32768 > 0.9 * cfg.layout.n_params
    # a worked example: ResNet-50 bucket 0 (7,564,264 elements) among 32 ranks, last chunk 236,360 long
    st, _, tiles = B.es_plan_tiles(32, 7564264, [(0, 7564264)], 4, 2048, 0)
    last = [t for t in tiles if t[2] == 31]
    assert sum(t[1] for t in last) == 236360 and last[0][0] == 31 * 236384


def test_rejects_bad_arguments():
    ok = dict(n_logical=2, n_params=8, buckets=[(0, 8)], chunk_align=1)
    assert B.es_plan_tiles(2, 8, [(0, 8)], 1, 100, 0)[0] == B.ES_EINVAL      # tile size
    assert B.es_plan_tiles(2, 8, [(0, 8)], 1, 2048, 5)[0] == B.ES_EINVAL     # big unroll
    assert B.es_plan_tiles(2, 8, [(0, 4)], 1, 2048, 0)[0] == B.ES_EINVAL     # layout does not cover
    assert B.es_plan_tiles(0, 8, [(0, 8)], 1, 2048, 0)[0] == B.ES_EINVAL
    assert B.es_plan_tiles(2, 8, [(0, 8)], 1, 2048, 0)[0] == B.ES_OK


def test_only_the_first_tile_of_a_chunk_may_start_unaligned():
    """Chunk boundaries inside a 128-byte line (alignment 1 or 2, odd lengths): the chunk opens
    with a tile that ends on a line boundary, every later tile starts on one, and big tiles are
    still used."""
    for N, A in ((3, 1), (7, 1), (16, 1), (5, 2), (6, 3)):
        lay = buckets.custom([N * 40000 + 5, 1001, 3, N * 300000 + 7, 2])
        bstart = [o for o, _ in lay.buckets]
        for tile, big in ((2048, 0), (2048, 32), (256, 8)):
            n_big, _ = check(N, lay, A, tile, big)
            st, _, tiles = B.es_plan_tiles(N, lay.n_params, lay.buckets, A, tile, big)
            first_of_chunk = {}
            for off, ln, r0 in tiles:
                b = int(np.searchsorted(bstart, off, side="right")) - 1
                first_of_chunk[(b, r0)] = min(first_of_chunk.get((b, r0), off), off)
            unaligned_chunks = 0
            for off, ln, r0 in tiles:
                b = int(np.searchsorted(bstart, off, side="right")) - 1
                if off != first_of_chunk[(b, r0)]:
                    assert off % 32 == 0, (N, A, tile, big, off, ln, r0)      # on a 128-byte line
                elif off % 4:
                    unaligned_chunks += 1
                    assert (off + ln) % 4 == 0 or ln < 4 or off + ln == lay.buckets[b][0] + oracle.chunk_bounds(
                        lay.buckets[b][1], N, A, r0)[1]
            assert unaligned_chunks > 0                       # the case is really exercised
            if big:
                assert n_big * 256 * big * 4 > 0.5 * lay.n_params


def test_swap_in_plan_is_the_oracle_models_schedule():
    """es_plan_swap_in (what the library enqueues for host-resident slots) against the oracle-side
    model: the same list, and executed by the model under random interleavings it gives the plain
    reduce."""
    import numpy as np

    import oracle
    from oracle.est_model import run_swap_in, swap_in_schedule
    for n in range(0, 12):
        st, plan = B.es_plan_swap_in(n)
        assert st == B.ES_OK and plan == swap_in_schedule(n), n
    rng = np.random.default_rng(8)
    lens = [37, 0, 4, 1000, 1, 513, 64, 9]
    rows = [rng.standard_normal((5, L)).astype(np.float32) for L in lens]
    _, plan = B.es_plan_swap_in(len(lens))
    for seed in range(10):
        got = run_swap_in(plan, lambda b: rows[b], lens, 5, 4, np.random.default_rng(seed))
        for b, L in enumerate(lens):
            want = oracle.ring_order_reduce(rows[b], 4)
            assert np.array_equal(got[b].view(np.uint32), want.view(np.uint32)), (seed, b)
    n = B.ctypes.c_uint64()
    assert B.lib().es_plan_swap_in(3, (B.EsSwapOp * 2)(), 2, B.ctypes.byref(n)) == B.ES_EINVAL   # capacity too small
