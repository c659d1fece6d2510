"""The five benchmark configurations at full size, in the launch configuration bench.py times.

Every output element of every configuration is compared with the CPU oracle.
Configurations 1, 2 and 4 are small enough for the message-passing oracle to
replay the whole job on the host in one go.  Configurations 3 and 5 are
streamed: after every global step the N gradient rows of one bucket at a time
are generated again, copied into a pinned host buffer and run through the ring
simulator; the averaged gradient of that bucket is compared with the device's,
then the oracle's SGD-momentum update is applied to the host copy of that
bucket's parameters and momentum, which are compared in full after the last
step (3 steps for configuration 3, 2 for configuration 5, so momentum carried
over from an earlier step enters the update).  One bucket per step also goes
through the closed-form fold.  Every dropout mask and RNG state is replayed.
The other groupings, and the launch configuration bench.py times, must then
reproduce the first grouping's vectors bit for bit (compared on the device)."""
from typing import Dict, List, Tuple

import numpy as np
import pytest
import torch

import oracle
import scenario as S
from oracle import fold_def
from workloads import configs, synth

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import gpu_harness as G


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def dev_bits_equal(a: torch.Tensor, b: torch.Tensor) -> bool:
    return bool(torch.equal(a.view(torch.int32), b.view(torch.int32)))


@pytest.mark.parametrize("cid", [1, 2, 4])
def test_full_replay(cid):
    cfg = configs.config(cid)
    sc = S.from_config(cfg, steps=2 if cid == 4 else 3)
    ref = S.run_ddp_reference(sc, gen_device=G.DEV)
    for gi, g in enumerate(cfg.groupings):
        got = G.run_gpu(sc, g, fused=bool(gi % 2), use_switch=bool(gi % 2))
        S.assert_same(got, ref, f"config {cid} grouping {g.name}")
    bench_launch_configuration(sc, cfg.groupings[0], ref.p, ref.v)


def bench_launch_configuration(sc, g, want_p, want_v):
    """Exactly what bench.py times: one in-order stream, one flat gradient vector per EST, every EST
    boundary one es_est_boundary launch (stage + save + restore of the next EST), fused reduce+update
    without storing the average."""
    job = G.make_job(sc, g, use_streams="one")
    try:
        G.init_contexts(sc, job)
        G.run_steps(sc, job, g, fused=True, boundary=True, store_avg=False,
                    sync_each_est=sc.layout.n_params * sc.n_logical > (1 << 31))
        if isinstance(want_p, np.ndarray):
            assert np.array_equal(bits(job.p.cpu().numpy()), bits(want_p)), "bench configuration: parameters"
            assert np.array_equal(bits(job.v.cpu().numpy()), bits(want_v)), "bench configuration: momentum"
        else:                                   # device tensors of another run of the same job
            assert dev_bits_equal(job.p, want_p) and dev_bits_equal(job.v, want_v), "bench configuration"
    finally:
        job.close()


def streamed_oracle_step(sc, job, t, pin, host_p, host_v, what):
    """Global step t of the whole job on the host, one bucket at a time, against the device's
    averaged gradient; updates host_p / host_v with the oracle's SGD-momentum."""
    N = sc.n_logical
    for b, (off, L) in enumerate(sc.layout.buckets):
        if L == 0:
            continue
        rows = pin[:N * L].view(N, L)
        for r in range(N):             # seeded inputs, evaluated by torch on the device
            rows[r].copy_(S.grad(sc, t, r, b, G.DEV), non_blocking=True)
        torch.cuda.synchronize()
        ranks = rows.numpy()
        closed_form = fold_def.fold_reduce(ranks, sc.chunk_align) if b == t % sc.layout.n_buckets else None
        want = oracle.ring_order_reduce(ranks, sc.chunk_align, clobber=True)
        if closed_form is not None:
            assert np.array_equal(bits(closed_form), bits(want)), (what, "simulator vs closed form", t, b)
        got = job.avg[off:off + L].cpu().numpy()
        assert np.array_equal(bits(got), bits(want)), (what, "averaged gradient", "step", t, "bucket", b)
        oracle.sgd_momentum(host_p[off:off + L], host_v[off:off + L], want, sc.lr, sc.momentum)
    print(f"[oracle] {what}: step {t} checked on all {sc.layout.n_buckets} buckets", flush=True)


def run_streamed(cid: int, steps: int):
    cfg = configs.config(cid)
    sc = S.from_config(cfg, steps=steps)
    N = sc.n_logical
    pin = torch.empty(N * max(L for _, L in sc.layout.buckets), dtype=torch.float32, pin_memory=True)
    # the per-rank state (RNG states, masks) is cheap to replay in full on the host
    want_masks, want_philox = {}, None
    if sc.mask_n:
        want_philox = np.array([[S.philox_seed(sc, e), 0] for e in range(N)], dtype=np.uint64)
        for t in range(steps):
            for e in range(N):
                want_masks[(t, e)] = S.digest(oracle.dropout_mask(want_philox[e], sc.mask_n, sc.p_drop))
    keep = None
    for gi, g in enumerate(cfg.groupings):
        what = f"config {cid} grouping {g.name}"
        print(f"[gpu-run] {what} steps={steps}", flush=True)
        job = G.make_job(sc, g)
        try:
            G.init_contexts(sc, job)
            masks = {}
            if gi == 0:
                host_p = synth.params(sc.layout, sc.seed, G.DEV).cpu().numpy()
                host_v = np.zeros_like(host_p)
                for t in range(steps):          # unfused here, so that every step's average is stored
                    G.run_steps(sc, job, g, fused=False, use_switch=False, sync_each_est=True,
                                masks=masks, steps=[t])
                    streamed_oracle_step(sc, job, t, pin, host_p, host_v, what)
                assert np.array_equal(bits(job.p.cpu().numpy()), bits(host_p)), (what, "parameters")
                assert np.array_equal(bits(job.v.cpu().numpy()), bits(host_v)), (what, "momentum")
                del host_p, host_v
            else:
                G.run_steps(sc, job, g, fused=bool(gi % 2), use_switch=bool(gi % 2),
                            sync_each_est=True, masks=masks)
            if sc.mask_n:
                assert masks == want_masks, what
                got = G.collect(sc, job, masks)
                assert np.array_equal(got.philox, want_philox), what
            cur = (job.avg.clone(), job.p.clone(), job.v.clone())
            if keep is None:
                keep = cur
            else:                       # the other groupings reproduce the vectors the oracle has checked
                for x, y, name in zip(keep, cur, ("avg", "p", "v")):
                    assert dev_bits_equal(x, y), (what, name)
        finally:
            job.close()
        torch.cuda.empty_cache()
    # ... and so does the launch configuration bench.py times
    bench_launch_configuration(sc, cfg.groupings[0], keep[1], keep[2])


def test_config3_bert_base_with_philox_context():
    # 16 ranks x 13 buckets (one of them the 93 MiB embedding), 3 global steps, all through the ring simulator
    run_streamed(3, steps=3)


def test_config5_gpt2_medium_uneven_groupings():
    # 64 ranks x 355M parameters: 90.8 GB of gradient slots on the device, 2 global steps
    run_streamed(5, steps=2)
