"""The paper's accuracy-consistency experiment (section 5.1.1) in miniature: a real autograd
training loop whose N logical workers are time-sliced on one GPU under different
EST-to-worker groupings must end with bitwise identical parameters, and equal to the run
in which every EST has a worker of its own (= ordinary N-worker data parallelism).

The model's forward/backward is PyTorch (that compute is not part of the library); all
state handling goes through libes: parameters and momentum live in the job's flat vectors,
BatchNorm running statistics and the dropout RNG state are EST context, masks come from
es_dropout_mask, gradients are staged per bucket, reduced in ring order and applied by the
fused update.  In every global step the averaged gradient is also checked against the CPU
oracle fed with the very gradients the ESTs produced.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from workloads import buckets as WB
from workloads import configs, synth

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from paper_2208_14228_amd.job import ESTJob
    DEV = "cuda:0"

D_IN, D_H, D_OUT, BATCH = 64, 128, 10, 32
# parameters in forward order; the flat space holds them in reverse (bucket) order
SHAPES = [("w1", (D_H, D_IN)), ("b1", (D_H,)), ("bn_w", (D_H,)), ("bn_b", (D_H,)),
          ("w2", (D_OUT, D_H)), ("b2", (D_OUT,))]
P_DROP = 0.1


def layout():
    sizes, off, place = [], 0, {}
    for name, shape in reversed(SHAPES):
        n = int(np.prod(shape))
        place[name] = (off, n, shape)
        off += n
    # three buckets: (b2, w2), (bn_b, bn_w, b1), (w1)
    cuts = [place["w2"][0] + place["w2"][1], place["b1"][0] + place["b1"][1], off]
    bk, start = [], 0
    for c in cuts:
        bk.append((start, c - start))
        start = c
    return off, bk, place


def bits(t):
    return t.detach().cpu().numpy().view(np.uint32)


def batch_for(seed, step, est):
    lay = WB.single_bucket(BATCH * D_IN)
    x = synth.values(lay, 0, BATCH * D_IN, seed, step, 5000 + est, 1.0, False, DEV).view(BATCH, D_IN)
    y = (synth.field_sums(0, BATCH, synth.stream_key(seed, step, 9000 + est), DEV) % D_OUT).long()
    return x, y


def run(grouping, steps=4, seed=0x7EA1):
    N = len(grouping.worker_of_est)
    P, bk, place = layout()
    seg_bytes = [16, 4 * D_H, 4 * D_H]                     # Philox state, BN running mean, running var
    job = ESTJob(N, P, bk, 4, seg_bytes, grouping.worker_of_est, grouping.slot_of_est, DEV, use_streams="two")
    try:
        with job.stream_ctx():
            job.p.copy_(synth.values(WB.single_bucket(P), 0, P, seed, 0, synth.STREAM_PARAM, 0.1, False, DEV))
            job.v.zero_()
        for e in range(N):                                 # initial contexts: own RNG stream, mean 0, var 1
            live = job.live_of(e)
            with job.stream_ctx():
                st = np.array([synth.stream_key(seed, 0, 100 + e), 0], dtype=np.uint64)
                live[0].copy_(torch.from_numpy(st.view(np.uint8)).to(DEV))
                live[1].view(torch.float32).zero_()
                live[2].view(torch.float32).fill_(1.0)
            job.ctx_save(e)
            job.sync()
        mask = torch.empty(BATCH * D_H, dtype=torch.uint8, device=DEV)
        for t in range(steps):
            grads = {}
            for e in grouping.schedule():
                job.ctx_restore(e)
                live = job.live_of(e)
                job.dropout_mask(e, 0, mask, P_DROP)
                with job.stream_ctx():
                    w = {n: job.p[o:o + k].view(shape).detach().clone().requires_grad_()
                         for n, (o, k, shape) in place.items()}
                    x, y = batch_for(seed, t, e)
                    h = F.linear(x, w["w1"], w["b1"])
                    mean, var = h.mean(0), h.var(0, unbiased=False)
                    rm, rv = live[1].view(torch.float32), live[2].view(torch.float32)
                    rm.mul_(0.9).add_(mean.detach() * 0.1)             # running statistics: EST context
                    rv.mul_(0.9).add_(var.detach() * 0.1)
                    h = (h - mean) / torch.sqrt(var + 1e-5) * w["bn_w"] + w["bn_b"]
                    h = torch.relu(h) * mask.view(BATCH, D_H).to(h.dtype) / (1.0 - P_DROP)
                    loss = F.cross_entropy(F.linear(h, w["w2"], w["b2"]), y)
                    loss.backward()
                    flat = torch.cat([w[n].grad.reshape(-1) for n, _ in reversed(SHAPES)]).contiguous()
                grads[e] = flat
                job.accumulate_batch(e, list(range(len(bk))), [flat[o:o + k] for o, k in bk])
                job.ctx_save(e)
            job.reduce_sgd_step(0.1, 0.9)
            job.sync(); torch.cuda.synchronize()
            # the library's average of exactly these gradients vs. the oracle's ring simulation
            host = np.stack([grads[e].cpu().numpy() for e in range(N)])
            want = np.concatenate([oracle.ring_order_reduce(np.ascontiguousarray(host[:, o:o + k]), A=4)
                                   for o, k in bk])
            assert np.array_equal(bits(job.avg), want.view(np.uint32)), (grouping.name, t)
        ctx = []
        for e in range(N):
            job.ctx_restore(e); job.sync(); torch.cuda.synchronize()
            ctx.append(torch.cat([x.clone() for x in job.live_of(e)]).cpu().numpy())
        return bits(job.p), bits(job.v), np.stack(ctx)
    finally:
        job.close()


def test_training_is_bitwise_identical_under_every_grouping():
    torch.use_deterministic_algorithms(True, warn_only=True)
    try:
        N = 6
        ddp = configs.contiguous([1] * N, "1x6")           # every EST on a worker of its own
        ref = run(ddp)
        again = run(ddp)
        if not all(np.array_equal(a, b) for a, b in zip(ref, again)):
            pytest.skip("the framework's own forward/backward is not run-to-run deterministic here")
        for g in (configs.contiguous([N]), configs.contiguous([2, 4]), configs.round_robin([1, 2, 3]),
                  configs.reversed_slots(configs.contiguous([3, 3]))):
            got = run(g)
            for name, a, b in zip(("parameters", "momentum", "EST contexts"), got, ref):
                assert np.array_equal(a, b), (g.name, name)
        # and training did something: parameters moved, every EST drew from its own RNG stream
        assert len({c[:16].tobytes() for c in ref[2]}) == N
    finally:
        torch.use_deterministic_algorithms(False)
