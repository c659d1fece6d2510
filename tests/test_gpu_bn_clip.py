"""BatchNorm batch statistics along the fixed tree and the clipped update on the GPU vs. the CPU
oracle, bit for bit, through the C boundary."""
import numpy as np
import pytest
import torch

import oracle
from test_oracle_tree import golden_witness, witness_inputs

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from paper_2208_14228_amd import binding as B
    from paper_2208_14228_amd.job import ESTJob
    DEV = "cuda:0"


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def gpu_bn(x: np.ndarray, shift=0, stream=None):
    Bn, C, HW = x.shape
    buf = torch.zeros(x.size + 8, device=DEV)
    xd = buf[shift:shift + x.size]
    xd.copy_(torch.from_numpy(x.reshape(-1)))
    mean = torch.full((max(C, 1),), float("nan"), device=DEV)
    var = torch.full((max(C, 1),), float("nan"), device=DEV)
    nws = B.es_bn_workspace_floats(Bn, C, HW)
    ws = torch.full((max(nws, 1),), float("nan"), device=DEV)
    torch.cuda.synchronize()
    print(f"[gpu-case] es_bn_batch_stats B={Bn} C={C} HW={HW} shift={shift}", flush=True)
    st = B.es_bn_batch_stats(xd.data_ptr(), Bn, C, HW, mean.data_ptr(), var.data_ptr(), ws.data_ptr(), nws,
                             stream.cuda_stream if stream is not None else 0)
    if st:
        return st
    torch.cuda.synchronize()
    return mean.cpu().numpy()[:C], var.cpu().numpy()[:C]


@pytest.mark.parametrize("Bn,C,HW", [(1, 1, 1), (2, 3, 49), (3, 2, 4097), (5, 4, 3136), (32, 7, 196),
                                     (7, 1, 150_001), (4, 64, 56 * 56), (2, 300, 13),
                                     (1, 65535, 5), (2, 1, (1 << 26) + 3)])    # most channels; a long channel
def test_bn_statistics_parity(Bn, C, HW):
    rng = np.random.default_rng(Bn * 1000 + HW)
    x = (rng.standard_normal((Bn, C, HW)) * 3 + rng.standard_normal((1, C, 1)) * 10).astype(np.float32)
    want_m, want_v = oracle.bn_batch_stats(x)
    for shift in (0, 1):                       # x 16-byte aligned and only 4-byte aligned
        got_m, got_v = gpu_bn(x, shift)
        assert np.array_equal(bits(got_m), bits(want_m)), ("mean", shift)
        assert np.array_equal(bits(got_v), bits(want_v)), ("var", shift)


def test_bn_witnesses_and_arguments():
    gold = golden_witness()
    a = witness_inputs()["A"]
    y = np.where(a == 4096, np.float32(2.0 ** 24), a).astype(np.float32)
    want = np.float32(gold["A"][1]) / np.float32(4096)
    for Bn in (1, 2, 4):
        got_m, _ = gpu_bn(y.reshape(Bn, 1, 4096 // Bn))
        assert bits(got_m)[0] == bits(want)[0]
    b = witness_inputs()["B"]
    yb = np.where(b == 4096, np.float32(2.0 ** 24), b).astype(np.float32)
    got_m, _ = gpu_bn(yb.reshape(5, 1, yb.size // 5), stream=torch.cuda.Stream(DEV))
    assert bits(got_m)[0] == bits(np.float32(gold["B"][1]) / np.float32(yb.size))[0]
    # arguments
    x = torch.zeros(64, device=DEV)
    o = torch.zeros(8, device=DEV)
    p = x.data_ptr()
    assert B.es_bn_batch_stats(p, 0, 2, 8, o.data_ptr(), o.data_ptr() + 8, o.data_ptr() + 16, 2) == B.ES_EINVAL
    assert B.es_bn_batch_stats(p, 2, 70000, 8, o.data_ptr(), o.data_ptr() + 8, o.data_ptr() + 16, 2) == B.ES_EINVAL
    assert B.es_bn_batch_stats(p, 1 << 20, 2, 1 << 12, o.data_ptr(), o.data_ptr() + 8, o.data_ptr() + 16, 2) == B.ES_EINVAL
    assert B.es_bn_batch_stats(p + 2, 2, 2, 8, o.data_ptr(), o.data_ptr() + 8, o.data_ptr() + 16, 2) == B.ES_EINVAL
    assert B.es_bn_batch_stats(p, 2, 2, 8, o.data_ptr(), o.data_ptr() + 8, o.data_ptr() + 16, 1) == B.ES_EINVAL   # workspace too small
    assert B.es_bn_batch_stats(p, 2, 0, 8, 0, 0, 0, 0) == B.ES_OK                                                   # no channels
    assert B.es_bn_workspace_floats(2, 2, 8) == 2 and B.es_bn_workspace_floats(3, 5, 4097) == 5 * 4


def test_clipped_update_parity():
    rng = np.random.default_rng(9)
    n = 3 * 4096 + 37
    for max_norm, eps, streaming in ((0.5, 1e-6, 0), (1e9, 1e-6, 1), (2.0, 0.0, 1), (0.5, 1e-6, 1)):
        g = rng.standard_normal(n).astype(np.float32) * np.float32(0.05)
        p0 = rng.standard_normal(n).astype(np.float32)
        v0 = rng.standard_normal(n).astype(np.float32)
        ssq = np.float32(oracle.tree_sumsq(g))
        norm = np.sqrt(ssq)
        coef = oracle.clip_coef(norm, max_norm, eps)
        want_p, want_v = p0.copy(), v0.copy()
        oracle.sgd_momentum_scaled(want_p, want_v, g, 0.1, 0.9, coef)
        job = ESTJob(1, n, [(0, n)], 1)
        try:
            job.set_option("nontemporal_pv", streaming)      # cacheable and streaming form of the update kernel
            job.p.copy_(torch.from_numpy(p0)); job.v.copy_(torch.from_numpy(v0)); job.avg.copy_(torch.from_numpy(g))
            out2 = torch.zeros(2, device=DEV)
            torch.cuda.synchronize()
            B.check(B.es_grad_sq_norm(job.h, job.avg.data_ptr(), out2.data_ptr()), "es_grad_sq_norm", job.h)
            B.check(B.es_clip_sgd_step(job.h, job.p.data_ptr(), job.v.data_ptr(), job.avg.data_ptr(),
                                       out2.data_ptr(), max_norm, eps, 0.1, 0.9), "es_clip_sgd_step", job.h)
            job.sync()
            assert np.array_equal(bits(job.p.cpu().numpy()), bits(want_p)), (max_norm, eps, float(coef))
            assert np.array_equal(bits(job.v.cpu().numpy()), bits(want_v)), (max_norm, eps, float(coef))
            if max_norm == 1e9:                  # not clipped: the plain update
                pp, vv = p0.copy(), v0.copy()
                oracle.sgd_momentum(pp, vv, g, 0.1, 0.9)
                assert np.array_equal(bits(want_p), bits(pp))
            else:
                assert coef < 1.0
            # arguments
            assert B.es_clip_sgd_step(job.h, job.p.data_ptr(), job.v.data_ptr(), job.avg.data_ptr(), 0,
                                      1.0, 0.0, 0.1, 0.9) == B.ES_EINVAL
            assert B.es_clip_sgd_step(job.h, job.p.data_ptr(), job.v.data_ptr(), job.avg.data_ptr(),
                                      out2.data_ptr(), -1.0, 0.0, 0.1, 0.9) == B.ES_EINVAL
            assert B.es_clip_sgd_step(job.h, job.p.data_ptr(), job.p.data_ptr(), job.avg.data_ptr(),
                                      out2.data_ptr(), 1.0, 0.0, 0.1, 0.9) == B.ES_EINVAL
        finally:
            job.close()
