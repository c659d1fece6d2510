"""The allocation-free norm (es_grad_sq_norm_static, block partials in a fixed device array of
the library) against es_grad_sq_norm on the same vectors, bit for bit, and against the CPU
oracle: two calls in a row, the second on a smaller input, so that what the first call left
in the shared array is there when the second runs."""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from paper_2208_14228_amd import binding as B
    from paper_2208_14228_amd.job import ESTJob
    DEV = "cuda:0"


def _vec(n, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(n) * np.exp2(rng.integers(-12, 12, n))).astype(np.float32)


def _with_handle(x_dev, n):
    job = ESTJob(1, n, [(0, n)], 1)
    try:
        out = torch.full((2,), float("nan"), device=DEV)
        B.check(B.es_grad_sq_norm(job.h, x_dev.data_ptr(), out.data_ptr()), "es_grad_sq_norm", job.h)
        job.sync()
        return out.cpu().numpy()
    finally:
        job.close()


def test_two_calls_in_a_row_second_smaller():
    sizes = [5 * 4096 * 256 + 4097 + 3, 3 * 4096 + 37]           # 1,281 partials, then 4
    xs = [_vec(n, 100 + k) for k, n in enumerate(sizes)]
    devs = [torch.from_numpy(x).to(DEV) for x in xs]
    outs = [torch.full((2,), float("nan"), device=DEV) for _ in xs]
    stream = torch.cuda.Stream(DEV)
    torch.cuda.synchronize()
    # both calls back to back on one stream, nothing in between
    for n, d, o in zip(sizes, devs, outs):
        print(f"[gpu-case] es_grad_sq_norm_static n={n}", flush=True)
        B.check(B.es_grad_sq_norm_static(d.data_ptr(), n, o.data_ptr(), stream.cuda_stream),
                "es_grad_sq_norm_static")
    stream.synchronize()
    torch.cuda.synchronize()
    for n, x, d, o in zip(sizes, xs, devs, outs):
        got = o.cpu().numpy()
        ref = _with_handle(d, n)
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), (n, got, ref)
        want = np.float32(oracle.tree_sumsq(x))
        assert got[0].view(np.uint32) == want.view(np.uint32), n
        assert got[1].view(np.uint32) == np.sqrt(want).view(np.uint32), n


def test_limits_and_arguments():
    out = torch.zeros(2, device=DEV)
    x = torch.ones(8, device=DEV)
    assert B.es_grad_sq_norm_static(x.data_ptr(), (1 << 30) + 1, out.data_ptr(), 0) == B.ES_EINVAL
    assert B.es_grad_sq_norm_static(x.data_ptr() + 4, 4, out.data_ptr(), 0) == B.ES_EINVAL
    assert B.es_grad_sq_norm_static(x.data_ptr(), 8, 0, 0) == B.ES_EINVAL
    assert B.es_grad_sq_norm_static(0, 8, out.data_ptr(), 0) == B.ES_EINVAL
    # n = 0 is the empty sum
    out.fill_(7.0)
    torch.cuda.synchronize()
    B.check(B.es_grad_sq_norm_static(0, 0, out.data_ptr(), 0), "es_grad_sq_norm_static")
    torch.cuda.synchronize()
    assert tuple(out.cpu().numpy()) == (0.0, 0.0)
    B.check(B.es_grad_sq_norm_static(x.data_ptr(), 8, out.data_ptr(), 0), "es_grad_sq_norm_static")
    torch.cuda.synchronize()
    assert out.cpu().numpy()[0] == 8.0


def test_maximum_size():
    """n = 2^30, the documented limit: every one of the 2^18 partials of the fixed array is used."""
    n = 1 << 30
    rng = np.random.default_rng(5)
    x = rng.integers(-8, 9, n, dtype=np.int8).astype(np.float32)
    x *= np.float32(1.0 / 3.0)                           # squares no longer exact: the order matters
    want = np.float32(oracle.tree_sumsq(x))
    d = torch.from_numpy(x).to(DEV)
    out = torch.full((2,), float("nan"), device=DEV)
    torch.cuda.synchronize()
    print(f"[gpu-case] es_grad_sq_norm_static n={n}", flush=True)
    B.check(B.es_grad_sq_norm_static(d.data_ptr(), n, out.data_ptr(), 0), "es_grad_sq_norm_static")
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert got[0].view(np.uint32) == want.view(np.uint32), (got, want)
    assert got[1].view(np.uint32) == np.sqrt(want).view(np.uint32)
