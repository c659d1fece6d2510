"""Fixed-tree global norm on the GPU vs. the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from paper_2208_14228_amd import binding as B
    from paper_2208_14228_amd.job import ESTJob
    DEV = "cuda:0"


def gpu_norm(x: np.ndarray, shift=0):
    n = x.size
    job = ESTJob(1, n, [(0, n)], 1)
    try:
        buf = torch.zeros(n + 8, device=DEV)
        vec = buf[shift:shift + n]
        vec.copy_(torch.from_numpy(x))
        out = torch.full((2,), float("nan"), device=DEV)
        torch.cuda.synchronize()
        st = B.es_grad_sq_norm(job.h, vec.data_ptr(), out.data_ptr())
        if st:
            return st
        job.sync()
        return out.cpu().numpy()
    finally:
        job.close()


@pytest.mark.parametrize("n", [1, 3, 255, 4095, 4096, 4097, 8191, 3 * 4096 + 37, 256 * 4096 + 1,
                               1_300_003, 25_557_032])
def test_norm_parity(n):
    rng = np.random.default_rng(n)
    x = (rng.standard_normal(n) * np.exp2(rng.integers(-12, 12, n))).astype(np.float32)
    got = gpu_norm(x)
    want = oracle.tree_sumsq(x)
    assert got[0].view(np.uint32) == np.float32(want).view(np.uint32)
    assert got[1].view(np.uint32) == np.sqrt(np.float32(want)).view(np.uint32)


def test_norm_special_values_and_alignment():
    x = np.zeros(10_000, dtype=np.float32)
    assert tuple(gpu_norm(x)) == (0.0, 0.0)
    x[:] = 1e-30                                         # squares underflow to denormals / zero alike
    got = gpu_norm(x)
    assert got[0].view(np.uint32) == np.float32(oracle.tree_sumsq(x)).view(np.uint32)
    x = np.ones(100_003, dtype=np.float32)
    assert gpu_norm(x)[0] == 100_003.0
    assert gpu_norm(x, shift=1) == B.ES_EINVAL           # 4-byte aligned only: rejected
    assert gpu_norm(x, shift=4)[0] == 100_003.0          # 16-byte aligned view


def test_hand_derived_tree_witness_on_gpu():
    """The two order witnesses of tests/golden/tree_witness.txt: the kernel's tree has to be the
    specified one, not merely agree with the oracle."""
    from test_oracle_tree import golden_witness, witness_inputs
    gold = golden_witness()
    for name, x in witness_inputs().items():
        got = gpu_norm(x)
        assert int(got[0].view(np.uint32)) == gold[name][2], (name, got)
