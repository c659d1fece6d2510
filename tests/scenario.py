"""A multi-step EST job described once and run three ways: as N ordinary ranks
(oracle.ddp_reference), as time-sliced ESTs on simulated workers on the CPU
(oracle.est_model), and through the HIP library (tests/test_gpu_*.py).

Per global step t, EST e's mini-batch (a) draws a dropout mask from its RNG
state, (b) moves its BatchNorm running statistics by one fp32 add of a seeded
delta (so a stale or mixed-up context shows in every later step), and
(c) produces a seeded synthetic gradient.
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from workloads import synth
from workloads.buckets import Layout
from workloads.configs import Config, Grouping


@dataclass(frozen=True)
class Scenario:
    n_logical: int
    layout: Layout
    chunk_align: int
    seed: int
    steps: int = 3
    lr: float = 0.1
    momentum: float = 0.9
    mask_n: int = 0
    p_drop: float = 0.1
    bn_channels: Tuple[int, ...] = ()

    @property
    def bn_len(self) -> int:
        return 2 * sum(self.bn_channels)

    @property
    def bn_segments(self) -> List[Tuple[int, int]]:
        """(offset, len) of every live BN tensor inside an EST's BN vector: mean, var per layer."""
        segs, off = [], 0
        for c in self.bn_channels:
            segs += [(off, c), (off + c, c)]
            off += 2 * c
        return segs


def from_config(cfg: Config, steps: Optional[int] = None, mask_n: Optional[int] = None) -> Scenario:
    n_mask = 0
    if cfg.dropout:
        n_mask = int(np.prod((32, 128, 768))) if mask_n is None else mask_n
    return Scenario(cfg.n_logical, cfg.layout, cfg.chunk_align, cfg.seed,
                    cfg.steps if steps is None else steps, cfg.lr, cfg.momentum,
                    n_mask, 0.1, cfg.bn_channels)


def philox_seed(sc: Scenario, e: int) -> int:
    return synth.stream_key(sc.seed, 0, 7_000_000 + e)


def grad(sc: Scenario, t: int, e: int, b: int, device="cpu"):
    return synth.gradient(sc.layout, b, sc.seed, t, e, device)


def _bn_layout(sc: Scenario) -> Layout:
    n = sc.bn_len
    return Layout(n, ((0, n),), ((0, n, 1),))


def bn_init(sc: Scenario, e: int, device="cpu"):
    return synth.values(_bn_layout(sc), 0, sc.bn_len, sc.seed, 0, synth.STREAM_BN + e, 1.0, False, device)


def bn_delta(sc: Scenario, t: int, e: int, device="cpu"):
    return synth.values(_bn_layout(sc), 0, sc.bn_len, sc.seed, t + 1, synth.STREAM_BN + e, 0.1, False, device)


def digest(a: np.ndarray) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


@dataclass
class Result:
    p: np.ndarray
    v: np.ndarray
    avg: np.ndarray                      # averaged gradient of the last step
    philox: Optional[np.ndarray]         # (N, 2) uint64
    bn: Optional[np.ndarray]             # (N, bn_len) fp32
    masks: Dict[Tuple[int, int], str] = field(default_factory=dict)   # (step, est) -> sha256


def assert_same(a: Result, b: Result, what: str = "") -> None:
    def eq(x, y, name):
        if x is None and y is None:
            return
        xb = np.ascontiguousarray(x).view(np.uint8)
        yb = np.ascontiguousarray(y).view(np.uint8)
        assert xb.shape == yb.shape, (what, name)
        if not np.array_equal(xb, yb):
            xs = np.ascontiguousarray(x).reshape(-1)
            ys = np.ascontiguousarray(y).reshape(-1)
            bad = np.flatnonzero(xs.view(np.uint32 if xs.dtype == np.float32 else xs.dtype)
                                 != ys.view(np.uint32 if ys.dtype == np.float32 else ys.dtype))
            raise AssertionError(f"{what}: {name} differs at {bad.size} of {xs.size} places, "
                                 f"first {bad[:5]}: {xs[bad[:5]]} vs {ys[bad[:5]]}")
    eq(a.avg, b.avg, "averaged gradient")
    eq(a.v, b.v, "momentum")
    eq(a.p, b.p, "parameters")
    eq(a.philox, b.philox, "philox state")
    eq(a.bn, b.bn, "bn state")
    assert a.masks == b.masks, (what, "dropout masks")


def run_ddp_reference(sc: Scenario, gen_device="cpu") -> Result:
    """``gen_device`` only chooses where torch evaluates the seeded input generator
    (same bits on either device); the reference itself runs on the host."""
    from oracle.ddp_reference import DDPReference
    N = sc.n_logical
    seeds = [philox_seed(sc, e) for e in range(N)] if sc.mask_n else None
    bn0 = np.stack([bn_init(sc, e).numpy() for e in range(N)]) if sc.bn_len else None
    ref = DDPReference(N, sc.layout.buckets, sc.layout.n_params, sc.chunk_align, sc.lr, sc.momentum,
                       synth.params(sc.layout, sc.seed).numpy(), seeds, bn0)
    masks = {}
    for t in range(sc.steps):
        for r in range(N):
            m = ref.local_step(r, sc.mask_n, sc.p_drop,
                               bn_delta(sc, t, r).numpy() if sc.bn_len else None)
            if m is not None:
                masks[(t, r)] = digest(m)
        ref.global_step(lambda r, b: grad(sc, t, r, b, gen_device).cpu().numpy())
    return Result(ref.p, ref.v, ref.avg, ref.philox, ref.bn, masks)


def run_est_model(sc: Scenario, g: Grouping, regroup_at: Optional[Dict[int, Grouping]] = None,
                  model_cls=None) -> Result:
    """``regroup_at`` maps a step index to the grouping the job continues with from that
    step on, through an on-demand checkpoint and a fresh model (an elasticity event)."""
    from oracle.est_model import ESTModel
    if model_cls is not None:
        ESTModel = model_cls
    N = sc.n_logical
    seeds = [philox_seed(sc, e) for e in range(N)] if sc.mask_n else None
    bn0 = np.stack([bn_init(sc, e).numpy() for e in range(N)]) if sc.bn_len else None
    m = ESTModel(N, g.worker_of_est, g.slot_of_est, sc.layout.buckets, sc.layout.n_params,
                 sc.chunk_align, sc.lr, sc.momentum, synth.params(sc.layout, sc.seed).numpy(),
                 seeds, bn0)
    masks = {}
    for t in range(sc.steps):
        if regroup_at and t in regroup_at:
            ck = m.checkpoint()
            g = regroup_at[t]
            junk = np.full(sc.layout.n_params, np.nan, dtype=np.float32)
            m = ESTModel(N, g.worker_of_est, g.slot_of_est, sc.layout.buckets, sc.layout.n_params,
                         sc.chunk_align, sc.lr, sc.momentum, junk,
                         [0] * N if sc.mask_n else None,
                         np.full((N, sc.bn_len), np.nan, dtype=np.float32) if sc.bn_len else None)
            m.load_checkpoint(ck)
        for e in g.schedule():
            m.ctx_restore(e)
            mk = m.local_step(e, sc.mask_n, sc.p_drop,
                              bn_delta(sc, t, e).numpy() if sc.bn_len else None)
            if mk is not None:
                masks[(t, e)] = digest(mk)
            for b in range(sc.layout.n_buckets):
                m.accumulate(e, b, grad(sc, t, e, b).numpy())
            m.ctx_save(e)
        m.reduce_and_update()
    philox = np.stack([m.est_rng(e) for e in range(N)]) if sc.mask_n else None
    bn = np.stack([m.est_bn(e) for e in range(N)]) if sc.bn_len else None
    return Result(m.p, m.v, m.avg, philox, bn, masks)
