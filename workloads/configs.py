"""The five benchmark configurations and their EST-to-worker groupings.

A grouping assigns every logical worker (EST, identified by its constant
virtual rank, paper §3.3 D1) to a simulated physical worker and to a slot
inside that worker's arena, and fixes the order in which each worker runs its
ESTs.  Results must not depend on it.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

from . import shapes
from .buckets import Layout, ddp_buckets, single_bucket

SEED_BASE = 0x5EED0000
LR = 0.1
MOMENTUM = 0.9
DROPOUT_P = 0.1
DROPOUT_SHAPE = (32, 128, 768)


@dataclass(frozen=True)
class Grouping:
    name: str
    worker_of_est: Tuple[int, ...]
    slot_of_est: Tuple[int, ...]

    @property
    def n_workers(self) -> int:
        return max(self.worker_of_est) + 1

    def schedule(self) -> List[int]:
        """ESTs in execution order: worker by worker, each worker in slot order."""
        n = len(self.worker_of_est)
        return sorted(range(n), key=lambda e: (self.worker_of_est[e], self.slot_of_est[e]))


def contiguous(sizes: Sequence[int], name: str = "") -> Grouping:
    w, s = [], []
    for wi, k in enumerate(sizes):
        w += [wi] * k
        s += list(range(k))
    return Grouping(name or "x".join(map(str, sizes)), tuple(w), tuple(s))


def round_robin(sizes: Sequence[int], name: str = "") -> Grouping:
    """Deal ESTs to workers in turn until each worker holds its size."""
    n = sum(sizes)
    left = list(sizes)
    w = [0] * n
    s = [0] * n
    cnt = [0] * len(sizes)
    wi = 0
    for e in range(n):
        while left[wi] == 0:
            wi = (wi + 1) % len(sizes)
        w[e], s[e] = wi, cnt[wi]
        cnt[wi] += 1
        left[wi] -= 1
        wi = (wi + 1) % len(sizes)
    return Grouping(name or "rr" + "-".join(map(str, sizes)), tuple(w), tuple(s))


def reversed_slots(g: Grouping) -> Grouping:
    """Same workers, but every worker stores and runs its ESTs in reverse order."""
    cnt: Dict[int, int] = {}
    for w in g.worker_of_est:
        cnt[w] = cnt.get(w, 0) + 1
    return Grouping(g.name + "-rev", g.worker_of_est,
                    tuple(cnt[w] - 1 - s for w, s in zip(g.worker_of_est, g.slot_of_est)))


@dataclass(frozen=True)
class Config:
    cid: int
    name: str
    n_logical: int
    layout: Layout
    chunk_align: int
    groupings: Tuple[Grouping, ...]
    bn_channels: Tuple[int, ...] = ()
    dropout: bool = False
    steps: int = 3
    lr: float = LR
    momentum: float = MOMENTUM

    @property
    def seed(self) -> int:
        return SEED_BASE + self.cid


def config(cid: int) -> Config:
    if cid == 1:
        return Config(1, "flat-1M", 4, single_bucket(1 << 20), 4,
                      (contiguous([4]), contiguous([1] * 4, "1x4")))
    if cid == 2:
        return Config(2, "resnet50", 8, ddp_buckets(shapes.resnet50()), 4,
                      (contiguous([8]), contiguous([4, 4])))
    if cid == 3:
        return Config(3, "bert-base+philox", 16, ddp_buckets(shapes.bert_base()), 4,
                      (contiguous([16]), contiguous([1] * 16, "1x16")), dropout=True)
    if cid == 4:
        return Config(4, "resnet50+bn", 32, ddp_buckets(shapes.resnet50()), 4,
                      (contiguous([32]), contiguous([8] * 4), contiguous([1] * 32, "1x32")),
                      bn_channels=tuple(shapes.resnet50_bn_channels()))
    if cid == 5:
        sizes = [3, 5, 7, 9, 11, 13, 16]
        return Config(5, "gpt2-medium", 64, ddp_buckets(shapes.gpt2_medium()), 4,
                      (contiguous([64]), contiguous(sizes), round_robin(sizes)))
    raise ValueError(f"no configuration {cid}")
