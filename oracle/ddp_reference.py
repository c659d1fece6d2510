"""N-rank data-parallel reference run.  TEST INFRASTRUCTURE ONLY.

The paper's claim (§3.1, §3.3 D1) is that N ESTs time-sliced on any number of
workers produce bitwise the same result as N ordinary DDP workers.  This is
that ordinary run, written out: N ranks that each own their RNG state and
BatchNorm running statistics for the whole job (never saved, restored or
moved), a per-bucket ring all-reduce of their gradients through the
message-passing simulator, /N, and one SGD-momentum update of the single
parameter replica per global step (§3.2).
"""
from __future__ import annotations

from typing import Callable, List, Optional, Sequence, Tuple

import numpy as np

from . import dropout_mask, ring_order_reduce, sgd_momentum


class DDPReference:
    def __init__(self, n_ranks: int, buckets: Sequence[Tuple[int, int]], n_params: int,
                 chunk_align: int, lr: float, momentum: float, p0: np.ndarray,
                 philox_seeds: Optional[Sequence[int]] = None,
                 bn0: Optional[np.ndarray] = None):
        self.N = n_ranks
        self.buckets = list(buckets)
        self.P = n_params
        self.A = chunk_align
        self.lr, self.mu = lr, momentum
        self.p = np.array(p0, dtype=np.float32, copy=True)
        self.v = np.zeros(n_params, dtype=np.float32)
        self.avg = np.zeros(n_params, dtype=np.float32)
        self.philox = None
        if philox_seeds is not None:
            self.philox = np.array([[s, 0] for s in philox_seeds], dtype=np.uint64)
        self.bn = None
        if bn0 is not None:
            self.bn = np.array(bn0, dtype=np.float32, copy=True)        # (N, total channels*2)

    # one rank's mini-batch: the parts of it that touch per-rank state
    def local_step(self, rank: int, mask_n: int = 0, p_drop: float = 0.0,
                   bn_delta: Optional[np.ndarray] = None) -> Optional[np.ndarray]:
        mask = None
        if self.philox is not None and mask_n:
            mask = dropout_mask(self.philox[rank], mask_n, p_drop)
        if self.bn is not None and bn_delta is not None:
            self.bn[rank] = self.bn[rank] + bn_delta.astype(np.float32)
        return mask

    # end of the global step: aggregate and update
    def global_step(self, fetch_grad: Callable[[int, int], np.ndarray]) -> None:
        """``fetch_grad(rank, bucket)`` returns that rank's fp32 gradient bucket."""
        for b, (off, ln) in enumerate(self.buckets):
            ranks = np.empty((self.N, ln), dtype=np.float32)
            for r in range(self.N):
                ranks[r] = fetch_grad(r, b)
            self.avg[off:off + ln] = ring_order_reduce(ranks, self.A, clobber=True)
        sgd_momentum(self.p, self.v, self.avg, self.lr, self.mu)
