"""Time-sliced EST execution on simulated workers, on the CPU.  TEST INFRASTRUCTURE ONLY.

Follows the paper's §3.2 step by step: every worker owns one live copy of the
small per-EST state (RNG state, BatchNorm running statistics) and an arena of
context slots, one per EST it hosts.  Within a global step a worker runs its
ESTs one after the other; for each it restores the EST's context into the live
state, lets the EST's mini-batch touch the live state, stages the EST's
gradients in its slot, and saves the live state back.  When every EST has run,
gradients are all-reduced among ESTs by *virtual rank* (§3.3 D1), never by
worker or slot, and the shared replica is updated once.

Pinned against ddp_reference.DDPReference (N ranks that never switch): every
grouping has to give the same bits.
"""
from __future__ import annotations

from typing import Callable, List, Optional, Sequence, Tuple

import numpy as np

from . import dropout_mask, ring_order_reduce, sgd_momentum


class ESTModel:
    def __init__(self, n_logical: int, worker_of_est: Sequence[int], slot_of_est: Sequence[int],
                 buckets: Sequence[Tuple[int, int]], n_params: int, chunk_align: int,
                 lr: float, momentum: float, p0: np.ndarray,
                 philox_seeds: Optional[Sequence[int]] = None,
                 bn0: Optional[np.ndarray] = None):
        self.N = n_logical
        self.worker_of_est = list(worker_of_est)
        self.slot_of_est = list(slot_of_est)
        self.buckets = list(buckets)
        self.A = chunk_align
        self.lr, self.mu = lr, momentum
        self.p = np.array(p0, dtype=np.float32, copy=True)
        self.v = np.zeros(n_params, dtype=np.float32)
        self.avg = np.zeros(n_params, dtype=np.float32)
        n_workers = max(self.worker_of_est) + 1
        per_worker = [sum(1 for w in self.worker_of_est if w == i) for i in range(n_workers)]
        self.has_rng = philox_seeds is not None
        self.has_bn = bn0 is not None
        bn_len = bn0.shape[1] if self.has_bn else 0
        # live state: one per worker; deliberately filled with junk so that a
        # missing restore shows
        self.live_rng = [np.full(2, 0xDEADBEEF, dtype=np.uint64) for _ in range(n_workers)]
        self.live_bn = [np.full(bn_len, np.nan, dtype=np.float32) for _ in range(n_workers)]
        # arenas: slot -> context
        self.slot_rng = [np.zeros((k, 2), dtype=np.uint64) for k in per_worker]
        self.slot_bn = [np.zeros((k, bn_len), dtype=np.float32) for k in per_worker]
        self.slot_grad = [[[None] * len(self.buckets) for _ in range(k)] for k in per_worker]
        for e in range(self.N):
            w, s = self.worker_of_est[e], self.slot_of_est[e]
            if self.has_rng:
                self.slot_rng[w][s] = (philox_seeds[e], 0)
            if self.has_bn:
                self.slot_bn[w][s] = bn0[e]

    def ctx_restore(self, e: int) -> None:
        w, s = self.worker_of_est[e], self.slot_of_est[e]
        self.live_rng[w][:] = self.slot_rng[w][s]
        self.live_bn[w][:] = self.slot_bn[w][s]

    def ctx_save(self, e: int) -> None:
        w, s = self.worker_of_est[e], self.slot_of_est[e]
        self.slot_rng[w][s] = self.live_rng[w]
        self.slot_bn[w][s] = self.live_bn[w]

    def accumulate(self, e: int, b: int, grad: np.ndarray) -> None:
        w, s = self.worker_of_est[e], self.slot_of_est[e]
        self.slot_grad[w][s][b] = np.array(grad, dtype=np.float32, copy=True)

    def local_step(self, e: int, mask_n: int = 0, p_drop: float = 0.0,
                   bn_delta: Optional[np.ndarray] = None) -> Optional[np.ndarray]:
        """The part of EST e's mini-batch that touches live state on its worker."""
        w = self.worker_of_est[e]
        mask = None
        if self.has_rng and mask_n:
            mask = dropout_mask(self.live_rng[w], mask_n, p_drop)
        if self.has_bn and bn_delta is not None:
            self.live_bn[w][:] = self.live_bn[w] + bn_delta.astype(np.float32)
        return mask

    def reduce_and_update(self) -> None:
        for b, (off, ln) in enumerate(self.buckets):
            ranks = np.empty((self.N, ln), dtype=np.float32)
            for e in range(self.N):                      # row index = virtual rank
                w, s = self.worker_of_est[e], self.slot_of_est[e]
                ranks[e] = self.slot_grad[w][s][b]
                self.slot_grad[w][s][b] = None
            self.avg[off:off + ln] = ring_order_reduce(ranks, self.A, clobber=True)
        sgd_momentum(self.p, self.v, self.avg, self.lr, self.mu)

    # On-demand checkpoint (paper section 3.2, "Adapting to elasticity"): the contexts of all
    # ESTs, keyed by virtual rank, plus ONE copy of the shared state.  A job resumed from it
    # may spread the ESTs over workers in any other way.
    def checkpoint(self) -> dict:
        return {
            "rng": [self.est_rng(e).copy() for e in range(self.N)] if self.has_rng else None,
            "bn": [self.est_bn(e).copy() for e in range(self.N)] if self.has_bn else None,
            "p": self.p.copy(), "v": self.v.copy(),
        }

    def load_checkpoint(self, ck: dict) -> None:
        for e in range(self.N):
            w, s = self.worker_of_est[e], self.slot_of_est[e]
            if self.has_rng:
                self.slot_rng[w][s] = ck["rng"][e]
            if self.has_bn:
                self.slot_bn[w][s] = ck["bn"][e]
        self.p[:] = ck["p"]
        self.v[:] = ck["v"]

    def est_rng(self, e: int) -> np.ndarray:
        return self.slot_rng[self.worker_of_est[e]][self.slot_of_est[e]]

    def est_bn(self, e: int) -> np.ndarray:
        return self.slot_bn[self.worker_of_est[e]][self.slot_of_est[e]]


# ---------------------------------------------------------------------------------------------
# Host-swapped gradient contexts (paper section 3.2: an EST's gradients are copied to host
# memory when it is switched out; section 5.1.3: the copies overlap with compute).  At the end of
# the global step the buckets come back one at a time into TWO device buffers: while bucket b is
# reduced out of one buffer, bucket b+1 is copied into the other.  This is pure data movement:
# the result has to be the one of reduce_and_update above.  What has to be right is the
# schedule: which bucket is resident in which buffer when.
#
# The schedule is a list of operations for two in-order queues (copy, compute):
#   ("fill",   b, half, wait)   copy queue:    bucket b of all N ranks -> buffer `half`
#   ("reduce", b, half, wait)   compute queue: ring-ordered reduce of bucket b out of buffer `half`
# `wait` is the index (in the list) of the one operation of the OTHER queue that must have
# finished first, or -1: fill b waits for reduce b-2 (the previous user of its buffer), reduce b
# waits for fill b.  Operations of one queue run in list order.
# ---------------------------------------------------------------------------------------------
def swap_in_schedule(n_buckets: int) -> List[Tuple[str, int, int, int]]:
    ops: List[Tuple[str, int, int, int]] = []
    reduce_at = {}
    for b in range(n_buckets):
        half = b % 2
        ops.append(("fill", b, half, reduce_at.get(b - 2, -1)))
        ops.append(("reduce", b, half, len(ops) - 1))
        reduce_at[b] = len(ops) - 1
    return ops


def run_swap_in(ops: Sequence[Tuple[str, int, int, int]], host_rows: Callable[[int], np.ndarray],
                bucket_lens: Sequence[int], n_ranks: int, chunk_align: int,
                rng: Optional[np.random.Generator] = None) -> List[np.ndarray]:
    """Executes a schedule on real data under ONE legal interleaving of the two queues (chosen by
    ``rng``; None = strictly alternating) and returns the averaged gradient per bucket.

    ``host_rows(b)`` returns the (N, L_b) array of the ranks' host-resident gradients of bucket b.
    A buffer is poisoned (NaN) as soon as its reduce has run, and a fill overwrites whatever the
    buffer holds, so a schedule that reduces before the fill has finished, or refills a buffer
    that is still to be read, produces NaNs or another bucket's numbers.  Raises on deadlock."""
    lmax = max(list(bucket_lens) + [1])
    bufs = [np.full((n_ranks, lmax), np.nan, dtype=np.float32) for _ in range(2)]
    holds = [None, None]                          # which bucket each buffer holds now
    done = [False] * len(ops)
    out: List[Optional[np.ndarray]] = [None] * len(bucket_lens)
    queues = {"fill": [i for i, o in enumerate(ops) if o[0] == "fill"],
              "reduce": [i for i, o in enumerate(ops) if o[0] == "reduce"]}
    heads = {"fill": 0, "reduce": 0}
    turn = 0
    while not all(done):
        ready = []
        for q in ("fill", "reduce"):
            if heads[q] < len(queues[q]):
                i = queues[q][heads[q]]
                w = ops[i][3]
                if w < 0 or done[w]:
                    ready.append(q)
        if not ready:
            raise RuntimeError("schedule deadlocks")
        if rng is None:
            q = ready[turn % len(ready)]
            turn += 1
        else:
            q = ready[int(rng.integers(len(ready)))]
        i = queues[q][heads[q]]
        kind, b, half, _ = ops[i]
        L = bucket_lens[b]
        if kind == "fill":
            bufs[half][:, :L] = host_rows(b)
            holds[half] = b
        else:
            if holds[half] != b:
                raise AssertionError(f"reduce of bucket {b} finds bucket {holds[half]} in buffer {half}")
            out[b] = ring_order_reduce(np.ascontiguousarray(bufs[half][:, :L]), chunk_align)
            bufs[half][:] = np.nan
            holds[half] = None
        done[i] = True
        heads[q] += 1
    return out


class SwappedESTModel(ESTModel):
    """ESTModel whose staged gradients live in host memory and come back through the two-buffer
    schedule at the end of the global step."""

    def reduce_and_update(self, rng: Optional[np.random.Generator] = None, ops=None) -> None:
        def rows(b):
            r = np.empty((self.N, self.buckets[b][1]), dtype=np.float32)
            for e in range(self.N):
                w, s = self.worker_of_est[e], self.slot_of_est[e]
                r[e] = self.slot_grad[w][s][b]
            return r
        lens = [ln for _, ln in self.buckets]
        avg = run_swap_in(ops if ops is not None else swap_in_schedule(len(self.buckets)), rows, lens,
                          self.N, self.A, rng)
        for b, (off, ln) in enumerate(self.buckets):
            self.avg[off:off + ln] = avg[b]
            for e in range(self.N):
                self.slot_grad[self.worker_of_est[e]][self.slot_of_est[e]][b] = None
        sgd_momentum(self.p, self.v, self.avg, self.lr, self.mu)
