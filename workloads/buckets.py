"""DDP-style gradient bucket layout for a list of tensors.

The paper (§3.3) says gradients are gathered into buckets whose mapping first
follows the reversed topological order of the graph, and that the mapping is
recorded and reinstated rather than rebuilt (D1).  It gives no bucket size.
The reading used here: walk the tensors in reverse forward order, never split
a tensor, close a bucket as soon as it holds at least ``cap_bytes`` (25 MiB of
fp32 by default); a single tensor larger than the cap is a bucket of its own.
The flat parameter space is the concatenation of the buckets, so every bucket
is a contiguous [offset, offset+len) range of it.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence, Tuple

from .shapes import Tensor

CAP_BYTES = 25 * 2**20


@dataclass(frozen=True)
class Layout:
    """Flat fp32 parameter space split into buckets, plus per-tensor placement."""
    n_params: int
    buckets: Tuple[Tuple[int, int], ...]          # (offset_elems, len_elems)
    tensors: Tuple[Tuple[int, int, int], ...]     # (offset_elems, len_elems, fan_in), flat order

    @property
    def n_buckets(self) -> int:
        return len(self.buckets)


def ddp_buckets(tensors: Sequence[Tensor], cap_bytes: int = CAP_BYTES) -> Layout:
    cap = cap_bytes // 4
    buckets: List[Tuple[int, int]] = []
    placed: List[Tuple[int, int, int]] = []
    off = 0
    start = 0
    for t in reversed(list(tensors)):
        placed.append((off, t.numel, t.fan_in))
        off += t.numel
        if off - start >= cap:
            buckets.append((start, off - start))
            start = off
    if off > start:
        buckets.append((start, off - start))
    return Layout(off, tuple(buckets), tuple(placed))


def single_bucket(n: int, fan_in: int = 1) -> Layout:
    return Layout(n, ((0, n),), ((0, n, fan_in),))


def custom(bucket_lens: Sequence[int], fan_in: int = 1) -> Layout:
    """Arbitrary bucket lengths (tests: ragged and empty buckets)."""
    buckets, off = [], 0
    for L in bucket_lens:
        buckets.append((off, L))
        off += L
    return Layout(off, tuple(buckets), tuple((o, l, fan_in) for o, l in buckets if l))
