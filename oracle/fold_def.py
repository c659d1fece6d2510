"""Closed form of the ring-ordered reduction, in numpy.  TEST INFRASTRUCTURE ONLY.

Unrolling the reduce-scatter of an N-rank ring shows that the partial sum of
chunk c starts at rank c and visits ranks c+1, c+2, ... (mod N) in turn, so

    out[i] = ( (..((g[c][i] + g[c+1][i]) + g[c+2][i]) ..) + g[c+N-1][i] ) / N

for every element i of chunk c, each + and the / rounded to fp32.  This file
writes that out directly.  It is deliberately independent of es_oracle.c (own
chunk geometry, numpy arithmetic): the tests use it to cross-check the
message-passing simulator, and to evaluate sampled outputs of buckets too
large for the simulator to hold.
"""
from __future__ import annotations

from typing import Callable, Tuple

import numpy as np


def chunk_len(L: int, N: int, A: int) -> int:
    per_rank = -(-L // N)
    return -(-per_rank // A) * A


def chunk_of(i: int, L: int, N: int, A: int) -> int:
    return i // chunk_len(L, N, A) if L else 0


def chunk_range(c: int, L: int, N: int, A: int) -> Tuple[int, int]:
    cl = chunk_len(L, N, A)
    return min(L, c * cl), min(L, (c + 1) * cl)


def fold_window(fetch: Callable[[int, int, int], np.ndarray], lo: int, hi: int,
                L: int, N: int, A: int) -> np.ndarray:
    """Averaged gradient for bucket-local indices [lo, hi).

    ``fetch(rank, a, b)`` returns rank's fp32 gradient values for bucket-local
    indices [a, b)."""
    out = np.empty(hi - lo, dtype=np.float32)
    n = np.float32(N)
    a = lo
    while a < hi:
        c = chunk_of(a, L, N, A)
        b = min(hi, chunk_range(c, L, N, A)[1])
        acc = fetch(c % N, a, b).astype(np.float32, copy=True)
        for k in range(1, N):
            acc = acc + fetch((c + k) % N, a, b)
        out[a - lo:b - lo] = acc / n
        a = b
    return out


def fold_reduce(rank_grads: np.ndarray, A: int = 1) -> np.ndarray:
    """Averaged gradient of a whole bucket from the (N, L) array of rank gradients."""
    N, L = rank_grads.shape
    g = np.asarray(rank_grads, dtype=np.float32)
    return fold_window(lambda r, a, b: g[r, a:b], 0, L, L, N, A)


def fold_reduce_gather(rank_grads: np.ndarray, A: int = 1) -> np.ndarray:
    """The same closed form, one gather per step of the fold instead of one loop per chunk:
    element i of chunk c(i) adds ranks c(i), c(i)+1, ... (mod N) in turn.  For buckets with very
    many ranks and few elements per chunk, where the per-chunk loop above is too slow."""
    g = np.asarray(rank_grads, dtype=np.float32)
    N, L = g.shape
    if L == 0:
        return np.zeros(0, dtype=np.float32)
    idx = np.arange(L)
    start = idx // chunk_len(L, N, A)
    acc = g[start % N, idx].astype(np.float32, copy=True)
    for k in range(1, N):
        acc = acc + g[(start + k) % N, idx]
    return acc / np.float32(N)
