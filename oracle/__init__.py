"""CPU oracle of the EST step.  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  The product (the HIP library and its
Python binding) never does, and this package imports nothing of the product.

  es_oracle.c       message-passing ring all-reduce among N simulated ranks,
                    /N, SGD-momentum (also with the gradient clipped by its global
                    norm), Philox4x32-10 dropout mask, fixed-tree sum of squares and
                    BatchNorm batch statistics along the same tree (plain C, fp32)
  fold_def.py       the closed form of the same reduction (per-chunk rotated
                    left fold) in numpy: cross-check of the simulator and
                    evaluator of sampled outputs at sizes the simulator cannot hold
  ddp_reference.py  N independent ranks, each with its own RNG and BatchNorm
                    state that is never switched: the plain definition that a
                    time-sliced, grouped EST run has to reproduce bit for bit

Parity pins (tests/test_oracle_*.py): N=1 identity; integer-valued inputs vs.
exact integer sums; explicit parenthesised brute force for N<=4; an
order-sensitivity witness with hand-derived bits (tests/golden/); recursive
summation error bound vs. exact rational sums; division vs. exact rational
rounding; SGD vs. exact rationals and a non-contraction witness; Philox vs. an
independent big-integer implementation, vs. the Philox engine that ships in
PyTorch's headers, and round-function invertibility; dropout keep rate and
stream splitting; the fixed-tree sum of squares vs. a numpy twin built from
reshapes, exact integer cases, single-element cases and the pairwise-summation
error bound, and two hand-derived order witnesses (tests/golden/tree_witness.txt);
the clip coefficient vs. exact rational rounding and the unclipped case vs. the plain
update; BatchNorm statistics vs. the witnesses, exact dyadic cases, a numpy twin, the
float64 mean/variance within the summation error bound, and layout permutations.
No function here is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "es_oracle.c")
_LIB = os.path.join(_HERE, "libes_oracle.so")
_LIB_OMP = os.path.join(_HERE, "libes_oracle_omp.so")
CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-Wall",
          "-Wno-unknown-pragmas"]

_lib = None
_threaded = False


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc: the single-threaded oracle, and the same file with -fopenmp
    (used only for the all-core timing in bench.py).  Returns the path of the former."""
    for out, extra in ((_LIB, []), (_LIB_OMP, ["-fopenmp"])):
        if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
            subprocess.check_call(["gcc", *CFLAGS, *extra, _SRC, "-o", out])
    return _LIB


def use_all_cores(on: bool) -> None:
    """Switch every function of this module to the -fopenmp build of es_oracle.c (or back).
    Same operations on the same operands; only bench.py's all-core timing asks for it."""
    global _lib, _threaded
    if on != _threaded:
        _lib, _threaded = None, on


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB_OMP if _threaded else _LIB)
        f32p = ctypes.POINTER(ctypes.c_float)
        u64p = ctypes.POINTER(ctypes.c_uint64)
        u32p = ctypes.POINTER(ctypes.c_uint32)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        L.eso_chunk_bounds.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32,
                                       ctypes.c_uint32, u64p, u64p]
        L.eso_chunk_bounds.restype = None
        L.eso_ring_allreduce.argtypes = [f32p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32]
        L.eso_ring_allreduce.restype = ctypes.c_int
        L.eso_ring_order_reduce.argtypes = [f32p, ctypes.c_uint64, ctypes.c_uint32,
                                            ctypes.c_uint32, f32p]
        L.eso_ring_order_reduce.restype = ctypes.c_int
        L.eso_sgd_momentum.argtypes = [f32p, f32p, f32p, ctypes.c_uint64,
                                       ctypes.c_float, ctypes.c_float]
        L.eso_sgd_momentum.restype = None
        L.eso_philox4x32_10.argtypes = [u32p, u32p, u32p]
        L.eso_philox4x32_10.restype = None
        L.eso_dropout_threshold.argtypes = [ctypes.c_double]
        L.eso_dropout_threshold.restype = ctypes.c_uint64
        L.eso_dropout_mask.argtypes = [u64p, u8p, ctypes.c_uint64, ctypes.c_uint64]
        L.eso_dropout_mask.restype = None
        L.eso_tree_sumsq.argtypes = [f32p, ctypes.c_uint64]
        L.eso_tree_sumsq.restype = ctypes.c_float
        L.eso_clip_coef.argtypes = [ctypes.c_float, ctypes.c_float, ctypes.c_float]
        L.eso_clip_coef.restype = ctypes.c_float
        L.eso_sgd_momentum_scaled.argtypes = [f32p, f32p, f32p, ctypes.c_uint64, ctypes.c_float,
                                              ctypes.c_float, ctypes.c_float]
        L.eso_sgd_momentum_scaled.restype = None
        L.eso_bn_batch_stats.argtypes = [f32p, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64, f32p, f32p]
        L.eso_bn_batch_stats.restype = None
        _lib = L
    return _lib


def _f32(a: np.ndarray):
    assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def chunk_bounds(L: int, N: int, A: int, c: int) -> Tuple[int, int]:
    lo, hi = ctypes.c_uint64(), ctypes.c_uint64()
    lib().eso_chunk_bounds(L, N, A, c, ctypes.byref(lo), ctypes.byref(hi))
    return lo.value, hi.value


def ring_allreduce(rank_bufs: np.ndarray, A: int = 1) -> np.ndarray:
    """Ring all-reduce (sum) among the N rows of ``rank_bufs`` (N, L) fp32.

    Returns the (N, L) array of what every rank holds afterwards."""
    buf = np.array(rank_bufs, dtype=np.float32, order="C", copy=True)
    N, L = buf.shape
    rc = lib().eso_ring_allreduce(_f32(buf), L, N, A)
    if rc:
        raise MemoryError("oracle ring_allreduce failed")
    return buf


def ring_order_reduce(rank_grads: np.ndarray, A: int = 1, clobber: bool = False) -> np.ndarray:
    """Averaged gradient of one bucket: ring all-reduce over the N rows, then /N.

    ``clobber=True`` lets the simulator use ``rank_grads`` itself as the ranks'
    private buffers (saves a copy at large sizes)."""
    if clobber:
        buf = rank_grads
        assert buf.dtype == np.float32 and buf.flags["C_CONTIGUOUS"]
    else:
        buf = np.array(rank_grads, dtype=np.float32, order="C", copy=True)
    N, L = buf.shape
    out = np.empty(L, dtype=np.float32)
    rc = lib().eso_ring_order_reduce(_f32(buf), L, N, A, _f32(out))
    if rc == -2:
        raise AssertionError("simulated ranks disagree after the all-gather")
    if rc:
        raise MemoryError("oracle ring_order_reduce failed")
    return out


def sgd_momentum(p: np.ndarray, v: np.ndarray, g: np.ndarray, lr: float, mu: float) -> None:
    """In place: v <- mu*v + g ; p <- p - lr*v (fp32, every operation rounded)."""
    assert p.shape == v.shape == g.shape
    lib().eso_sgd_momentum(_f32(p), _f32(v), _f32(g), p.size, lr, mu)


def philox4x32_10(ctr, key) -> Tuple[int, int, int, int]:
    c = (ctypes.c_uint32 * 4)(*ctr)
    k = (ctypes.c_uint32 * 2)(*key)
    o = (ctypes.c_uint32 * 4)()
    lib().eso_philox4x32_10(c, k, o)
    return tuple(o)


def dropout_threshold(p: float) -> int:
    return lib().eso_dropout_threshold(p)


def dropout_mask(state: np.ndarray, n: int, p: float) -> np.ndarray:
    """Keep-mask of n bytes from state = uint64[2] {seed, offset}; advances the offset."""
    assert state.dtype == np.uint64 and state.shape == (2,)
    mask = np.empty(n, dtype=np.uint8)
    lib().eso_dropout_mask(state.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)),
                           mask.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)),
                           n, dropout_threshold(p))
    return mask


def tree_sumsq(x: np.ndarray) -> np.float32:
    """Sum of squares of a flat fp32 vector along the fixed tree (see es_oracle.c)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return np.float32(lib().eso_tree_sumsq(_f32(x) if x.size else None, x.size))


def clip_coef(norm, max_norm, eps) -> np.float32:
    """min(1, max_norm / (norm + eps)), every operation rounded to fp32."""
    return np.float32(lib().eso_clip_coef(np.float32(norm), np.float32(max_norm), np.float32(eps)))


def sgd_momentum_scaled(p: np.ndarray, v: np.ndarray, g: np.ndarray, lr: float, mu: float, coef) -> None:
    """In place: g' = coef*g ; v <- mu*v + g' ; p <- p - lr*v (fp32, every operation rounded)."""
    assert p.shape == v.shape == g.shape
    lib().eso_sgd_momentum_scaled(_f32(p), _f32(v), _f32(g), p.size, lr, mu, np.float32(coef))


def bn_batch_stats(x: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Per-channel mean and biased variance of x[B, C, HW] along the fixed tree (see es_oracle.c)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    B, C, HW = x.shape
    mean = np.empty(C, dtype=np.float32)
    var = np.empty(C, dtype=np.float32)
    if C:
        lib().eso_bn_batch_stats(_f32(x) if x.size else None, B, C, HW, _f32(mean), _f32(var))
    return mean, var
