"""ctypes binding of libes (include/es.h): same names, argument marshalling only.

Every function takes the raw handle / device addresses as integers
(``tensor.data_ptr()``, ``stream.cuda_stream``) and returns the library's
status code; ``check`` turns a negative status into an exception.  Nothing is
computed here.  If the built library is missing the import of ``lib()`` fails
loudly: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

from . import build as _build

ES_OK, ES_EINVAL, ES_ESTATE, ES_ENOMEM, ES_EHIP = 0, -1, -2, -3, -4


class EsBucket(ctypes.Structure):
    _fields_ = [("offset_elems", ctypes.c_uint64), ("len_elems", ctypes.c_uint64)]


class EsBucketLayout(ctypes.Structure):
    _fields_ = [("n_params", ctypes.c_uint64),
                ("n_buckets", ctypes.c_uint32),
                ("buckets", ctypes.POINTER(EsBucket)),
                ("chunk_align", ctypes.c_uint32),
                ("n_state_segs", ctypes.c_uint32),
                ("state_seg_bytes", ctypes.POINTER(ctypes.c_uint64)),
                ("dev_alloc", ctypes.c_void_p),
                ("dev_free", ctypes.c_void_p),
                ("user", ctypes.c_void_p)]


# es_dev_alloc_fn / es_dev_free_fn of include/es.h
DEV_ALLOC_FN = ctypes.CFUNCTYPE(ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p)
DEV_FREE_FN = ctypes.CFUNCTYPE(None, ctypes.c_void_p, ctypes.c_void_p)


class EsSwapOp(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_uint32), ("bucket", ctypes.c_uint32), ("half", ctypes.c_uint32),
                ("wait", ctypes.c_int32)]


class EsTile(ctypes.Structure):
    _fields_ = [("offset_elems", ctypes.c_uint64), ("len_elems", ctypes.c_uint32),
                ("start_rank", ctypes.c_uint32)]


ES_SCHED_MAX_TYPES, ES_SCHED_MAX_P = 8, 4096
ES_SCHED_WASTE_PER_GPU, ES_SCHED_WASTE_AS_PRINTED = 0, 1


class EsSchedPlan(ctypes.Structure):
    """es_sched_plan of include/es_sched.h."""
    _fields_ = [("n_used", ctypes.c_uint32 * ES_SCHED_MAX_TYPES),
                ("est_per_gpu", ctypes.c_uint32 * ES_SCHED_MAX_TYPES),
                ("n_gpus", ctypes.c_uint32), ("n_est", ctypes.c_uint32),
                ("f_overload", ctypes.c_double), ("waste", ctypes.c_double),
                ("throughput", ctypes.c_double)]


class EsError(RuntimeError):
    def __init__(self, status: int, where: str, hip: int = 0):
        self.status = status
        self.hip = hip
        msg = lib().es_strerror(status).decode()
        super().__init__(f"{where}: {msg} (status {status}" + (f", hipError {hip})" if hip else ")"))


_lib: Optional[ctypes.CDLL] = None

_VP = ctypes.c_void_p
_SIGS = {
    "es_init": (ctypes.c_int, [ctypes.POINTER(_VP), ctypes.c_uint32, ctypes.POINTER(EsBucketLayout)]),
    "es_destroy": (ctypes.c_int, [_VP]),
    "es_set_streams": (ctypes.c_int, [_VP, _VP, _VP, _VP]),
    "es_set_grouping": (ctypes.c_int, [_VP, ctypes.c_uint32, ctypes.POINTER(ctypes.c_uint32),
                                       ctypes.POINTER(ctypes.c_uint32)]),
    "es_bind_live_state": (ctypes.c_int, [_VP, ctypes.c_uint32, ctypes.POINTER(_VP)]),
    "es_ctx_restore": (ctypes.c_int, [_VP, ctypes.c_uint32]),
    "es_ctx_save": (ctypes.c_int, [_VP, ctypes.c_uint32]),
    "es_ctx_switch": (ctypes.c_int, [_VP, ctypes.c_uint32, ctypes.c_uint32]),
    "es_accumulate": (ctypes.c_int, [_VP, ctypes.c_uint32, ctypes.c_uint32, _VP]),
    "es_accumulate_batch": (ctypes.c_int, [_VP, ctypes.c_uint32, ctypes.c_uint32,
                                           ctypes.POINTER(ctypes.c_uint32), ctypes.POINTER(_VP)]),
    "es_accumulate_many": (ctypes.c_int, [_VP, ctypes.c_uint32, ctypes.POINTER(ctypes.c_uint32),
                                          ctypes.POINTER(_VP)]),
    "es_est_boundary": (ctypes.c_int, [_VP, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32,
                                       ctypes.POINTER(ctypes.c_uint32), ctypes.POINTER(_VP)]),
    "es_accumulate_in_place": (ctypes.c_int, [_VP, ctypes.c_uint32, _VP]),
    "es_grad_slot": (_VP, [_VP, ctypes.c_uint32, ctypes.c_uint32]),
    "es_stage_fence": (ctypes.c_int, [_VP]),
    "es_dropout_mask": (ctypes.c_int, [_VP, ctypes.c_uint32, ctypes.c_uint32, _VP,
                                       ctypes.c_uint64, ctypes.c_double]),
    "es_ring_order_reduce": (ctypes.c_int, [_VP, _VP]),
    "es_sgd_step": (ctypes.c_int, [_VP, _VP, _VP, _VP, ctypes.c_float, ctypes.c_float]),
    "es_reduce_sgd_step": (ctypes.c_int, [_VP, _VP, _VP, _VP, ctypes.c_float, ctypes.c_float]),
    "es_grad_sq_norm": (ctypes.c_int, [_VP, _VP, _VP]),
    "es_grad_sq_norm_static": (ctypes.c_int, [_VP, ctypes.c_uint64, _VP, _VP]),
    "es_clip_sgd_step": (ctypes.c_int, [_VP, _VP, _VP, _VP, _VP, ctypes.c_float, ctypes.c_float,
                                        ctypes.c_float, ctypes.c_float]),
    "es_bn_workspace_floats": (ctypes.c_uint64, [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64]),
    "es_bn_batch_stats": (ctypes.c_int, [_VP, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64, _VP, _VP,
                                         _VP, ctypes.c_uint64, _VP]),
    "es_checkpoint_bytes": (ctypes.c_uint64, [_VP]),
    "es_checkpoint_export": (ctypes.c_int, [_VP, _VP, ctypes.c_uint64, _VP, _VP, ctypes.c_uint64]),
    "es_checkpoint_import": (ctypes.c_int, [_VP, _VP, ctypes.c_uint64, _VP, _VP,
                                            ctypes.POINTER(ctypes.c_uint64)]),
    "es_sync": (ctypes.c_int, [_VP]),
    "es_set_option": (ctypes.c_int, [_VP, ctypes.c_char_p, ctypes.c_int64]),
    "es_get_option": (ctypes.c_int, [_VP, ctypes.c_char_p, ctypes.POINTER(ctypes.c_int64)]),
    "es_plan_tiles": (ctypes.c_int, [ctypes.c_uint32, ctypes.POINTER(EsBucketLayout), ctypes.c_uint32,
                                     ctypes.c_uint32, ctypes.POINTER(EsTile), ctypes.c_uint64,
                                     ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_uint64)]),
    "es_plan_swap_in": (ctypes.c_int, [ctypes.c_uint32, ctypes.POINTER(EsSwapOp), ctypes.c_uint64,
                                       ctypes.POINTER(ctypes.c_uint64)]),
    "es_query": (ctypes.c_int, [_VP, ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_uint32),
                                ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_uint32),
                                ctypes.POINTER(ctypes.c_uint64)]),
    "es_last_hip_error": (ctypes.c_int, [_VP]),
    "es_strerror": (ctypes.c_char_p, [ctypes.c_int]),
    "es_version": (ctypes.c_char_p, []),
    # include/es_sched.h
    "es_sched_evaluate": (ctypes.c_int, [ctypes.c_uint32, ctypes.POINTER(ctypes.c_double),
                                         ctypes.POINTER(ctypes.c_uint32), ctypes.POINTER(ctypes.c_uint32),
                                         ctypes.c_uint32, ctypes.c_int, ctypes.POINTER(EsSchedPlan)]),
    "es_sched_best_mapping": (ctypes.c_int, [ctypes.c_uint32, ctypes.POINTER(ctypes.c_double),
                                             ctypes.POINTER(ctypes.c_uint32), ctypes.c_uint32,
                                             ctypes.POINTER(EsSchedPlan)]),
    "es_sched_enumerate": (ctypes.c_int, [ctypes.c_uint32, ctypes.POINTER(ctypes.c_double),
                                          ctypes.POINTER(ctypes.c_uint32), ctypes.c_uint32, ctypes.c_uint32,
                                          ctypes.POINTER(EsSchedPlan), ctypes.POINTER(ctypes.c_uint32)]),
    "es_sched_grouping": (ctypes.c_int, [ctypes.c_uint32, ctypes.POINTER(EsSchedPlan), ctypes.c_uint32,
                                         ctypes.POINTER(ctypes.c_uint32), ctypes.POINTER(ctypes.c_uint32),
                                         ctypes.POINTER(ctypes.c_uint32)]),
}
EXPORTS = tuple(_SIGS)


def lib() -> ctypes.CDLL:
    """The loaded libes.so.  It is built first if there is none or if the one there was built from
    other sources than the tree holds; a library whose compiled-in source hash still differs
    afterwards is refused."""
    global _lib
    if _lib is None:
        _build.build(force=False)
        L = ctypes.CDLL(_build.LIB)
        for name, (res, args) in _SIGS.items():
            fn = getattr(L, name)          # AttributeError if a declared symbol is missing
            fn.restype, fn.argtypes = res, args
        version, want = L.es_version().decode(), _build.source_hash()
        if not version.endswith("src:" + want):
            raise RuntimeError(f"{_build.LIB} is '{version}' but the sources hash to {want}: rebuild it "
                               f"(python -m paper_2208_14228_amd.build)")
        _lib = L
    return _lib


def check(status: int, where: str, h: Optional[int] = None) -> int:
    if status < 0:
        hip = lib().es_last_hip_error(h) if (h and status == ES_EHIP) else 0
        raise EsError(status, where, hip)
    return status


# ---- thin wrappers: one per entry point, same names ---------------------------------

def es_init(n_logical: int, n_params: int, buckets: Sequence[Tuple[int, int]], chunk_align: int,
            state_seg_bytes: Sequence[int] = (), dev_alloc=None, dev_free=None) -> Tuple[int, int]:
    """Returns (status, handle).  ``dev_alloc`` / ``dev_free`` are DEV_ALLOC_FN / DEV_FREE_FN objects
    (or None for hipMalloc); the caller keeps them alive until es_destroy has returned."""
    arr = (EsBucket * max(1, len(buckets)))(*[EsBucket(o, l) for o, l in buckets])
    segs = (ctypes.c_uint64 * max(1, len(state_seg_bytes)))(*state_seg_bytes)
    lay = EsBucketLayout(n_params, len(buckets), arr, chunk_align, len(state_seg_bytes), segs,
                         ctypes.cast(dev_alloc, ctypes.c_void_p) if dev_alloc else None,
                         ctypes.cast(dev_free, ctypes.c_void_p) if dev_free else None, None)
    h = _VP()
    st = lib().es_init(ctypes.byref(h), n_logical, ctypes.byref(lay))
    return st, (h.value or 0)


def es_destroy(h): return lib().es_destroy(h)
def es_set_streams(h, main, ctx, stage): return lib().es_set_streams(h, main, ctx, stage)


def es_set_grouping(h, worker_of_est: Sequence[int], slot_of_est: Sequence[int]) -> int:
    n = len(worker_of_est)
    w = (ctypes.c_uint32 * n)(*worker_of_est)
    s = (ctypes.c_uint32 * n)(*slot_of_est)
    return lib().es_set_grouping(h, (max(worker_of_est) + 1) if n else 0, w, s)


def es_bind_live_state(h, worker: int, live_ptrs: Sequence[int]) -> int:
    arr = (_VP * max(1, len(live_ptrs)))(*live_ptrs)
    return lib().es_bind_live_state(h, worker, arr)


def es_ctx_restore(h, est): return lib().es_ctx_restore(h, est)
def es_ctx_save(h, est): return lib().es_ctx_save(h, est)
def es_ctx_switch(h, est_out, est_in): return lib().es_ctx_switch(h, est_out, est_in)
def es_accumulate(h, est, bucket, d_grad): return lib().es_accumulate(h, est, bucket, d_grad)


def es_accumulate_batch(h, est, buckets: Sequence[int], d_grads: Sequence[int]) -> int:
    n = len(buckets)
    b = (ctypes.c_uint32 * max(1, n))(*buckets)
    g = (_VP * max(1, n))(*d_grads)
    return lib().es_accumulate_batch(h, est, n, b, g)


ES_NO_EST = 0xFFFFFFFF


class Marshalled:
    """Bucket indices and device pointers of one batch as C arrays, built once and handed to
    es_accumulate_batch / es_est_boundary again every global step (marshalling only)."""

    def __init__(self, buckets: Sequence[int], d_grads: Sequence[int]):
        self.n = len(buckets)
        self.b = (ctypes.c_uint32 * max(1, self.n))(*buckets)
        self.g = (_VP * max(1, self.n))(*d_grads)


def es_accumulate_batch_m(h, est, m: Marshalled) -> int:
    return lib().es_accumulate_batch(h, est, m.n, m.b, m.g)


def es_accumulate_many(h, ests: Sequence[int], d_flat_grads: Sequence[int]) -> int:
    n = len(ests)
    e = (ctypes.c_uint32 * max(1, n))(*ests)
    g = (_VP * max(1, n))(*d_flat_grads)
    return lib().es_accumulate_many(h, n, e, g)


def es_est_boundary(h, est_out, est_in, buckets: Sequence[int], d_grads: Sequence[int]) -> int:
    """``est_in`` None or ES_NO_EST: save est_out only."""
    m = Marshalled(buckets, d_grads)
    return lib().es_est_boundary(h, est_out, ES_NO_EST if est_in is None else est_in, m.n, m.b, m.g)


def es_est_boundary_m(h, est_out, est_in, m: Marshalled) -> int:
    return lib().es_est_boundary(h, est_out, ES_NO_EST if est_in is None else est_in, m.n, m.b, m.g)


def es_accumulate_in_place(h, est, d_flat_grad): return lib().es_accumulate_in_place(h, est, d_flat_grad)
def es_grad_slot(h, est, bucket): return lib().es_grad_slot(h, est, bucket) or 0
def es_stage_fence(h): return lib().es_stage_fence(h)


def es_dropout_mask(h, est, state_seg, d_mask, n, p):
    return lib().es_dropout_mask(h, est, state_seg, d_mask, n, p)


def es_ring_order_reduce(h, d_avg): return lib().es_ring_order_reduce(h, d_avg)


def es_sgd_step(h, d_param, d_momentum, d_avg, lr, mu):
    return lib().es_sgd_step(h, d_param, d_momentum, d_avg, lr, mu)


def es_reduce_sgd_step(h, d_param, d_momentum, d_avg, lr, mu):
    return lib().es_reduce_sgd_step(h, d_param, d_momentum, d_avg, lr, mu)


def es_grad_sq_norm(h, d_vec, d_out2): return lib().es_grad_sq_norm(h, d_vec, d_out2)
def es_grad_sq_norm_static(d_vec, n, d_out2, stream=0): return lib().es_grad_sq_norm_static(d_vec, n, d_out2, stream)
def es_clip_sgd_step(h, d_param, d_momentum, d_avg, d_norm2, max_norm, eps, lr, mu):
    return lib().es_clip_sgd_step(h, d_param, d_momentum, d_avg, d_norm2, max_norm, eps, lr, mu)


def es_bn_workspace_floats(n_images, n_channels, n_positions):
    return lib().es_bn_workspace_floats(n_images, n_channels, n_positions)


def es_bn_batch_stats(d_x, n_images, n_channels, n_positions, d_mean, d_var, d_workspace, workspace_floats,
                      stream=0):
    return lib().es_bn_batch_stats(d_x, n_images, n_channels, n_positions, d_mean, d_var, d_workspace,
                                   workspace_floats, stream)


def es_checkpoint_bytes(h): return lib().es_checkpoint_bytes(h)


def es_checkpoint_export(h, host_addr: int, capacity: int, d_param, d_momentum, global_step: int) -> int:
    return lib().es_checkpoint_export(h, host_addr, capacity, d_param, d_momentum, global_step)


def es_checkpoint_import(h, host_addr: int, size: int, d_param, d_momentum) -> Tuple[int, int]:
    """Returns (status, global_step)."""
    step = ctypes.c_uint64()
    st = lib().es_checkpoint_import(h, host_addr, size, d_param, d_momentum, ctypes.byref(step))
    return st, step.value


def es_sync(h): return lib().es_sync(h)
def es_set_option(h, name: str, value: int): return lib().es_set_option(h, name.encode(), value)


def es_get_option(h, name: str) -> Tuple[int, int]:
    v = ctypes.c_int64()
    st = lib().es_get_option(h, name.encode(), ctypes.byref(v))
    return st, v.value


def _layout(n_params, buckets, chunk_align, state_seg_bytes=()):
    arr = (EsBucket * max(1, len(buckets)))(*[EsBucket(o, l) for o, l in buckets])
    segs = (ctypes.c_uint64 * max(1, len(state_seg_bytes)))(*state_seg_bytes)
    lay = EsBucketLayout(n_params, len(buckets), arr, chunk_align, len(state_seg_bytes), segs, None, None, None)
    lay._keep = (arr, segs)
    return lay


def es_plan_tiles(n_logical: int, n_params: int, buckets, chunk_align: int, tile_elems: int,
                  big_unroll: int):
    """Returns (status, n_big, [(offset, len, start_rank), ...])."""
    lay = _layout(n_params, buckets, chunk_align)
    nt, nb = ctypes.c_uint64(), ctypes.c_uint64()
    st = lib().es_plan_tiles(n_logical, ctypes.byref(lay), tile_elems, big_unroll, None, 0,
                             ctypes.byref(nt), ctypes.byref(nb))
    if st:
        return st, 0, []
    out = (EsTile * max(1, nt.value))()
    st = lib().es_plan_tiles(n_logical, ctypes.byref(lay), tile_elems, big_unroll, out, nt.value,
                             ctypes.byref(nt), ctypes.byref(nb))
    return st, nb.value, [(t.offset_elems, t.len_elems, t.start_rank) for t in out[:nt.value]]


def es_plan_swap_in(n_buckets: int):
    """Returns (status, [(kind, bucket, half, wait), ...]) with kind "fill" or "reduce"."""
    n = ctypes.c_uint64()
    st = lib().es_plan_swap_in(n_buckets, None, 0, ctypes.byref(n))
    if st:
        return st, []
    out = (EsSwapOp * max(1, n.value))()
    st = lib().es_plan_swap_in(n_buckets, out, n.value, ctypes.byref(n))
    return st, [("fill" if o.kind == 0 else "reduce", o.bucket, o.half, o.wait) for o in out[:n.value]]


def es_query(h):
    """Returns (status, dict)."""
    P, nb, cb, nw, nt = (ctypes.c_uint64(), ctypes.c_uint32(), ctypes.c_uint64(),
                         ctypes.c_uint32(), ctypes.c_uint64())
    st = lib().es_query(h, ctypes.byref(P), ctypes.byref(nb), ctypes.byref(cb),
                        ctypes.byref(nw), ctypes.byref(nt))
    return st, dict(n_params=P.value, n_buckets=nb.value, ctx_bytes=cb.value,
                    n_workers=nw.value, n_reduce_tiles=nt.value)


def es_last_hip_error(h): return lib().es_last_hip_error(h)
def es_strerror(status): return lib().es_strerror(status).decode()
def es_version(): return lib().es_version().decode()


# ---- include/es_sched.h: host-only planning ------------------------------------------

def _dbl(xs): return (ctypes.c_double * max(1, len(xs)))(*[float(x) for x in xs])
def _u32(xs): return (ctypes.c_uint32 * max(1, len(xs)))(*[int(x) for x in xs])


def _plan_dict(p: EsSchedPlan, n_types: int) -> dict:
    return dict(n_used=tuple(p.n_used[:n_types]), est_per_gpu=tuple(p.est_per_gpu[:n_types]),
                n_gpus=p.n_gpus, n_est=p.n_est, f_overload=p.f_overload, waste=p.waste,
                throughput=p.throughput)


def es_sched_evaluate(capability, n_used, est_per_gpu, max_p: int, waste_reading: int = ES_SCHED_WASTE_PER_GPU):
    """Returns (status, plan dict or None)."""
    out = EsSchedPlan()
    st = lib().es_sched_evaluate(len(capability), _dbl(capability), _u32(n_used), _u32(est_per_gpu),
                                 max_p, waste_reading, ctypes.byref(out))
    return st, (_plan_dict(out, len(capability)) if st == ES_OK else None)


def es_sched_best_mapping(capability, n_used, max_p: int):
    """Returns (status, plan dict or None)."""
    out = EsSchedPlan()
    st = lib().es_sched_best_mapping(len(capability), _dbl(capability), _u32(n_used), max_p, ctypes.byref(out))
    return st, (_plan_dict(out, len(capability)) if st == ES_OK else None)


def es_sched_enumerate(capability, available, max_p: int, top_k: int):
    """Returns (status, [plan dict, ...])."""
    out = (EsSchedPlan * max(1, top_k))()
    n = ctypes.c_uint32()
    st = lib().es_sched_enumerate(len(capability), _dbl(capability), _u32(available), max_p, top_k,
                                  out, ctypes.byref(n))
    return st, ([_plan_dict(out[k], len(capability)) for k in range(n.value)] if st == ES_OK else [])


def es_sched_grouping(n_used, est_per_gpu, max_p: int):
    """Returns (status, n_workers, worker_of_est, slot_of_est)."""
    plan = EsSchedPlan()
    for i, (n, a) in enumerate(zip(n_used, est_per_gpu)):
        plan.n_used[i], plan.est_per_gpu[i] = int(n), int(a)
    wo, so = (ctypes.c_uint32 * max(1, max_p))(), (ctypes.c_uint32 * max(1, max_p))()
    nw = ctypes.c_uint32()
    st = lib().es_sched_grouping(len(n_used), ctypes.byref(plan), max_p, wo, so, ctypes.byref(nw))
    if st != ES_OK:
        return st, 0, [], []
    return st, nw.value, list(wo[:max_p]), list(so[:max_p])
