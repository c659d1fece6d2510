"""An EST job: the torch tensors and streams around one libes handle.

Plumbing only: allocation, pointer marshalling and stream objects.  Every step
of the path (context save/restore, gradient staging, dropout mask, ring-ordered
reduce, SGD update) is a call into libes.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import torch

from . import binding as B


class TorchDeviceMemory:
    """The library's device memory taken from torch's caching allocator (the allocator callbacks
    of es_bucket_layout): every block is a uint8 tensor that lives until the library frees it."""

    def __init__(self, device):
        self.device = device
        self.blocks = {}
        self.alloc_fn = B.DEV_ALLOC_FN(self._alloc)
        self.free_fn = B.DEV_FREE_FN(self._free)

    def _alloc(self, nbytes, _user):
        try:
            t = torch.empty(max(int(nbytes), 1), dtype=torch.uint8, device=self.device)
        except Exception:               # out of memory: the library reports ES_ENOMEM
            return None
        self.blocks[t.data_ptr()] = t
        return t.data_ptr()

    def _free(self, ptr, _user):
        self.blocks.pop(ptr, None)

    @property
    def nbytes(self):
        return sum(t.numel() for t in self.blocks.values())


class ESTJob:
    def __init__(self, n_logical: int, n_params: int, buckets: Sequence[Tuple[int, int]],
                 chunk_align: int, state_seg_bytes: Sequence[int] = (),
                 worker_of_est: Optional[Sequence[int]] = None,
                 slot_of_est: Optional[Sequence[int]] = None,
                 device: str = "cuda:0", use_streams=True, live_alloc=None, torch_memory=True):
        if not torch.cuda.is_available():
            raise RuntimeError("ESTJob needs a GPU: libes has no CPU path")
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.N = n_logical
        self.P = n_params
        self.buckets = list(buckets)
        self.seg_bytes = list(state_seg_bytes)
        # torch owns the device memory of the job (gradient slots included) unless told otherwise
        self.memory = TorchDeviceMemory(self.device) if torch_memory else None
        st, self.h = B.es_init(n_logical, n_params, self.buckets, chunk_align, self.seg_bytes,
                               self.memory.alloc_fn if self.memory else None,
                               self.memory.free_fn if self.memory else None)
        B.check(st, "es_init")
        self.worker_of = list(worker_of_est) if worker_of_est is not None else [0] * n_logical
        self.slot_of = list(slot_of_est) if slot_of_est is not None else list(range(n_logical))
        # es_init starts with one worker that holds every EST in rank order: only another grouping
        # needs a regrouping (which holds both sets of gradient slots while it runs)
        if self.worker_of != [0] * n_logical or self.slot_of != list(range(n_logical)):
            B.check(B.es_set_grouping(self.h, self.worker_of, self.slot_of), "es_set_grouping", self.h)
        self.main = self.ctx = self.stage = None
        # use_streams: True / "three" = separate main, ctx and stage streams (staging and context
        # traffic overlap with the EST's compute); "two" = main (also small-state context) + stage;
        # "one" = a single stream for everything (strictly in order, no events); False = null stream
        if use_streams == "one":
            self.main = self.ctx = self.stage = torch.cuda.Stream(self.device)
        elif use_streams == "two":
            self.main = self.ctx = torch.cuda.Stream(self.device)
            self.stage = torch.cuda.Stream(self.device)
        elif use_streams:
            self.main = torch.cuda.Stream(self.device)
            self.ctx = torch.cuda.Stream(self.device)
            self.stage = torch.cuda.Stream(self.device)
        if self.main is not None:
            B.check(B.es_set_streams(self.h, self.main.cuda_stream, self.ctx.cuda_stream,
                                     self.stage.cuda_stream), "es_set_streams", self.h)
        # live small-state tensors: one set per worker, every segment its own allocation
        # (live_alloc(nbytes) -> uint8 tensor lets a caller choose placement/alignment)
        self._live_alloc = live_alloc or (lambda nb: torch.full((nb,), 0xAB, dtype=torch.uint8,
                                                                 device=self.device))
        self.live: List[List[torch.Tensor]] = []
        self._bind_live()
        self.p = torch.zeros(max(n_params, 1), dtype=torch.float32, device=self.device)[:n_params]
        self.v = torch.zeros_like(self.p)
        self.avg = torch.zeros_like(self.p)

    def _bind_live(self):
        self.live = []
        for w in range(max(self.worker_of) + 1):
            segs = [self._live_alloc(nb) for nb in self.seg_bytes]
            self.live.append(segs)
            if segs:
                B.check(B.es_bind_live_state(self.h, w, [t.data_ptr() for t in segs]),
                        "es_bind_live_state", self.h)

    def set_grouping(self, worker_of_est, slot_of_est):
        B.check(B.es_set_grouping(self.h, list(worker_of_est), list(slot_of_est)),
                "es_set_grouping", self.h)
        self.worker_of, self.slot_of = list(worker_of_est), list(slot_of_est)
        self._bind_live()

    def stream_ctx(self):
        return torch.cuda.stream(self.main) if self.main is not None else torch.cuda.stream(None)

    # ---- forwards -------------------------------------------------------------
    def ctx_restore(self, e): B.check(B.es_ctx_restore(self.h, e), "es_ctx_restore", self.h)
    def ctx_save(self, e): B.check(B.es_ctx_save(self.h, e), "es_ctx_save", self.h)
    def ctx_switch(self, a, b): B.check(B.es_ctx_switch(self.h, a, b), "es_ctx_switch", self.h)

    def accumulate(self, e, b, grad: torch.Tensor):
        assert grad.dtype == torch.float32 and grad.is_contiguous() and grad.numel() == self.buckets[b][1]
        B.check(B.es_accumulate(self.h, e, b, grad.data_ptr()), "es_accumulate", self.h)

    def accumulate_batch(self, e, buckets, grads):
        for b, g in zip(buckets, grads):
            assert g.dtype == torch.float32 and g.is_contiguous() and g.numel() == self.buckets[b][1]
        B.check(B.es_accumulate_batch(self.h, e, list(buckets), [g.data_ptr() for g in grads]),
                "es_accumulate_batch", self.h)

    def accumulate_in_place(self, e, flat_grad: torch.Tensor):
        assert flat_grad.dtype == torch.float32 and flat_grad.is_contiguous() and flat_grad.numel() == self.P
        B.check(B.es_accumulate_in_place(self.h, e, flat_grad.data_ptr()), "es_accumulate_in_place", self.h)

    def dropout_mask(self, e, seg, mask: torch.Tensor, p: float):
        assert mask.dtype == torch.uint8 and mask.is_contiguous()
        B.check(B.es_dropout_mask(self.h, e, seg, mask.data_ptr(), mask.numel(), p),
                "es_dropout_mask", self.h)

    def ring_order_reduce(self):
        B.check(B.es_ring_order_reduce(self.h, self.avg.data_ptr()), "es_ring_order_reduce", self.h)

    def sgd_step(self, lr, mu):
        B.check(B.es_sgd_step(self.h, self.p.data_ptr(), self.v.data_ptr(), self.avg.data_ptr(), lr, mu),
                "es_sgd_step", self.h)

    def reduce_sgd_step(self, lr, mu, store_avg=True):
        B.check(B.es_reduce_sgd_step(self.h, self.p.data_ptr(), self.v.data_ptr(),
                                     self.avg.data_ptr() if store_avg else 0, lr, mu),
                "es_reduce_sgd_step", self.h)

    def checkpoint_export(self, global_step: int):
        """Host blob (numpy uint8) holding all EST contexts, parameters and momentum."""
        import numpy as np
        n = B.es_checkpoint_bytes(self.h)
        blob = np.empty(n, dtype=np.uint8)
        B.check(B.es_checkpoint_export(self.h, blob.ctypes.data, n, self.p.data_ptr(), self.v.data_ptr(),
                                       global_step), "es_checkpoint_export", self.h)
        return blob

    def checkpoint_import(self, blob) -> int:
        st, step = B.es_checkpoint_import(self.h, blob.ctypes.data, blob.size, self.p.data_ptr(),
                                          self.v.data_ptr())
        B.check(st, "es_checkpoint_import", self.h)
        return step

    def sync(self): B.check(B.es_sync(self.h), "es_sync", self.h)
    def set_option(self, name, value): B.check(B.es_set_option(self.h, name, value), "es_set_option", self.h)

    def live_of(self, e) -> List[torch.Tensor]:
        return self.live[self.worker_of[e]]

    def close(self):
        if self.h:
            B.es_destroy(self.h)
            self.h = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
