#!/usr/bin/env python3
"""Benchmark of the EST step on one MI355X.

One *step* = one global step of the whole hot path on synthetic gradients that
are already resident in HBM: for every EST its context restore (or the fused
switch from the previous EST of its worker), its dropout mask where the
configuration has an RNG context, the staging of all its gradient buckets into
its context slot, its context save; then the ring-ordered N-way reduce and the
SGD-momentum update (one fused kernel by default, --split times them as two).

Prints ONE JSON line.  The headline workload is configuration 5 (GPT-2-medium
shaped, N = 64, 90.8 GB of gradient slots), the largest one: `value` is its
whole-step throughput on algorithmic bytes, `roofline` prices its reduce kernel
against the HBM peak from HIP-event timings taken inside the timed region
(mean, median and min), `cpu_baseline` is the CPU oracle (the message-passing
ring simulator, streamed bucket by bucket) timed on one host core for one full
global step of the same workload, and `zero_ulp` says whether every bit of the
GPU's parameters and momentum after that step equals the oracle's.  `configs`
carries the same measurements, shorter, for all five configurations.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, vendor figure
CACHE_FIT_BYTES = 284 << 20     # parameters + momentum up to this size stay cacheable by default


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=5, help="headline configuration 1..5 (default: the largest)")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the short measurements of the other configurations (`configs` array)")
    ap.add_argument("--split", action="store_true", help="reduce and SGD as two kernels")
    ap.add_argument("--per-bucket", action="store_true",
                    help="stage with one es_accumulate launch per bucket instead of es_accumulate_batch")
    ap.add_argument("--separate-calls", action="store_true",
                    help="an EST boundary as two launches (es_ctx_switch, then es_accumulate_batch) instead of "
                         "the single es_est_boundary launch")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle legs (no zero_ulp either)")
    ap.add_argument("--no-switch", action="store_true", help="skip the EST-switch timing")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip every leg but the timed step (no cache-swept reduce, in-place, zero-copy, graph, "
                         "norm, checkpoint, host-swap, ceilings)")
    ap.add_argument("--streams", choices=["one", "two", "three"], default="one",
                    help="one in-order stream (default: nothing to overlap with in this benchmark) or "
                         "separate main/ctx/stage streams wired with events")
    ap.add_argument("--host-slots", action="store_true",
                    help="memory-pressure mode: gradient slots in pinned host memory (host-link bound)")
    ap.add_argument("--standin", type=int, default=0,
                    help="side length of a bf16 matmul every EST runs on main before its boundary call: a "
                         "compute-bound stand-in for forward/backward that staging on its own stream can "
                         "overlap with (0 = none; the default line carries this experiment as staging_overlap)")
    ap.add_argument("--ceilings", action="store_true",
                    help="separate experiment: what this box's HBM gives the library's plain copy and "
                         "pure-read kernels on 1 GiB (prints its own JSON line)")
    ap.add_argument("--hip-malloc", action="store_true",
                    help="the library allocates its device memory with hipMalloc instead of taking it from "
                         "torch's caching allocator through the allocator callbacks")
    ap.add_argument("--opt", action="append", default=[], help="library option name=value")
    return ap.parse_args()


def stats_ms(xs):
    return {"mean": round(statistics.fmean(xs), 4), "median": round(statistics.median(xs), 4),
            "min": round(min(xs), 4), "n": len(xs)}


def est_switch_us(torch, reps=200):
    """EST switch latency on the BatchNorm context of the ResNet-50 configuration
    (106 live tensors, 212,480 bytes) plus a 16-byte RNG state: the fused
    save+restore kernel, and a save followed by a restore, per stream mode."""
    from paper_2208_14228_amd.job import ESTJob
    from workloads import shapes
    segs = [16] + [4 * c for c in shapes.resnet50_bn_channels() for _ in (0, 1)]
    out = {"ctx_bytes": sum(segs), "live_tensors": len(segs)}
    for mode in ("one", "two", "three"):
        job = ESTJob(4, 1024, [(0, 1024)], 4, segs, use_streams=mode)
        try:
            for e in range(4):
                job.ctx_save(e)
            job.sync()

            def timed(fn):
                for i in range(10):
                    fn(i)
                job.sync()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(job.ctx)
                t0 = time.perf_counter()
                for i in range(reps):
                    fn(i)
                e1.record(job.ctx)
                job.sync()
                torch.cuda.synchronize()
                wall = (time.perf_counter() - t0) / reps * 1e6
                return e0.elapsed_time(e1) / reps * 1e3, wall

            def pair(i):
                job.ctx_save(i % 4)
                job.ctx_restore((i + 1) % 4)

            gpu, wall = timed(lambda i: job.ctx_switch(i % 4, (i + 1) % 4))
            gpu2, wall2 = timed(pair)
            out[f"streams_{mode}"] = {"switch_us": round(gpu, 3), "switch_wall_us": round(wall, 3),
                                      "save_then_restore_us": round(gpu2, 3),
                                      "save_then_restore_wall_us": round(wall2, 3)}
        finally:
            job.close()
    return out


def ceilings():
    """Plain streaming rates on this machine, measured with the library's own kernels: the staging
    copy (k_copy_f4, read + write) and the norm's first stage (k_sq_partials, read only) on a
    1 GiB vector.  Context for the roofline fractions; the vendor peak stays the denominator."""
    import torch

    from paper_2208_14228_amd import binding as B
    from paper_2208_14228_amd.job import ESTJob

    P = 1 << 28
    job = ESTJob(1, P, [(0, P)], 4, use_streams="one")
    src = torch.ones(P, device="cuda:0")
    out2 = torch.zeros(2, device="cuda:0")
    slot = B.es_grad_slot(job.h, 0, 0)

    def timed(fn, reps=10):
        for _ in range(3):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(job.main)
        for _ in range(reps):
            fn()
        e1.record(job.main)
        job.sync(); torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    def copy():
        B.es_accumulate(job.h, 0, 0, src.data_ptr())
        job.ring_order_reduce()    # N = 1: ends the step so the bucket can be staged again

    # the N = 1 reduce is itself a 1 GiB copy (read slot, write avg): time it alone and subtract
    B.es_accumulate(job.h, 0, 0, src.data_ptr()); job.ring_order_reduce(); job.sync()

    def reduce_only():
        B.es_accumulate(job.h, 0, 0, slot)
        job.ring_order_reduce()

    t_both, t_red = timed(copy), timed(reduce_only)
    t_norm = timed(lambda: B.es_grad_sq_norm(job.h, src.data_ptr(), out2.data_ptr()))
    gb = 4 * P / 1e9
    res = {"note": "plain streaming rates of the library's own kernels on 1 GiB: what this box's HBM "
                   "delivers (the vendor peak stays the denominator of every frac)",
           "copy_read_plus_write_GBps": round(2 * gb / ((t_both - t_red) * 1e-3), 1),
           "n1_reduce_read_plus_write_GBps": round(2 * gb / (t_red * 1e-3), 1),
           "norm_read_only_pass_GBps": round(gb / (t_norm * 1e-3), 1), "hbm_peak_GBps": HBM_PEAK_GBPS}
    job.close()
    del src
    torch.cuda.empty_cache()
    return res


class OracleLeg:
    """The CPU oracle on one full global step of a configuration, streamed bucket by bucket:
    the N gradient rows of a bucket are copied from the device into one pinned host buffer, the
    message-passing ring simulator runs on them in place, /N, then SGD-momentum on that bucket's
    slice of the parameters; the result is compared bit for bit with the GPU's.  Only the
    oracle's own calls are timed (the copies from the device are not CPU-baseline work)."""

    def __init__(self, torch, n_floats):
        self.torch = torch
        self.pin = torch.empty(n_floats, dtype=torch.float32, pin_memory=True)

    def run(self, cfg, src, p0, gpu_p, gpu_v, all_cores):
        import numpy as np

        import oracle
        torch = self.torch
        lay, N = cfg.layout, cfg.n_logical
        oracle.use_all_cores(all_cores)
        oracle.lib()
        secs, same = 0.0, True
        for off, L in lay.buckets:
            if L == 0:
                continue
            rows = self.pin[:N * L].view(N, L)
            for r in range(N):
                rows[r].copy_(src[r][off:off + L], non_blocking=True)
            p = p0[off:off + L].cpu().numpy().copy()
            torch.cuda.synchronize()
            v = np.zeros(L, dtype=np.float32)
            ranks = rows.numpy()
            t0 = time.perf_counter()
            avg = oracle.ring_order_reduce(ranks, cfg.chunk_align, clobber=True)
            oracle.sgd_momentum(p, v, avg, cfg.lr, cfg.momentum)
            secs += time.perf_counter() - t0
            gp = gpu_p[off:off + L].cpu().numpy()
            gv = gpu_v[off:off + L].cpu().numpy()
            same = same and bool(np.array_equal(gp.view(np.uint32), p.view(np.uint32)) and
                                 np.array_equal(gv.view(np.uint32), v.view(np.uint32)))
        oracle.use_all_cores(False)
        return secs, same


def measure(torch, a, cid, headline, oracle_leg):
    """All measurements of one configuration; the short form (fewer steps, no variant legs)
    unless ``headline``."""
    from paper_2208_14228_amd import binding as B
    from paper_2208_14228_amd.job import ESTJob
    from workloads import configs, synth

    cfg = configs.config(cid)
    lay, N, P = cfg.layout, cfg.n_logical, cfg.layout.n_params
    g = cfg.groupings[0]
    dev = "cuda:0"
    print(f"[bench] config {cid} ({'headline' if headline else 'short form'})", file=sys.stderr, flush=True)
    steps = a.steps if headline else min(a.steps, 10)
    warmup = a.warmup if headline else min(a.warmup, 3)
    segs = []
    if cfg.dropout:
        segs.append(16)
    segs += [4 * c for c in cfg.bn_channels for _ in (0, 1)]

    job = ESTJob(N, P, lay.buckets, cfg.chunk_align, segs, g.worker_of_est, g.slot_of_est, dev,
                 use_streams=a.streams, torch_memory=not a.hip_malloc)
    if a.host_slots:
        job.set_option("host_slots", 1)
        job.set_grouping(g.worker_of_est, g.slot_of_est)
    for kv in a.opt:
        k, v = kv.split("=")
        job.set_option(k, int(v))
    opts = {k: B.es_get_option(job.h, k)[1] for k in
            ("reduce_tile_elems", "reduce_unroll", "reduce_rank_batch", "nontemporal", "nontemporal_pv",
             "reduce_big_unroll", "reduce_big_rank_batch")}

    # synthetic inputs, resident in HBM before anything is timed
    src = []
    for e in range(N):
        t = torch.empty(P, dtype=torch.float32, device=dev)
        for b, (off, ln) in enumerate(lay.buckets):
            synth.gradient(lay, b, cfg.seed, 0, e, dev, out=t[off:off + ln])
        src.append(t)
    p0 = synth.params(lay, cfg.seed, dev)
    mask = torch.empty(32 * 128 * 768, dtype=torch.uint8, device=dev) if cfg.dropout else None
    # optional compute-bound stand-in for an EST's forward+backward (a bf16 matmul on main): what the
    # staging copy on its own stream can overlap with
    standin = None
    if getattr(a, "standin", 0):
        standin = [torch.randn(a.standin, a.standin, device=dev, dtype=torch.bfloat16) for _ in range(2)]
        standin.append(torch.empty(a.standin, a.standin, device=dev, dtype=torch.bfloat16))
    for e in range(N):
        if segs:
            job.ctx_save(e)
    job.sync()
    torch.cuda.synchronize()

    fused = not a.split
    all_buckets = list(range(lay.n_buckets))
    src_ptrs = [[src[e].data_ptr() + 4 * off for off, _ in lay.buckets] for e in range(N)]
    marshalled = [B.Marshalled(all_buckets, src_ptrs[e]) for e in range(N)]
    one_launch = not (a.per_bucket or a.separate_calls)

    def events(n):
        return [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]

    ev_r, ev_s, ev_c = events(steps), events(steps), events(steps)

    # EST e takes over the worker's live state: the first EST of a worker is restored, later
    # ones switch in with the fused save+restore kernel, the last one is saved at the end
    sched = g.schedule()
    prev_of = {e: (sched[k - 1] if k and g.worker_of_est[sched[k - 1]] == g.worker_of_est[e] else None)
               for k, e in enumerate(sched)}
    last_of_worker = [e for k, e in enumerate(sched)
                      if k + 1 == len(sched) or g.worker_of_est[sched[k + 1]] != g.worker_of_est[e]]

    next_of = {p: e for e, p in prev_of.items() if p is not None}

    def enter(e, fused_boundary=False):
        if not segs:
            return
        if prev_of[e] is None:
            job.ctx_restore(e)
        elif not fused_boundary:              # else the previous EST's boundary launch has switched it in
            job.ctx_switch(prev_of[e], e)

    def leave(fused_boundary=False):
        if segs and not fused_boundary:       # else each worker's last boundary launch has saved it
            for e in last_of_worker:
                job.ctx_save(e)

    def finish(i=None):
        if i is not None:
            ev_c[i][1].record(job.stage)
            B.es_stage_fence(job.h)
            ev_r[i][0].record(job.main)
        if fused:
            job.reduce_sgd_step(cfg.lr, cfg.momentum, store_avg=False)
            if i is not None:
                ev_r[i][1].record(job.main)
        else:
            job.ring_order_reduce()
            if i is not None:
                ev_r[i][1].record(job.main)
                ev_s[i][0].record(job.main)
            job.sgd_step(cfg.lr, cfg.momentum)
            if i is not None:
                ev_s[i][1].record(job.main)

    def step(i=None):
        if i is not None:
            if job.stage is not job.main:
                job.stage.wait_stream(job.main)  # the interval below must not include the previous reduce
            ev_c[i][0].record(job.stage)
        for e in sched:
            enter(e, one_launch)
            if mask is not None:
                job.dropout_mask(e, 0, mask, configs.DROPOUT_P)
            if standin is not None:
                with torch.cuda.stream(job.main):
                    torch.mm(standin[0], standin[1], out=standin[2])
            if one_launch:                    # stage e, save e, restore the worker's next EST: one launch
                B.es_est_boundary_m(job.h, e, next_of.get(e), marshalled[e])
            elif a.per_bucket:
                for b, (off, ln) in enumerate(lay.buckets):
                    B.es_accumulate(job.h, e, b, src[e].data_ptr() + 4 * off)
            else:
                B.es_accumulate_batch_m(job.h, e, marshalled[e])
        leave(one_launch)
        finish(i)

    # ---- one step on the GPU from (p0, v = 0), kept for the bit check against the oracle ----
    cpu = cpu_all = zero_ulp = None
    if not a.no_cpu:
        job.p.copy_(p0); job.v.zero_()
        torch.cuda.synchronize()
        step()
        job.sync(); torch.cuda.synchronize()
        gpu_p, gpu_v = job.p.clone(), job.v.clone()
        cpu_bytes = (N + 1) * 4 * P + 5 * 4 * P
        sample = (f"one full global step of config {cid}: ring all-reduce simulation of all {lay.n_buckets} "
                  f"buckets among {N} ranks, streamed bucket by bucket, /N, SGD-momentum; bytes counted as "
                  f"(N+1)*4P + 5*4P; gradient staging and the copies from the device not included")
        print(f"[bench] config {cid}: CPU oracle, one core", file=sys.stderr, flush=True)
        dt, same1 = oracle_leg.run(cfg, src, p0, gpu_p, gpu_v, all_cores=False)
        print(f"[bench] config {cid}: CPU oracle, all cores", file=sys.stderr, flush=True)
        cpu = {"value": round(cpu_bytes / dt / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "seconds": round(dt, 3), "sample": sample}
        dt, same2 = oracle_leg.run(cfg, src, p0, gpu_p, gpu_v, all_cores=True)
        threads = int(os.environ.get("OMP_NUM_THREADS") or os.cpu_count() or 1)
        cpu_all = {"value": round(cpu_bytes / dt / 1e9, 3), "unit": "GB/s", "cores": threads,
                   "kind": "oracle, same source built with -fopenmp (threads over the ring's ranks)",
                   "seconds": round(dt, 3), "sample": sample}
        zero_ulp = bool(same1 and same2)
        del gpu_p, gpu_v

    # ---- timed region ----
    print(f"[bench] config {cid}: timed steps", file=sys.stderr, flush=True)
    job.p.copy_(p0); job.v.zero_()
    torch.cuda.synchronize()
    for _ in range(warmup):
        step()
    job.sync(); torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    job.sync(); torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_step = dt / steps * 1e3

    ctx_bytes = sum(segs)
    bytes_stage = 2 * N * 4 * P
    bytes_reduce = (N + 4) * 4 * P if fused else (N + 1) * 4 * P
    bytes_sgd = 0 if fused else 5 * 4 * P
    bytes_ctx = 2 * N * ctx_bytes + (N * mask.numel() if mask is not None else 0)
    total = bytes_stage + bytes_reduce + bytes_sgd + bytes_ctx

    red = [x.elapsed_time(y) for x, y in ev_r]
    stg = [x.elapsed_time(y) for x, y in ev_c]
    sgd = [x.elapsed_time(y) for x, y in ev_s] if not fused else None
    red_ms = statistics.fmean(red)
    stage_ms = statistics.fmean(stg)
    red_gbps = bytes_reduce / (red_ms * 1e-3) / 1e9
    pv_cacheable = opts["nontemporal_pv"] == 0 and fused
    kname = ("k_ring_reduce_big" if opts["reduce_big_unroll"] else "k_ring_reduce") + (" (fused SGD)" if fused else "")

    res = {
        "config": cid,
        "workload": f"config {cid}: {cfg.name}-shaped gradient set, N={N} ESTs, P={P} fp32 in "
                    f"{lay.n_buckets} DDP buckets, grouping {g.name}",
        "n_logical": N, "n_params": P, "n_buckets": lay.n_buckets, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_step, 4),
        "step_GBps": round(total / dt * steps / 1e9, 2),
        "step_frac": round(total / dt * steps / 1e9 / HBM_PEAK_GBPS, 4),
        "step_bytes": {"staging": bytes_stage, "reduce": bytes_reduce, "sgd": bytes_sgd,
                       "context": bytes_ctx, "total": total},
        "reduce": {"kernel": kname, "bytes_per_launch": bytes_reduce, "launch_ms": stats_ms(red),
                   "achieved": round(red_gbps, 1), "unit": "GB/s", "frac": round(red_gbps / HBM_PEAK_GBPS, 4),
                   "frac_at_min": round(bytes_reduce / (min(red) * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                   "memory": ("Infinity-Cache-assisted: parameters and momentum (4 of the N+4 units) are left "
                              "cacheable and can come back from the 256 MB cache, not from HBM"
                              if pv_cacheable else "all units stream from and to HBM")},
        "staging": {"kernel": "k_copy_f4" if a.per_bucket else ("k_est_boundary" if one_launch else "k_copy_runs"),
                    "launches_per_step": N * sum(1 for _, ln in lay.buckets if ln) if a.per_bucket else N,
                    "bytes_per_step": bytes_stage, "stream_ms_per_step": stats_ms(stg),
                    "includes": ("each launch also saves the EST's small state and restores the next EST's; "
                                 if one_launch else "the per-EST context switches are launches of their own "
                                 "between the copies; ") + "the dropout-mask launches sit between the copies too",
                    "achieved": round(bytes_stage / (stage_ms * 1e-3) / 1e9, 1), "unit": "GB/s",
                    "frac": round(bytes_stage / (stage_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)},
        "context_bytes_per_est": ctx_bytes, "mask_bytes_per_est": mask.numel() if mask is not None else 0,
        "zero_ulp": zero_ulp, "cpu_baseline": cpu, "cpu_baseline_all_cores": cpu_all,
        "options": opts,
    }
    if sgd is not None:
        res["sgd"] = {"kernel": "k_sgd", "launch_ms": stats_ms(sgd),
                      "achieved": round(bytes_sgd / (statistics.fmean(sgd) * 1e-3) / 1e9, 1), "unit": "GB/s"}

    # ---- the reduce with nothing in the Infinity Cache: a 1 GiB fill sweeps the cache before every
    # launch.  Only where parameters and momentum would fit it; both cache policies. ----
    slot_ptrs = [[B.es_grad_slot(job.h, e, b) for b in all_buckets] for e in range(N)]
    slot_m = [B.Marshalled(all_buckets, slot_ptrs[e]) for e in range(N)]
    if fused and 2 * 4 * P <= CACHE_FIT_BYTES and not a.host_slots and not a.no_extras:
        sweep = torch.empty(1 << 28, dtype=torch.float32, device=dev)
        cold = {}
        for nt_pv in (0, 1):
            job.set_option("nontemporal_pv", nt_pv)
            ev = events(steps)
            for i in range(-2, steps):
                for e in sched:                                   # gradients stay where they are in the slots
                    B.es_accumulate_batch_m(job.h, e, slot_m[e])
                with torch.cuda.stream(job.main):
                    sweep.fill_(1.0)
                if i >= 0:
                    ev[i][0].record(job.main)
                job.reduce_sgd_step(cfg.lr, cfg.momentum, store_avg=False)
                if i >= 0:
                    ev[i][1].record(job.main)
            job.sync(); torch.cuda.synchronize()
            ms = [x.elapsed_time(y) for x, y in ev]
            gb = bytes_reduce / (statistics.fmean(ms) * 1e-3) / 1e9
            cold["streaming_pv" if nt_pv else "cacheable_pv"] = {
                "launch_ms": stats_ms(ms), "achieved": round(gb, 1), "unit": "GB/s",
                "frac": round(gb / HBM_PEAK_GBPS, 4)}
        job.set_option("nontemporal_pv", opts["nontemporal_pv"])
        res["reduce_hbm_only"] = {
            "note": "the same reduce launched right after a 1 GiB fill has swept the Infinity Cache, so that "
                    "every one of its (N+4)*4P bytes moves to or from HBM; cacheable_pv = the default policy "
                    "at this size, streaming_pv = option nontemporal_pv=1", **cold}
        del sweep

    # ---- the two halves as kernels of their own: the reduce alone ((N+1)*4P bytes: N gradient
    # sets read, the average written) and the update alone (5*4P bytes) ----
    if fused and not a.no_extras and not a.host_slots:
        n_split = min(steps, 10)
        ev_a, ev_b = events(n_split), events(n_split)
        for i in range(-2, n_split):
            for e in sched:                                       # gradients stay where they are in the slots
                B.es_accumulate_batch_m(job.h, e, slot_m[e])
            if i >= 0:
                ev_a[i][0].record(job.main)
            job.ring_order_reduce()
            if i >= 0:
                ev_a[i][1].record(job.main)
                ev_b[i][0].record(job.main)
            job.sgd_step(cfg.lr, cfg.momentum)
            if i >= 0:
                ev_b[i][1].record(job.main)
        job.sync(); torch.cuda.synchronize()
        ms_a = [x.elapsed_time(y) for x, y in ev_a]
        ms_b = [x.elapsed_time(y) for x, y in ev_b]
        gb_a = (N + 1) * 4 * P / (statistics.fmean(ms_a) * 1e-3) / 1e9
        gb_b = 5 * 4 * P / (statistics.fmean(ms_b) * 1e-3) / 1e9
        res["reduce_alone"] = {"kernel": kname.replace(" (fused SGD)", ""), "bytes_per_launch": (N + 1) * 4 * P,
                               "launch_ms": stats_ms(ms_a), "achieved": round(gb_a, 1), "unit": "GB/s",
                               "frac": round(gb_a / HBM_PEAK_GBPS, 4)}
        res["sgd_alone"] = {"kernel": "k_sgd", "bytes_per_launch": 5 * 4 * P, "launch_ms": stats_ms(ms_b),
                            "achieved": round(gb_b, 1), "unit": "GB/s", "frac": round(gb_b / HBM_PEAK_GBPS, 4),
                            "memory": ("the averaged gradient the reduce has just written, parameters and momentum "
                                       "can come from the Infinity Cache at this size" if 3 * 4 * P <= CACHE_FIT_BYTES
                                       else "streams from and to HBM")}

    if not a.no_extras:
        def timed_wall(fn):
            for _ in range(warmup):
                fn()
            job.sync(); torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                fn()
            job.sync(); torch.cuda.synchronize()
            return (time.perf_counter() - t0) / steps * 1e3

        # the same step when the EST's backward writes its buckets straight into the slots
        # (es_grad_slot): staging degenerates to marking the buckets present
        def step_zero_copy():
            for e in sched:
                enter(e)
                if mask is not None:
                    job.dropout_mask(e, 0, mask, configs.DROPOUT_P)
                B.es_accumulate_batch_m(job.h, e, slot_m[e])
            leave()
            finish()

        # the paper's own flow (section 5.1.3): the last EST a worker runs is not staged, the
        # reduce reads its gradients where backward left them
        def step_in_place_last():
            for e in sched:
                enter(e)
                if mask is not None:
                    job.dropout_mask(e, 0, mask, configs.DROPOUT_P)
                if e in last_of_worker:
                    B.es_accumulate_in_place(job.h, e, src[e].data_ptr())
                else:
                    B.es_accumulate_batch_m(job.h, e, marshalled[e])
            leave()
            finish()

        # several ESTs' gradients resident at once (one EST of each worker that shares the GPU, or
        # buffers not reused yet): 16 ESTs staged per launch by es_accumulate_many
        flat_ptrs = [src[e].data_ptr() for e in range(N)]

        def step_many():
            for e in sched:
                enter(e)
                if mask is not None:
                    job.dropout_mask(e, 0, mask, configs.DROPOUT_P)
            leave()
            B.es_accumulate_many(job.h, sched, [flat_ptrs[e] for e in sched])
            finish()

        ms_many = timed_wall(step_many)
        res["staged_16_per_launch_step"] = {
            "note": "all ESTs' gradients resident until the end of the step and staged 16 per launch "
                    "(es_accumulate_many)", "ms_per_step": round(ms_many, 4),
            "value": round(total / (ms_many * 1e-3) / 1e9, 2), "unit": "GB/s"}

        ms_ip = timed_wall(step_in_place_last)
        res["in_place_last_step"] = {
            "note": "each worker's last EST is not staged: the reduce reads its gradients in place "
                    "(es_accumulate_in_place)", "ms_per_step": round(ms_ip, 4),
            "value": round((total - bytes_stage * len(last_of_worker) // N) / (ms_ip * 1e-3) / 1e9, 2),
            "unit": "GB/s"}
        if a.streams == "one":
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=job.main):
                step()
            ms_graph = timed_wall(graph.replay)
            res["graph_step"] = {"note": "the same step captured into a HIP graph and replayed",
                                 "ms_per_step": round(ms_graph, 4),
                                 "value": round(total / (ms_graph * 1e-3) / 1e9, 2), "unit": "GB/s"}
            del graph
        ms_zc = timed_wall(step_zero_copy)
        res["zero_copy_step"] = {"note": "gradients produced directly in the slots (es_grad_slot), no staging copy",
                                 "ms_per_step": round(ms_zc, 4),
                                 "value": round((total - bytes_stage) / (ms_zc * 1e-3) / 1e9, 2), "unit": "GB/s"}

    if headline and not a.no_extras:
        # fixed-tree global norm of a vector of the job's size (one read of 4P bytes)
        out2 = torch.zeros(2, device=dev)
        for _ in range(3):
            B.es_grad_sq_norm(job.h, job.p.data_ptr(), out2.data_ptr())
        n0, n1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n0.record(job.main)
        for _ in range(steps):
            B.es_grad_sq_norm(job.h, job.p.data_ptr(), out2.data_ptr())
        n1.record(job.main)
        job.sync(); torch.cuda.synchronize()
        norm_ms = n0.elapsed_time(n1) / steps
        res["grad_sq_norm"] = {"note": "fixed-tree global norm (k_sq_partials + k_sq_final), 4P bytes read",
                               "avg_ms": round(norm_ms, 4),
                               "achieved": round(4 * P / (norm_ms * 1e-3) / 1e9, 1), "unit": "GB/s",
                               "frac": round(4 * P / (norm_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}

        # the update with the gradient clipped by that norm (coefficient formed on the device)
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for i in range(-2, steps):
            if i == 0:
                c0.record(job.main)
            B.es_clip_sgd_step(job.h, job.p.data_ptr(), job.v.data_ptr(), job.avg.data_ptr(), out2.data_ptr(),
                               1.0, 1e-6, cfg.lr, cfg.momentum)
        c1.record(job.main)
        job.sync(); torch.cuda.synchronize()
        clip_ms = c0.elapsed_time(c1) / steps
        res["clip_sgd_step"] = {"note": "k_sgd_clip: update with the averaged gradient clipped by its fixed-tree "
                                        "norm, 5*4P bytes", "avg_ms": round(clip_ms, 4),
                                "achieved": round(20 * P / (clip_ms * 1e-3) / 1e9, 1), "unit": "GB/s",
                                "frac": round(20 * P / (clip_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}

        # BatchNorm batch statistics along the fixed tree, on the activation shape of ResNet-50's first
        # BatchNorm layer at batch 32 (32 x 64 x 112 x 112 fp32 = 103 MB; two passes over it)
        bn_shape = (32, 64, 112 * 112)
        xbn = torch.randn(bn_shape, device=dev)
        nws = B.es_bn_workspace_floats(*bn_shape)
        ws = torch.empty(nws, device=dev)
        mv = torch.empty(2, 64, device=dev)
        torch.cuda.synchronize()
        b0, b1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for i in range(-2, steps):
            if i == 0:
                b0.record(job.main)
            B.es_bn_batch_stats(xbn.data_ptr(), *bn_shape, mv[0].data_ptr(), mv[1].data_ptr(), ws.data_ptr(), nws,
                                job.main.cuda_stream)
        b1.record(job.main)
        job.sync(); torch.cuda.synchronize()
        bn_ms = b0.elapsed_time(b1) / steps
        bn_bytes = 2 * 4 * xbn.numel()
        res["bn_batch_stats"] = {"note": "k_bn_partials + k_bn_final twice (mean, then variance) on 32x64x112x112 "
                                         "fp32; bytes = two reads of the activations (the second can come from "
                                         "the Infinity Cache: 103 MB)", "avg_ms": round(bn_ms, 4),
                                 "achieved": round(bn_bytes / (bn_ms * 1e-3) / 1e9, 1), "unit": "GB/s",
                                 "frac": round(bn_bytes / (bn_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
        del xbn, ws, mv

        # on-demand checkpoint (all EST contexts by virtual rank + one copy of p and v) to a pinned
        # host blob and back: host-link traffic, timed on the wall clock (the calls are synchronous)
        ck_n = B.es_checkpoint_bytes(job.h)
        blob = oracle_leg.pin.view(torch.uint8)[:ck_n] if (oracle_leg is not None and
                                                           oracle_leg.pin.numel() * 4 >= ck_n) \
            else torch.empty(ck_n, dtype=torch.uint8, pin_memory=True)
        ck_ms = {}
        for name in ("export", "import"):
            best = None
            for _ in range(3):
                t0 = time.perf_counter()
                if name == "export":
                    B.check(B.es_checkpoint_export(job.h, blob.data_ptr(), ck_n, job.p.data_ptr(),
                                                   job.v.data_ptr(), 1), "es_checkpoint_export", job.h)
                else:
                    B.check(B.es_checkpoint_import(job.h, blob.data_ptr(), ck_n, job.p.data_ptr(),
                                                   job.v.data_ptr())[0], "es_checkpoint_import", job.h)
                t = (time.perf_counter() - t0) * 1e3
                best = t if best is None else min(best, t)
            ck_ms[name] = best
        res["checkpoint"] = {"note": "es_checkpoint_export / es_checkpoint_import to and from a pinned host blob "
                                     "(host link, not HBM; best of 3)", "bytes": ck_n,
                             "export_ms": round(ck_ms["export"], 3), "import_ms": round(ck_ms["import"], 3),
                             "export_GBps": round(ck_n / (ck_ms["export"] * 1e-3) / 1e9, 1),
                             "import_GBps": round(ck_n / (ck_ms["import"] * 1e-3) / 1e9, 1)}

    # small working sets live in the 256 MB Infinity Cache between steps: also time the whole
    # step cold, after a 1 GiB fill has swept the cache (per-step HIP events, fill not timed)
    if (2 * N + 3) * 4 * P < (512 << 20) and not a.no_extras:
        sweep = torch.empty(1 << 28, dtype=torch.float32, device=dev)
        tot = []
        for _ in range(steps):
            with torch.cuda.stream(job.main):
                sweep.fill_(1.0)
            c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            c0.record(job.main)
            step()
            c1.record(job.main)
            job.sync(); torch.cuda.synchronize()
            tot.append(c0.elapsed_time(c1))
        res["cold_step"] = {"note": "working set fits the Infinity Cache: whole step timed after a 1 GiB cache sweep",
                            "ms_per_step": stats_ms(tot),
                            "value": round(total / (statistics.fmean(tot) * 1e-3) / 1e9, 2), "unit": "GB/s"}
        del sweep

    job.close()
    del src, p0, job
    torch.cuda.empty_cache()
    return res


def host_swap_leg(torch, a, cid=2):
    """Memory-pressure mode (the paper's own placement of EST gradients, section 3.2): gradient slots
    in pinned host memory.  Two ways of reaching them are timed on one configuration: direct access
    over the host link from the staging and reduce kernels, and swap-in (device-to-host staging by
    asynchronous copies, buckets streamed back through two HBM buffers while the previous bucket is
    reduced).  Priced against the link rate a plain pinned-memory copy reaches in the same process."""
    from paper_2208_14228_amd import binding as B
    from paper_2208_14228_amd.job import ESTJob
    from workloads import configs

    cfg = configs.config(cid)
    lay, N, P = cfg.layout, cfg.n_logical, cfg.layout.n_params
    dev = "cuda:0"
    steps = max(3, min(a.steps, 5))
    # link rate: plain copies of 1 GiB between pinned host memory and HBM
    pin = torch.empty(1 << 28, dtype=torch.float32, pin_memory=True)
    d = torch.empty(1 << 28, dtype=torch.float32, device=dev)
    link = {}
    for name, (dst, src) in (("h2d", (d, pin)), ("d2h", (pin, d))):
        dst.copy_(src, non_blocking=True); torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            dst.copy_(src, non_blocking=True)
        torch.cuda.synchronize()
        link[name] = 3 * 4 * (1 << 28) / (time.perf_counter() - t0) / 1e9
    del pin, d
    out = {"note": "gradient slots in pinned host memory (memory-pressure mode); host link, not HBM",
           "config": cid, "n_logical": N, "n_params": P, "slot_bytes": N * 4 * P,
           "link_GBps": {k: round(v, 1) for k, v in link.items()}}
    src = [torch.randn(P, device=dev) * 1e-2 for _ in range(N)]
    all_buckets = list(range(lay.n_buckets))
    for mode in ("direct", "swap_in"):
        job = ESTJob(N, P, lay.buckets, cfg.chunk_align, [], None, None, dev, use_streams="three")
        job.set_option("host_slots", 1)
        job.set_option("swap_in", 1 if mode == "swap_in" else 0)
        job.set_grouping([0] * N, list(range(N)))
        m = [B.Marshalled(all_buckets, [src[e].data_ptr() + 4 * off for off, _ in lay.buckets]) for e in range(N)]
        st, rd, wall = [], [], []
        for i in range(-1, steps):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for e in range(N):
                B.es_accumulate_batch_m(job.h, e, m[e])
            job.stage.synchronize()
            t1 = time.perf_counter()
            job.reduce_sgd_step(cfg.lr, cfg.momentum, store_avg=False)
            job.sync(); torch.cuda.synchronize()
            t2 = time.perf_counter()
            if i >= 0:
                st.append((t1 - t0) * 1e3); rd.append((t2 - t1) * 1e3); wall.append((t2 - t0) * 1e3)
        job.close()
        sm, rm = statistics.fmean(st), statistics.fmean(rd)
        out[mode] = {"staging_ms": round(sm, 3), "staging_d2h_GBps": round(N * 4 * P / (sm * 1e-3) / 1e9, 1),
                     "staging_frac_of_link": round(N * 4 * P / (sm * 1e-3) / 1e9 / link["d2h"], 3),
                     "reduce_ms": round(rm, 3), "reduce_h2d_GBps": round(N * 4 * P / (rm * 1e-3) / 1e9, 1),
                     "reduce_frac_of_link": round(N * 4 * P / (rm * 1e-3) / 1e9 / link["h2d"], 3),
                     "step_ms": round(statistics.fmean(wall), 3)}
    del src
    torch.cuda.empty_cache()
    return out


def traffic_from_profiles(cid, fused):
    """HBM traffic of the reduce kernel cannot be measured from inside the process: it comes from the
    committed rocprofv3 counter summary of this same command, and only while the kernels are still
    the ones that were profiled (the summary records the hash of the kernel source)."""
    import hashlib
    try:
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as fh:
            doc = json.load(fh)
        with open(os.path.join(ROOT, "paper_2208_14228_amd", "csrc", "es_kernels.hip"), "rb") as fh:
            now = hashlib.sha256(fh.read()).hexdigest()[:16]
        tr = doc.get(f"config{cid}_{'fused' if fused else 'split'}")
        if not tr:
            return None, "no rocprofv3 counter summary for this configuration"
        if tr.get("kernel_source_sha16") != now:
            return None, "profiles/traffic.json was measured on an earlier version of the kernels"
        return tr["traffic_bytes"], "profiles/traffic.json (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE)"
    except (OSError, ValueError):
        return None, "no rocprofv3 counter summary"


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs the EST step on one GPU only (no collectives, no "
              "multi-GPU sharding); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if a.ceilings:
        print(json.dumps(ceilings()))
        return

    import torch

    from workloads import configs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; libes has no CPU path", file=sys.stderr)
        sys.exit(1)

    others = [] if a.no_configs else [c for c in (1, 2, 3, 4, 5) if c != a.config]
    oracle_leg = None
    if not a.no_cpu:
        need = 0
        for c in others + [a.config]:
            cfg = configs.config(c)
            need = max(need, cfg.n_logical * max(ln for _, ln in cfg.layout.buckets))
        oracle_leg = OracleLeg(torch, need)

    short = {c: measure(torch, a, c, False, oracle_leg) for c in others}
    # the same step of the context-heavy configuration with separate main / ctx / stage streams wired
    # by events (the save of a worker's last EST then overlaps the reduce): what the hand-offs cost
    three = overlap = None
    if not a.no_extras and a.streams == "one" and not a.no_configs:
        import copy

        def variant(streams, standin=0):
            av = copy.copy(a)
            av.streams, av.no_cpu, av.no_extras, av.standin = streams, True, True, standin
            return measure(torch, av, 4, False, None)

        r2, r3 = variant("two"), variant("three")
        three = {"note": "configuration 4 with separate main, ctx and stage streams (events between them) "
                         "instead of one in-order stream; two_stream = main (also small state) + stage",
                 "ms_per_step": r3["ms_per_step"], "step_GBps": r3["step_GBps"],
                 "two_stream_ms_per_step": r2["ms_per_step"],
                 "one_stream_ms_per_step": short[4]["ms_per_step"] if 4 in short else None}
        # paper section 3.2: the gradient copy of an EST overlaps the next EST's compute.  Each EST
        # computes a stand-in (one 4096^3 bf16 matmul on main) before its boundary call.
        o1, o2, o3 = variant("one", 4096), variant("two", 4096), variant("three", 4096)
        n_est = short[4]["n_logical"] if 4 in short else o1["n_logical"]
        mm = [torch.randn(4096, 4096, device="cuda:0", dtype=torch.bfloat16) for _ in range(3)]
        for _ in range(8):
            torch.mm(mm[0], mm[1], out=mm[2])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(4 * n_est):
            torch.mm(mm[0], mm[1], out=mm[2])
        torch.cuda.synchronize()
        compute_ms = (time.perf_counter() - t0) / 4 * 1e3
        del mm
        overlap = {"note": "configuration 4, every EST runs a compute-bound stand-in (4096^3 bf16 matmul on main) "
                           "before its boundary call: with a stage stream of its own the gradient copy "
                           "overlaps the next EST's compute (paper section 3.2)",
                   "standin_compute_ms_per_step": round(compute_ms, 4),
                   "one_stream_ms_per_step": o1["ms_per_step"], "two_stream_ms_per_step": o2["ms_per_step"],
                   "three_stream_ms_per_step": o3["ms_per_step"]}
    ceil = None if a.no_extras else ceilings()
    host_swap = None if a.no_extras else host_swap_leg(torch, a)
    head = measure(torch, a, a.config, True, oracle_leg)
    switch = None if a.no_switch else est_switch_us(torch)

    fused = not a.split
    traffic, traffic_src = (None, "options changed") if (a.opt or a.host_slots) else traffic_from_profiles(a.config, fused)
    red = head["reduce"]
    out = {
        "metric": "ring-order N-way grad reduce GB/s (% HBM peak); EST switch µs; 0-ULP",
        "value": head["step_GBps"],
        "unit": "GB/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": head["workload"], "n_logical": head["n_logical"], "n_params": head["n_params"],
                   "n_buckets": head["n_buckets"],
                   "mode": "fused reduce+sgd" if fused else "reduce, then sgd",
                   "streams": a.streams, "slots": "pinned host memory" if a.host_slots else "HBM",
                   "staging": ("per bucket" if a.per_bucket else "batched per EST, context switch a launch of its own"
                               if a.separate_calls else "one launch per EST boundary (stage + save + restore)"),
                   **head["options"]},
        "step_bytes": head["step_bytes"],
        "roofline": {"bound": "hbm" if not a.host_slots else "host link (not an HBM figure)",
                     "kernel": red["kernel"], "achieved": red["achieved"], "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": red["frac"], "traffic": traffic, "traffic_source": traffic_src,
                     "bytes_per_launch": red["bytes_per_launch"], "avg_launch_ms": red["launch_ms"]["mean"],
                     "median_launch_ms": red["launch_ms"]["median"], "min_launch_ms": red["launch_ms"]["min"],
                     "frac_at_min": red["frac_at_min"], "memory": red["memory"]},
        "reduce_pct_hbm_peak": round(100 * red["frac"], 2),
        "step_pct_hbm_peak": round(100 * head["step_frac"], 2),
        "kernels": {head["staging"]["kernel"] + " (staging)": head["staging"]},
        "zero_ulp": head["zero_ulp"],
        "zero_ulp_all_configs": (None if a.no_cpu or a.no_configs else
                                 bool(head["zero_ulp"] and all(r["zero_ulp"] for r in short.values()))),
        "cpu_baseline": head["cpu_baseline"],
        "cpu_baseline_all_cores": head["cpu_baseline_all_cores"],
        "est_switch": switch,
        "ceilings": ceil,
        "host_swapped_slots": host_swap,
        "three_stream_step": three,
        "staging_overlap": overlap,
    }
    for k in ("sgd", "reduce_alone", "sgd_alone", "reduce_hbm_only", "staged_16_per_launch_step", "in_place_last_step", "graph_step", "zero_copy_step", "grad_sq_norm",
              "clip_sgd_step", "bn_batch_stats", "checkpoint", "cold_step"):
        if k in head:
            out[k] = head[k]
    if not a.no_configs:
        keep = ("config", "workload", "ms_per_step", "step_GBps", "step_frac", "step_bytes", "reduce", "staging",
                "reduce_alone", "sgd_alone", "reduce_hbm_only", "cold_step", "staged_16_per_launch_step", "in_place_last_step", "graph_step",
                "zero_copy_step", "context_bytes_per_est", "mask_bytes_per_est", "zero_ulp",
                "cpu_baseline", "cpu_baseline_all_cores")
        allc = dict(short)
        allc[a.config] = head
        out["configs"] = [{k: allc[c][k] for k in keep if k in allc[c]} for c in sorted(allc)]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
