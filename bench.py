#!/usr/bin/env python3
"""Benchmark of the EST step on one MI355X.

One *step* = one global step of the whole hot path on synthetic gradients that
are already resident in HBM: for every EST its context restore, the staging of
all its gradient buckets into its context slot, its context save; then the
ring-ordered N-way reduce and the SGD-momentum update (fused in one kernel by
default, --split times them as two kernels).

Prints ONE JSON line.  `value` is whole-step throughput on algorithmic bytes;
`roofline` prices the reduce kernel (the kernel the metric names) against the
HBM peak from HIP-event timings taken inside the timed region; `kernels` holds
the same figure for the staging copy; `cpu_baseline` is the CPU oracle timed on
the host cores for the same step, whose result is also compared bit for bit
with the GPU's (`zero_ulp`).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, vendor figure


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, help="benchmark configuration 1..5")
    ap.add_argument("--split", action="store_true", help="reduce and SGD as two kernels")
    ap.add_argument("--per-bucket", action="store_true",
                    help="stage with one es_accumulate launch per bucket instead of es_accumulate_batch")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--no-switch", action="store_true", help="skip the EST-switch timing")
    ap.add_argument("--streams", choices=["one", "two", "three"], default="one",
                    help="one in-order stream (default: nothing to overlap with in this benchmark) or "
                         "separate main/ctx/stage streams wired with events")
    ap.add_argument("--host-slots", action="store_true",
                    help="memory-pressure mode: gradient slots in pinned host memory (host-link bound)")
    ap.add_argument("--overlap-demo", action="store_true",
                    help="separate experiment: staging on its own stream overlapped with a compute-bound "
                         "stand-in for the next EST's forward/backward (prints its own JSON line)")
    ap.add_argument("--ceilings", action="store_true",
                    help="separate experiment: what this box's HBM gives the library's plain copy and "
                         "pure-read kernels on 1 GiB (prints its own JSON line)")
    ap.add_argument("--opt", action="append", default=[], help="library option name=value")
    return ap.parse_args()


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


def overlap_demo(a):
    """Paper section 3.2: an EST's gradient copy is overlapped with the next EST's compute.
    Each EST = one compute-bound stand-in (a bf16 matmul on main) followed by the staging of
    its gradients; with one stream the two serialise, with a separate staging stream they
    overlap.  Reports ms per global step for both."""
    import torch

    from paper_2208_14228_amd import binding as B
    from paper_2208_14228_amd.job import ESTJob
    from workloads import configs

    cfg = configs.config(a.config)
    lay, N, P = cfg.layout, cfg.n_logical, cfg.layout.n_params
    dev = "cuda:0"
    src = [torch.randn(P, device=dev) for _ in range(N)]
    A = torch.randn(4096, 4096, device=dev, dtype=torch.bfloat16)
    Bm = torch.randn(4096, 4096, device=dev, dtype=torch.bfloat16)
    C = torch.empty(4096, 4096, device=dev, dtype=torch.bfloat16)
    buckets = list(range(lay.n_buckets))
    out = {"experiment": "staging overlapped with the next EST's compute", "config": a.config,
           "n_logical": N, "n_params": P}
    for mode in ("one", "two"):
        job = ESTJob(N, P, lay.buckets, cfg.chunk_align, [], None, None, dev, use_streams=mode)
        ptrs = [[src[e].data_ptr() + 4 * off for off, _ in lay.buckets] for e in range(N)]

        def step(compute=True, stage=True):
            for e in range(N):
                if compute:
                    with torch.cuda.stream(job.main):
                        torch.mm(A, Bm, out=C)
                if stage:
                    B.es_accumulate_batch(job.h, e, buckets, ptrs[e])
                else:
                    B.es_accumulate_batch(job.h, e, buckets, [B.es_grad_slot(job.h, e, b) for b in buckets])
            job.reduce_sgd_step(cfg.lr, cfg.momentum, store_avg=False)

        def timed(**kw):
            for _ in range(a.warmup):
                step(**kw)
            job.sync(); torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(a.steps):
                step(**kw)
            job.sync(); torch.cuda.synchronize()
            return round((time.perf_counter() - t0) / a.steps * 1e3, 4)

        out[f"streams_{mode}"] = {"compute_and_staging_ms": timed(),
                                  "compute_only_ms": timed(stage=False),
                                  "staging_only_ms": timed(compute=False)}
        job.close()
    print(json.dumps(out))


def ceilings(a):
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
    res = {"experiment": "plain streaming rates of the library's kernels on 1 GiB",
           "copy_read_plus_write_GBps": round(2 * gb / ((t_both - t_red) * 1e-3), 1),
           "n1_reduce_read_plus_write_GBps": round(2 * gb / (t_red * 1e-3), 1),
           "norm_read_only_pass_GBps": round(gb / (t_norm * 1e-3), 1), "hbm_peak_GBps": HBM_PEAK_GBPS}
    job.close()
    print(json.dumps(res))


def main():
    a = parse()
    if a.ceilings:
        if a.gpus != 1:
            sys.exit(2)
        ceilings(a)
        return
    if a.overlap_demo:
        if a.gpus != 1:
            sys.exit(2)
        overlap_demo(a)
        return
    if a.gpus != 1:
        print("bench.py: this build runs the EST step on one GPU only (no collectives, no "
              "multi-GPU sharding); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2208_14228_amd import binding as B
    from paper_2208_14228_amd.job import ESTJob
    from workloads import configs, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; libes has no CPU path", file=sys.stderr)
        sys.exit(1)

    cfg = configs.config(a.config)
    lay, N, P = cfg.layout, cfg.n_logical, cfg.layout.n_params
    g = cfg.groupings[0]
    dev = "cuda:0"
    segs = []
    if cfg.dropout:
        segs.append(16)
    segs += [4 * c for c in cfg.bn_channels for _ in (0, 1)]

    job = ESTJob(N, P, lay.buckets, cfg.chunk_align, segs, g.worker_of_est, g.slot_of_est, dev,
                 use_streams=a.streams)
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
    for e in range(N):
        if segs:
            job.ctx_save(e)
    job.sync()
    torch.cuda.synchronize()

    fused = not a.split
    all_buckets = list(range(lay.n_buckets))
    src_ptrs = [[src[e].data_ptr() + 4 * off for off, _ in lay.buckets] for e in range(N)]
    ev_r = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
            for _ in range(a.steps)]
    ev_s = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
            for _ in range(a.steps)]
    ev_c = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
            for _ in range(a.steps)]

    # EST e takes over the worker's live state: the first EST of a worker is restored, later
    # ones switch in with the fused save+restore kernel, the last one is saved at the end
    sched = g.schedule()
    prev_of = {e: (sched[k - 1] if k and g.worker_of_est[sched[k - 1]] == g.worker_of_est[e] else None)
               for k, e in enumerate(sched)}
    last_of_worker = [e for k, e in enumerate(sched)
                      if k + 1 == len(sched) or g.worker_of_est[sched[k + 1]] != g.worker_of_est[e]]

    def enter(e):
        if not segs:
            return
        if prev_of[e] is None:
            job.ctx_restore(e)
        else:
            job.ctx_switch(prev_of[e], e)

    def leave():
        if segs:
            for e in last_of_worker:
                job.ctx_save(e)

    def step(i=None):
        if i is not None:
            if job.stage is not job.main:
                job.stage.wait_stream(job.main)  # the interval below must not include the previous reduce
            ev_c[i][0].record(job.stage)
        for e in sched:
            enter(e)
            if mask is not None:
                job.dropout_mask(e, 0, mask, configs.DROPOUT_P)
            if a.per_bucket:
                for b, (off, ln) in enumerate(lay.buckets):
                    B.es_accumulate(job.h, e, b, src[e].data_ptr() + 4 * off)
            else:
                B.es_accumulate_batch(job.h, e, all_buckets, src_ptrs[e])
        leave()
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

    # ---- bit check of one step against the CPU oracle, which is timed as the CPU baseline ----
    cpu = None
    zero_ulp = None
    if not a.no_cpu:
        import oracle
        from oracle.ddp_reference import DDPReference
        job.p.copy_(p0); job.v.zero_()
        torch.cuda.synchronize()
        step()
        job.sync(); torch.cuda.synchronize()
        gp, gv = job.p.cpu().numpy(), job.v.cpu().numpy()
        host = [t.cpu().numpy() for t in src]
        ref = DDPReference(N, lay.buckets, P, cfg.chunk_align, cfg.lr, cfg.momentum, p0.cpu().numpy())
        oracle.lib()
        t0 = time.perf_counter()
        ref.global_step(lambda r, b: host[r][lay.buckets[b][0]:lay.buckets[b][0] + lay.buckets[b][1]])
        dt = time.perf_counter() - t0
        zero_ulp = bool(np.array_equal(gp.view(np.uint32), ref.p.view(np.uint32)) and
                        np.array_equal(gv.view(np.uint32), ref.v.view(np.uint32)))
        # a bounded sample: the checked step plus further global steps of the same work until
        # about 10 s of CPU time have been spent (at most 40 steps)
        n_cpu = 1
        while dt < 10.0 and n_cpu < 40:
            t0 = time.perf_counter()
            ref.global_step(lambda r, b: host[r][lay.buckets[b][0]:lay.buckets[b][0] + lay.buckets[b][1]])
            dt += time.perf_counter() - t0
            n_cpu += 1
        cpu_bytes = (N + 1) * 4 * P + 5 * 4 * P
        cpu = {"value": round(n_cpu * cpu_bytes / dt / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "seconds": round(dt, 3),
               "sample": f"{n_cpu} full global steps of config {a.config} (ring all-reduce simulation of all "
                         f"{lay.n_buckets} buckets among {N} ranks, /N, SGD-momentum), bytes counted as "
                         f"(N+1)*4P + 5*4P per step; gradient staging not included"}
        del host

    # ---- timed region ----
    job.p.copy_(p0); job.v.zero_()
    torch.cuda.synchronize()
    for _ in range(a.warmup):
        step()
    job.sync(); torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(a.steps):
        step(i)
    job.sync(); torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_step = dt / a.steps * 1e3

    # small working sets live in the 256 MB Infinity Cache between steps: also time the step
    # cold, after a 1 GiB fill has swept the cache (per-step HIP events, fill not timed)
    cold_ms = None
    if (N + 3) * 4 * P + N * 4 * P < (512 << 20):
        sweep = torch.empty(1 << 28, dtype=torch.float32, device=dev)
        tot = 0.0
        for _ in range(a.steps):
            with torch.cuda.stream(job.main):
                sweep.fill_(1.0)
            c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            c0.record(job.main)
            step()
            c1.record(job.main)
            job.sync(); torch.cuda.synchronize()
            tot += c0.elapsed_time(c1)
        cold_ms = tot / a.steps
        del sweep

    # the same step when the EST's backward writes its buckets straight into the slots
    # (es_grad_slot): staging degenerates to marking the buckets present
    slot_ptrs = [[B.es_grad_slot(job.h, e, b) for b in all_buckets] for e in range(N)]

    def step_zero_copy():
        for e in sched:
            enter(e)
            if mask is not None:
                job.dropout_mask(e, 0, mask, configs.DROPOUT_P)
            B.es_accumulate_batch(job.h, e, all_buckets, slot_ptrs[e])
        leave()
        if fused:
            job.reduce_sgd_step(cfg.lr, cfg.momentum, store_avg=False)
        else:
            job.ring_order_reduce()
            job.sgd_step(cfg.lr, cfg.momentum)

    # the paper's own flow (section 5.1.3): the last EST a worker runs is not staged, the
    # reduce reads its gradients where backward left them
    def step_in_place_last():
        for e in sched:
            enter(e)
            if mask is not None:
                job.dropout_mask(e, 0, mask, configs.DROPOUT_P)
            if e in last_of_worker and len(last_of_worker) <= 8:
                B.es_accumulate_in_place(job.h, e, src[e].data_ptr())
            else:
                B.es_accumulate_batch(job.h, e, all_buckets, src_ptrs[e])
        leave()
        if fused:
            job.reduce_sgd_step(cfg.lr, cfg.momentum, store_avg=False)
        else:
            job.ring_order_reduce()
            job.sgd_step(cfg.lr, cfg.momentum)

    for _ in range(a.warmup):
        step_in_place_last()
    job.sync(); torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        step_in_place_last()
    job.sync(); torch.cuda.synchronize()
    dt_ip = time.perf_counter() - t0

    # the default step captured once into a HIP graph on the job's stream and replayed
    dt_graph = None
    if a.streams == "one":
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=job.main):
            step()
        for _ in range(a.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            graph.replay()
        torch.cuda.synchronize()
        dt_graph = time.perf_counter() - t0

    for _ in range(a.warmup):
        step_zero_copy()
    job.sync(); torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        step_zero_copy()
    job.sync(); torch.cuda.synchronize()
    dt_zc = time.perf_counter() - t0

    # fixed-tree global norm of a vector of the job's size (one read of 4P bytes)
    out2 = torch.zeros(2, device=dev)
    for _ in range(3):
        B.es_grad_sq_norm(job.h, job.p.data_ptr(), out2.data_ptr())
    n0, n1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n0.record(job.main)
    for _ in range(a.steps):
        B.es_grad_sq_norm(job.h, job.p.data_ptr(), out2.data_ptr())
    n1.record(job.main)
    job.sync(); torch.cuda.synchronize()
    norm_ms = n0.elapsed_time(n1) / a.steps

    # on-demand checkpoint (all EST contexts by virtual rank + one copy of p and v) to a pinned
    # host blob and back: host-link traffic, timed on the wall clock (the calls are synchronous)
    ck_n = B.es_checkpoint_bytes(job.h)
    blob = torch.empty(ck_n, dtype=torch.uint8, pin_memory=True)
    ck_ms = {}
    for name in ("export", "import"):
        best = None
        for _ in range(3):
            t0 = time.perf_counter()
            if name == "export":
                B.check(B.es_checkpoint_export(job.h, blob.data_ptr(), ck_n, job.p.data_ptr(), job.v.data_ptr(), 1),
                        "es_checkpoint_export", job.h)
            else:
                B.check(B.es_checkpoint_import(job.h, blob.data_ptr(), ck_n, job.p.data_ptr(), job.v.data_ptr())[0],
                        "es_checkpoint_import", job.h)
            t = (time.perf_counter() - t0) * 1e3
            best = t if best is None else min(best, t)
        ck_ms[name] = best

    ctx_bytes = sum(segs)
    bytes_stage = 2 * N * 4 * P
    bytes_reduce = (N + 4) * 4 * P if fused else (N + 1) * 4 * P
    bytes_sgd = 0 if fused else 5 * 4 * P
    bytes_ctx = 2 * N * ctx_bytes + (N * mask.numel() if mask is not None else 0)
    total = bytes_stage + bytes_reduce + bytes_sgd + bytes_ctx

    red_ms = sum(x.elapsed_time(y) for x, y in ev_r) / a.steps
    stage_ms = sum(x.elapsed_time(y) for x, y in ev_c) / a.steps
    sgd_ms = (sum(x.elapsed_time(y) for x, y in ev_s) / a.steps) if not fused else None
    red_gbps = bytes_reduce / (red_ms * 1e-3) / 1e9
    n_copies = N * sum(1 for _, ln in lay.buckets if ln) if a.per_bucket else N

    out = {
        "metric": "ring-order N-way grad reduce GB/s (% HBM peak); EST switch µs; 0-ULP",
        "value": round(total / dt * a.steps / 1e9, 2),
        "unit": "GB/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config {a.config}: {cfg.name}-shaped gradient set, N={N} ESTs, "
                               f"P={P} fp32 in {lay.n_buckets} DDP buckets, grouping {g.name}",
                   "n_logical": N, "n_params": P, "n_buckets": lay.n_buckets,
                   "mode": "fused reduce+sgd" if fused else "reduce, then sgd",
                   "streams": a.streams, "slots": "pinned host memory" if a.host_slots else "HBM",
                   "staging": "per bucket" if a.per_bucket else "batched per EST", **opts},
        "step_bytes": {"staging": bytes_stage, "reduce": bytes_reduce, "sgd": bytes_sgd,
                       "context": bytes_ctx, "total": total},
        "roofline": {"bound": "hbm" if not a.host_slots else "host link (not an HBM figure)", "kernel": "k_ring_reduce" + (" (fused SGD)" if fused else ""),
                     "achieved": round(red_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(red_gbps / HBM_PEAK_GBPS, 4), "traffic": None,
                     "bytes_per_launch": bytes_reduce, "avg_launch_ms": round(red_ms, 4)},
        "kernels": {
            ("k_copy_f4" if a.per_bucket else "k_copy_runs") + " (staging)": {
                "launches_per_step": n_copies, "bytes_per_step": bytes_stage,
                "stream_ms_per_step": round(stage_ms, 4),
                "achieved": round(bytes_stage / (stage_ms * 1e-3) / 1e9, 1), "unit": "GB/s",
                "frac": round(bytes_stage / (stage_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)},
        },
        "zero_copy_step": {"note": "gradients produced directly in the slots (es_grad_slot), no staging copy",
                           "ms_per_step": round(dt_zc / a.steps * 1e3, 4),
                           "value": round((total - bytes_stage) / dt_zc * a.steps / 1e9, 2), "unit": "GB/s"},
        "in_place_last_step": {"note": "each worker's last EST is not staged: the reduce reads its "
                                       "gradients in place (es_accumulate_in_place)",
                               "ms_per_step": round(dt_ip / a.steps * 1e3, 4),
                               "value": round((total - bytes_stage * min(len(last_of_worker), 8) // N
                                               if len(last_of_worker) <= 8 else total) / dt_ip * a.steps / 1e9, 2),
                               "unit": "GB/s"},
        "graph_step": None if dt_graph is None else {
            "note": "the same step captured into a HIP graph and replayed",
            "ms_per_step": round(dt_graph / a.steps * 1e3, 4),
            "value": round(total / dt_graph * a.steps / 1e9, 2), "unit": "GB/s"},
        "grad_sq_norm": {"note": "fixed-tree global norm (k_sq_partials + k_sq_final), 4P bytes read",
                         "avg_ms": round(norm_ms, 4),
                         "achieved": round(4 * P / (norm_ms * 1e-3) / 1e9, 1), "unit": "GB/s",
                         "frac": round(4 * P / (norm_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)},
        "checkpoint": {"note": "es_checkpoint_export / es_checkpoint_import to and from a pinned host blob "
                               "(host link, not HBM; best of 3)", "bytes": ck_n,
                       "export_ms": round(ck_ms["export"], 3), "import_ms": round(ck_ms["import"], 3),
                       "export_GBps": round(ck_n / (ck_ms["export"] * 1e-3) / 1e9, 1),
                       "import_GBps": round(ck_n / (ck_ms["import"] * 1e-3) / 1e9, 1)},
        "cold_step": None if cold_ms is None else {
            "note": "working set fits the Infinity Cache: step timed after a 1 GiB cache sweep",
            "ms_per_step": round(cold_ms, 4), "value": round(total / (cold_ms * 1e-3) / 1e9, 2), "unit": "GB/s"},
        "reduce_pct_hbm_peak": round(100 * red_gbps / HBM_PEAK_GBPS, 2),
        "zero_ulp": zero_ulp,
        "cpu_baseline": cpu,
    }
    if sgd_ms is not None:
        out["kernels"]["k_sgd"] = {"avg_launch_ms": round(sgd_ms, 4),
                                   "achieved": round(bytes_sgd / (sgd_ms * 1e-3) / 1e9, 1),
                                   "unit": "GB/s"}
    # HBM traffic of the reduce kernel is not measurable from inside the process: it is taken
    # from the committed rocprofv3 counter summary of this same command, when there is one
    try:
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as fh:
            tr = json.load(fh).get(f"config{a.config}_{'fused' if fused else 'split'}")
        if tr and not a.opt and not a.host_slots:
            out["roofline"]["traffic"] = tr["traffic_bytes"]
            out["roofline"]["traffic_source"] = "profiles/traffic.json (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE)"
    except (OSError, ValueError):
        pass
    job.close()
    if not a.no_switch:
        out["est_switch"] = est_switch_us(torch)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
