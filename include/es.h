/*
 * libes — the EasyScaleThread (EST) step on one AMD MI355X (gfx950).
 *
 * N logical data-parallel workers (ESTs) are time-sliced on one device.  Each
 * EST has a context: its gradient buckets, plus small determinism-critical
 * state such as an RNG state and BatchNorm running statistics (paper §3.2
 * "Context switching", §3.3 "implicit framework state").  Parameters and
 * optimizer state exist once and are updated once per global step (§3.2).
 * At the end of a global step the N gradient sets are reduced in the fixed
 * order an N-rank ring all-reduce would use, each EST acting under its
 * constant virtual communication rank, bucket by bucket with the recorded
 * bucket mapping (§3.3, level D1), so the result does not depend on how ESTs
 * are grouped onto physical workers.
 *
 * Conventions
 *  - Plain C ABI.  Every pointer argument is marked HOST or DEVICE.  DEVICE
 *    pointers are ordinary HIP device addresses on the device that was current
 *    at es_init.  fp32 DEVICE buffers must be 16-byte aligned.
 *  - Every call returns ES_OK (0) or a negative es_status; nothing throws or
 *    aborts.  Arguments are validated synchronously before anything is
 *    enqueued; a call that fails validation enqueues nothing.  GPU work is
 *    enqueued asynchronously on the streams given to es_set_streams; errors of
 *    asynchronous work surface at es_sync.
 *  - `est` is always the EST's virtual rank in [0, n_logical), never a
 *    physical slot.
 *  - The library owns the context arenas (allocated with hipMalloc at es_init /
 *    es_set_grouping, released at es_destroy).  Parameters, momentum, averaged
 *    gradient, gradient sources, live state tensors and masks belong to the
 *    caller and must stay valid until the work enqueued on them has finished.
 *  - A handle is not thread-safe; calls on one handle must not overlap.
 *  - No kernel of this library uses atomics, and every floating-point result
 *    is independent of grid size and launch configuration.
 */
#ifndef ES_H
#define ES_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct es_handle es_handle;           /* opaque, owned by the library */

typedef enum es_status {
    ES_OK      = 0,
    ES_EINVAL  = -1,   /* null / out-of-range / misaligned argument, bad layout */
    ES_ESTATE  = -2,   /* call not valid now: bucket accumulated twice, reduce before all
                          (est, bucket) pairs were accumulated, live state not bound, ... */
    ES_ENOMEM  = -3,   /* host or device allocation failed */
    ES_EHIP    = -4    /* a HIP call failed; see es_last_hip_error */
} es_status;

/* One gradient bucket: a range of the flat fp32 parameter space. */
typedef struct es_bucket {
    uint64_t offset_elems;
    uint64_t len_elems;            /* may be 0 */
} es_bucket;

/*
 * The recorded gradient-bucket mapping (paper §3.3: the mapping is stored and
 * reinstated, never rebuilt) and the shape of the small per-EST state.
 *   buckets          HOST array; ranges must be disjoint, ascending and cover
 *                    [0, n_params) exactly (n_params <= 2^40).  Copied by es_init.
 *   chunk_align      >= 1.  Each bucket of length L is cut into n_logical ring
 *                    chunks of length roundup(ceil(L / n_logical), chunk_align);
 *                    trailing chunks may be short or empty.  4 keeps every
 *                    16-byte vector inside one chunk when bucket offsets are
 *                    multiples of 4; any value is correct.
 *   state_seg_bytes  HOST array of n_state_segs sizes (> 0): the live small
 *                    state tensors of one worker, e.g. a 16-byte Philox state
 *                    and the running mean / variance of every BatchNorm layer.
 *                    Copied by es_init.
 */
typedef void* (*es_dev_alloc_fn)(size_t bytes, void* user);
typedef void  (*es_dev_free_fn)(void* dev_ptr, void* user);

typedef struct es_bucket_layout {
    uint64_t         n_params;
    uint32_t         n_buckets;
    const es_bucket* buckets;
    uint32_t         chunk_align;
    uint32_t         n_state_segs;
    const uint64_t*  state_seg_bytes;
    /*
     * Optional device allocator of the caller (e.g. a framework's caching allocator), so
     * that the context arenas - N * n_params floats of gradient slots, the bulk of the
     * job's memory - come out of the caller's pool.  Both NULL: hipMalloc / hipFree.
     *   dev_alloc  returns a DEVICE pointer to `bytes` bytes on the device that is current
     *              at the call, aligned to 256 bytes, or NULL if it cannot (-> ES_ENOMEM);
     *              it must not throw or unwind through the library
     *   dev_free   releases a pointer dev_alloc returned; called from es_set_grouping and
     *              es_destroy after the handle's streams have been synchronised
     *   user       passed back unchanged
     * The functions must stay callable until es_destroy has returned.  Host-resident
     * slots (option "host_slots") are pinned host memory and never go through them.
     */
    es_dev_alloc_fn  dev_alloc;
    es_dev_free_fn   dev_free;
    void*            user;
} es_bucket_layout;

/*
 * Create a job of n_logical EasyScaleThreads (paper section 3.2: the logical workers
 * whose number, not the number of GPUs, fixes the training procedure; 1 .. 65535) on
 * the current HIP device, with the recorded bucket mapping of section 3.3 (D1).
 * Starts with one simulated worker that holds all ESTs (slot = rank), all
 * streams = the null stream, and no live state bound.
 * Allocates n_logical gradient slots of n_params floats and n_logical small
 * context slots on the device.  *out is set only on success.
 */
int es_init(es_handle** out, uint32_t n_logical, const es_bucket_layout* layout);

/* Waits for the handle's streams, frees all device and host memory of the handle. */
int es_destroy(es_handle* h);

/*
 * Streams (HOST values of hipStream_t; NULL = the null stream).
 *   main   the EST's own compute, es_dropout_mask, es_ring_order_reduce,
 *          es_sgd_step, es_reduce_sgd_step
 *   ctx    es_ctx_save / es_ctx_restore / es_ctx_switch (small state)
 *   stage  es_accumulate (bulk gradient copies, paper §3.2: overlapped with the
 *          next EST's compute)
 * Ordering is wired with events inside the calls: a restore starts after the
 * work already enqueued on main and is visible to work enqueued on main
 * afterwards; a save or an accumulate starts after the work already enqueued
 * on main; the reduce starts after every accumulate of the step.  If all three
 * are the same stream no events are used.  Must not be called while work of
 * this handle is in flight (call es_sync first).  The streams stay the
 * caller's; they must exist until es_destroy (which waits on them) or until
 * another es_set_streams replaces them.
 */
int es_set_streams(es_handle* h, void* main, void* ctx, void* stage);

/*
 * Map ESTs onto simulated physical workers (paper §3.2: any EST can be placed
 * on any worker; §3.3 D1: results must not depend on the placement).
 *   worker_of_est, slot_of_est  HOST arrays of n_logical entries; (worker, slot)
 *   pairs must be distinct, workers 0..n_workers-1 each non-empty, and slots of
 *   a worker dense in [0, #ESTs of that worker).
 * Every worker gets its own arena allocation.  The small-state contexts of all
 * ESTs are carried over to their new slots (device copies); staged gradients
 * are not, so this must be called between global steps (ES_ESTATE otherwise).
 * Live-state bindings are dropped.  Synchronises the handle's streams.
 * The new arenas are allocated before the old ones are freed, so a call that
 * fails (ES_ENOMEM, ES_EHIP) leaves the previous grouping fully usable; the
 * price is that both sets of gradient slots exist for the duration of the call.
 */
int es_set_grouping(es_handle* h, uint32_t n_workers,
                    const uint32_t* worker_of_est, const uint32_t* slot_of_est);

/*
 * Bind the live small-state tensors of one worker.
 *   live_ptrs  HOST array of n_state_segs DEVICE pointers; tensor j holds
 *              state_seg_bytes[j] bytes.  Any alignment is accepted (16-byte
 *              aligned tensors whose size is a multiple of 16 take the vector
 *              path).  Tensors must not overlap.
 */
int es_bind_live_state(es_handle* h, uint32_t worker, void* const* live_ptrs);

/*
 * Context switching, paper section 3.2: when an EST is scheduled its context is
 * loaded into the worker's live state; section 3.3 names the small states that
 * belong to it (RNG state, BatchNorm statistics).
 * slot[est] -> live tensors of est's worker.  One batched copy kernel on the ctx stream.
 */
int es_ctx_restore(es_handle* h, uint32_t est);
/*
 * Paper section 3.2: at the end of an EST's mini-batch its context is saved.
 * live tensors of est's worker -> slot[est].  One batched copy kernel on the ctx stream.
 * Work enqueued on main afterwards is NOT made to wait for the save (so the
 * save of a step's last EST overlaps with the reduce): the live tensors must
 * not be written again before the next es_ctx_restore / es_ctx_switch on that
 * worker, or es_sync.
 */
int es_ctx_save(es_handle* h, uint32_t est);
/*
 * Save est_out and restore est_in (same worker, est_out != est_in) in a single
 * kernel: an EST switch at a mini-batch boundary (paper §3.2).  Equivalent to
 * es_ctx_save(est_out) followed by es_ctx_restore(est_in).
 */
int es_ctx_switch(es_handle* h, uint32_t est_out, uint32_t est_in);

/*
 * Stage one gradient bucket of one EST in its context (the paper's per-EST
 * gradient copy, §3.2 / §5.1.3; here device-to-device because all N gradient
 * sets fit in HBM).
 *   d_grad_bucket  DEVICE, len_elems floats of that bucket, 4-byte aligned
 *                  (any such source is copied with 16-byte accesses; fastest
 *                  when source and slot are equally far off a 128-byte line,
 *                  as a bucket of one flat gradient vector is).  If it
 *                  equals es_grad_slot(est, bucket) nothing is copied and the
 *                  bucket is only marked as present (zero-copy production).
 * Exactly one call per (est, bucket) per global step: a second one returns
 * ES_ESTATE.  The source must stay unmodified until the copy has run (e.g.
 * until es_stage_fence or es_sync).
 */
int es_accumulate(es_handle* h, uint32_t est, uint32_t bucket, const float* d_grad_bucket);

/*
 * es_accumulate (paper section 3.2, section 5.1.3: the per-EST gradient copy) for several
 * buckets of one EST at once, same rules per bucket.
 *   buckets         HOST array of n distinct bucket indices
 *   d_grad_buckets  HOST array of n DEVICE pointers, one source per bucket
 * Up to 16 runs are copied by one kernel launch; sources that continue each other
 * in memory for buckets that are adjacent in the parameter space are merged into
 * one contiguous run (a flat gradient vector is one run).  Validation covers the
 * whole batch before anything is enqueued or marked.
 */
int es_accumulate_batch(es_handle* h, uint32_t est, uint32_t n, const uint32_t* buckets,
                        const float* const* d_grad_buckets);

/*
 * es_accumulate of ALL buckets of several ESTs at once, each from one flat gradient
 * vector (paper section 3.2's per-EST gradient copy, for the case that several ESTs'
 * gradients are resident at the same time: one EST of each worker that shares the
 * device, or buffers the framework has not reused yet).  Up to 16 ESTs travel in one
 * kernel launch, more in several.
 *   ests          HOST array of n_ests distinct virtual ranks
 *   d_flat_grads  HOST array of n_ests DEVICE pointers: n_params floats each in flat
 *                 parameter order, 4-byte aligned; a pointer that equals the EST's slot
 *                 (es_grad_slot(est, 0)) only marks that EST as present
 * Same rules as es_accumulate per (est, bucket); validation covers the whole call
 * before anything is enqueued or marked.
 */
int es_accumulate_many(es_handle* h, uint32_t n_ests, const uint32_t* ests,
                       const float* const* d_flat_grads);

/*
 * One EST boundary in ONE kernel launch (paper section 3.2: at a mini-batch boundary the
 * outgoing EST's context is saved, its gradients are copied aside, and the next EST's
 * context is restored): es_accumulate_batch(est_out, ...) fused with
 * es_ctx_switch(est_out, est_in), or with es_ctx_save(est_out) if est_in is ES_NO_EST
 * (the last EST a worker runs in a global step).  Same results as the separate calls.
 * One launch when the stage stream IS the main stream (after the work already enqueued on
 * main and on ctx).  When staging has a stream of its own the call keeps the overlap that
 * stream is there for: the copy is enqueued on the stage stream and the save/restore on
 * the ctx stream, as the separate calls would, and work enqueued on main afterwards waits
 * for the restore only, not for the copy (so, as for es_accumulate, the sources must stay
 * unmodified until the copy has run: es_stage_fence orders main after it).  est_out and est_in
 * must be on the same worker,
 * whose live state must be bound if the layout has state segments.
 */
#define ES_NO_EST 0xFFFFFFFFu
int es_est_boundary(es_handle* h, uint32_t est_out, uint32_t est_in, uint32_t n,
                    const uint32_t* buckets, const float* const* d_grad_buckets);

/*
 * Take ALL buckets of one EST in place, without a staging copy: the next reduce
 * reads this EST's gradients straight from d_flat_grad.  This is the paper's
 * treatment of the last EST a worker runs in a global step: it does not copy its
 * gradients aside, it goes straight to synchronization (section 5.1.3).
 *   d_flat_grad  DEVICE, n_params floats in flat parameter order (all buckets back
 *                to back), 16-byte aligned; produced by work already enqueued on
 *                main; must stay unmodified until the reduce of this step has run and
 *                must not overlap that reduce's outputs (ES_EINVAL at the reduce).
 * Counts as the accumulate of every bucket of `est` (ES_ESTATE if one of them is
 * already present).  Any number of ESTs may be taken this way (with all of them
 * in place nothing is staged at all).  Nothing is enqueued; the effect ends with the
 * next reduce that succeeds (a reduce that fails leaves the step as it was).
 */
int es_accumulate_in_place(es_handle* h, uint32_t est, const float* d_flat_grad);

/*
 * Where EST `est` keeps gradient bucket `bucket` (paper section 3.2: the gradients are the
 * part of an EST's context that is kept per EST until the global step ends).  A backward
 * pass that writes there needs no copy (see es_accumulate).  DEVICE address, NULL on bad
 * arguments; changes at es_set_grouping.
 */
float* es_grad_slot(es_handle* h, uint32_t est, uint32_t bucket);

/* Makes work enqueued on main after this call wait for all staging copies enqueued so far. */
int es_stage_fence(es_handle* h);

/*
 * Dropout keep-mask from the live RNG state of est's worker (paper §3.3: the
 * Dropout operator depends on RNG state, which therefore is EST context).
 *   state_seg  index of a 16-byte state segment {uint64 seed, uint64 offset},
 *              whose live tensor must be 8-byte aligned
 *   d_mask     DEVICE, n bytes, any alignment
 *   p          drop probability in [0, 1]; threshold = floor(p * 2^32)
 * Byte j becomes 1 (keep) iff word (j mod 4) of Philox4x32-10 (Salmon et al.,
 * SC'11) with key = seed and counter = (offset + j/4, 0, 0) is >= threshold;
 * then offset += ceil(n/4).  Runs on main.
 */
int es_dropout_mask(es_handle* h, uint32_t est, uint32_t state_seg,
                    uint8_t* d_mask, uint64_t n, double p);

/*
 * EST-aware gradient all-reduce on one device (paper §3.3 D1, §4 ElasticDDP).
 * For every bucket, ring chunk c and element i of that chunk:
 *     avg[i] = (((g[c][i] + g[c+1][i]) + ...) + g[c+N-1][i]) / (float)N
 * ranks taken mod N, every + and the / rounded to fp32 (IEEE, denormals kept):
 * the association order of an N-rank ring reduce-scatter, then the average.
 *   d_avg_grad  DEVICE, n_params floats, 16-byte aligned; written once (all
 *               ranks of a real ring would hold this same vector).
 * Requires every (est, bucket) to have been accumulated exactly once since the
 * last reduce (ES_ESTATE otherwise) and starts a new global step.
 */
int es_ring_order_reduce(es_handle* h, float* d_avg_grad);

/*
 * SGD with momentum on the single shared replica (paper §3.2):
 *     v <- mu*v + g ;  p <- p - lr*v
 * every multiply and add rounded to fp32 on its own (no fused multiply-add).
 * All DEVICE, n_params floats, 16-byte aligned; p and v updated in place.  The
 * three buffers must not overlap one another (ES_EINVAL).
 */
int es_sgd_step(es_handle* h, float* d_param, float* d_momentum,
                const float* d_avg_grad, float lr, float mu);

/*
 * es_ring_order_reduce and es_sgd_step in one kernel: same bits, without the
 * round trip of the averaged gradient through HBM.  d_avg_grad may be NULL
 * (not stored) or a DEVICE buffer of n_params floats.  Buffers must not overlap
 * one another (ES_EINVAL).
 */
int es_reduce_sgd_step(es_handle* h, float* d_param, float* d_momentum,
                       float* d_avg_grad, float lr, float mu);

/*
 * Global norm of a flat vector of the job's size (e.g. the averaged gradient, for
 * clipping) along a FIXED summation tree, so the bits depend on the data alone and
 * not on the GPU, the grid or the launch (the property the paper's level D2 asks of
 * reductions, section 3.3; the tree is this library's own):
 *   blocks of 4096 elements, missing tail elements count as +0; in a block lane t
 *   (0..255) adds, from +0, the squares of elements 4*(256*q + t) + c, q = 0..3 outer,
 *   c = 0..3 inner; lane sums combine as v[t] += v[t+s] for t < s, s = 128, 64, .., 1;
 *   block partials combine the same way (lane t first adds partials t, t+256, ...).
 *   Every square and add is rounded to fp32; no atomics.
 *   d_vec   DEVICE, n_params floats, 16-byte aligned
 *   d_out2  DEVICE, 2 floats: [0] sum of squares, [1] its correctly rounded square root
 * Runs on main.
 */
int es_grad_sq_norm(es_handle* h, const float* d_vec, float* d_out2);

/*
 * es_sgd_step with the averaged gradient clipped by its global norm first (the usual
 * convention of training frameworks; the paper does not discuss clipping): with norm =
 * d_norm2[1] as es_grad_sq_norm left it in device memory (no host round trip),
 *     coef = min(1, max_norm / (norm + eps)) ;  g' = coef * g ;  v <- mu*v + g' ;  p <- p - lr*v
 * every operation rounded to fp32 on its own.  Because the norm comes from the fixed tree the
 * clipped step is as independent of the launch as everything else here; with coef = 1 the
 * result is that of es_sgd_step.  Buffers as for es_sgd_step; d_norm2 DEVICE, 2 floats;
 * max_norm >= 0, eps >= 0 (ES_EINVAL otherwise).  Runs on main.  The usual sequence is
 * es_ring_order_reduce(avg), es_grad_sq_norm(avg, norm2), es_clip_sgd_step(.., avg, norm2, ..).
 */
int es_clip_sgd_step(es_handle* h, float* d_param, float* d_momentum, const float* d_avg_grad,
                     const float* d_norm2, float max_norm, float eps, float lr, float mu);

/*
 * BatchNorm batch statistics along the same fixed tree (paper section 3.3: BatchNorm is the
 * operator whose statistics belong to the EST context; level D2 asks of reductions that their
 * result not depend on the GPU).  Needs no handle.
 *   d_x     DEVICE, n_images x n_channels x n_positions floats (NCHW with H*W = n_positions),
 *           4-byte aligned
 *   d_mean, d_var  DEVICE, n_channels floats each
 * For every channel the M = n_images * n_positions values in the order (image, position) are
 * the terms of the tree described at es_grad_sq_norm (terms instead of squares, terms beyond M
 * count as +0):  mean = T(y) / (float)M ;  var = T((y - mean)^2) / (float)M  (biased variance),
 * every subtraction, square, add and division rounded to fp32.  No atomics; the first stage
 * uses wave shuffles, the second an LDS stage.
 *   d_workspace      DEVICE scratch of at least es_bn_workspace_floats(..) floats, 4-byte aligned
 *   stream           HOST value of a hipStream_t on the current device (NULL = null stream)
 * Limits: M < 2^31, n_channels <= 65535, n_images and n_positions > 0 (ES_EINVAL otherwise;
 * es_bn_workspace_floats returns 0 for sizes it rejects or that need no scratch).
 */
uint64_t es_bn_workspace_floats(uint64_t n_images, uint64_t n_channels, uint64_t n_positions);
int es_bn_batch_stats(const float* d_x, uint64_t n_images, uint64_t n_channels, uint64_t n_positions,
                      float* d_mean, float* d_var, float* d_workspace, uint64_t workspace_floats,
                      void* stream);

/*
 * es_grad_sq_norm for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Needs no
 * handle and calls no hipMalloc / hipFree or any allocating routine: the block
 * partials go to a fixed 1 MiB array that is part of the library's code object
 * (every GPU the library runs on holds its own copy until the process ends).
 * Same tree, same bits as es_grad_sq_norm on a vector of n elements.
 *   d_vec    DEVICE, n floats, 16-byte aligned (may be NULL if n = 0)
 *   n        <= 2^30 elements (262,144 block partials); larger n: ES_EINVAL
 *   d_out2   DEVICE, 2 floats: [0] sum of squares, [1] its square root
 *   stream   HOST value of a hipStream_t on the current device (NULL = null stream)
 * Runs on the current HIP device.  All calls on one GPU share that GPU's array:
 * calls that can overlap on one GPU (different streams without ordering between
 * them) race and must be ordered by the caller; calls on one stream are safe.
 * Nothing in the array has to start at zero (each call writes every partial it
 * later reads), so nothing is cleared.  ES_EHIP if a HIP call fails.
 */
int es_grad_sq_norm_static(const float* d_vec, uint64_t n, float* d_out2, void* stream);

/*
 * On-demand checkpoint (paper §3.2 "Adapting to elasticity"; §3.3 D1: the bucket
 * mapping travels with the checkpoint and is reinstated, never rebuilt).  Taken
 * between global steps when resources change; the job continues from it with the
 * ESTs distributed over workers in any other way and produces the same bits.
 *
 * The blob holds one copy of the shared state and the contexts of all ESTs:
 *   header   8 x uint64, little endian: magic 0x3130544B50435345 ("ESCPKT01"),
 *            n_logical, n_params, n_buckets, chunk_align, n_state_segs,
 *            ctx_bytes (payload of one context slot), global_step
 *   buckets  n_buckets x {uint64 offset_elems, uint64 len_elems}
 *   segments n_state_segs x uint64 size in bytes
 *   contexts n_logical x ctx_bytes, by virtual rank; inside a context every state
 *            segment starts at the next multiple of 16 bytes
 *   param    n_params x fp32, then momentum n_params x fp32
 *
 * es_checkpoint_bytes   size of the blob for this handle (0 for a NULL handle).
 * es_checkpoint_export  host_blob HOST, capacity >= es_checkpoint_bytes; d_param and
 *                       d_momentum DEVICE (n_params floats each).  Every EST's live state
 *                       must have been saved (es_ctx_save) and no bucket may be staged
 *                       (ES_ESTATE).  Synchronises the handle's streams; blocking copies.
 * es_checkpoint_import  into a handle created with the same n_logical and layout
 *                       (ES_EINVAL if the blob's header, bucket mapping or state segments
 *                       differ, or size is wrong); the handle's current grouping decides
 *                       where each context lands.  Writes d_param, d_momentum, *global_step
 *                       (may be NULL).  Blocking.
 */
uint64_t es_checkpoint_bytes(es_handle* h);
int es_checkpoint_export(es_handle* h, void* host_blob, uint64_t capacity,
                         const float* d_param, const float* d_momentum, uint64_t global_step);
int es_checkpoint_import(es_handle* h, const void* host_blob, uint64_t size,
                         float* d_param, float* d_momentum, uint64_t* global_step);

/* Blocks until all streams of the handle are idle; returns ES_EHIP if any work failed. */
int es_sync(es_handle* h);

/*
 * Options (never change results).  Names:
 *   "host_slots"          0/1: placement of gradient slots at the NEXT es_set_grouping: 1 =
 *                         pinned host memory mapped into the device (the paper keeps the
 *                         per-EST gradients in host memory, section 3.2; here it is the
 *                         memory-pressure mode for N * n_params beyond HBM): staging and
 *                         reduce run unchanged and reach the gradients over the host link
 *   "hbm_slot_budget_mib" -1 (no limit, default) or 0 .. 2^40: at the NEXT es_set_grouping the
 *                         workers' gradient arenas are placed in HBM in worker order until
 *                         this many MiB are used; the arenas that no longer fit spill to
 *                         pinned host memory (only what does not fit pays the host link)
 *   "swap_in"             0/1 (only between global steps, ES_ESTATE otherwise): how host-resident
 *                         gradient slots are reached.  0: the staging copy and the reduce kernel
 *                         access the mapped host memory directly over the link.  1: the paper's
 *                         mechanism - an EST's gradients are staged by asynchronous device-to-host
 *                         copies (copy engines, the compute units stay free for the next EST), and
 *                         the reduce streams them back bucket by bucket into two HBM buffers of
 *                         2 * n_logical * (largest bucket) floats, copying bucket b+1 on the
 *                         library's own copy queue while bucket b is reduced (es_plan_swap_in);
 *                         slots that are in HBM are read where they are.  Same bits either way
 *   "slots_on_host"       read-only (es_get_option): ESTs whose gradient slot is on the host
 *   "reduce_tile_elems"   elements of one bucket chunk handled by one workgroup
 *                         (multiple of 4, 256 .. 65536)
 *   "reduce_unroll"       16-byte vectors per lane in flight per rank (1, 2, 4)
 *   "reduce_rank_batch"   ranks loaded before their adds are issued (1, 2, 4, 8, 16;
 *                         default 8, or the largest power of two <= n_logical below that)
 *   "reduce_lds_pad_kib"  -1 (default) or 0 .. 160: KiB of LDS a workgroup of the small-tile reduce
 *                         reserves without using it, which caps the workgroups resident per CU
 *                         (160 KiB per CU); -1 = 64 (2 per CU), below 4 ranks 53 (3 per CU; 32 = 5 per CU
 *                         for the unfused reduce), 160
 *                         (1 per CU) for 8 or at least 10 ranks when parameters and momentum stream
 *   "nontemporal"         0/1: streaming hint on gradient loads
 *   "nontemporal_pv"      0/1: streaming hint on parameter and momentum traffic of the update
 *                         (fused or es_sgd_step / es_clip_sgd_step) and on the store of the
 *                         averaged gradient (default: 1 if parameters and momentum together
 *                         exceed 284 MiB, else 0)
 *   "reduce_big_unroll"   0, 8, 16 or 32: if not 0, full aligned stretches of a ring chunk
 *                         are handled in big tiles of 256 * value * 4 elements (long
 *                         contiguous reads per gradient stream; default 32 from
 *                         n_logical = 11 on, else 0)
 *   "reduce_big_rank_batch"  ranks loaded ahead in big tiles (1, 2, 4; unroll * batch <= 32)
 * Returns ES_EINVAL for unknown names or values.
 */
int es_set_option(es_handle* h, const char* name, int64_t value);
int es_get_option(es_handle* h, const char* name, int64_t* value);

/*
 * Host-only planning helper (touches no device): the schedule of the swap-in reduce (option
 * "swap_in"; paper section 3.2 keeps the gradients of switched-out ESTs in host memory, section
 * 5.1.3 overlaps their copies with compute).  The buckets of all ranks come back one at a time
 * into TWO device buffers; the list says what the library enqueues, in this order, on its copy
 * queue (fill) and on main (reduce):
 *   kind    ES_SWAP_FILL: bucket `bucket` of every host-resident rank -> buffer `half`;
 *           ES_SWAP_REDUCE: ring-ordered reduce (and update) of that bucket out of buffer `half`
 *   wait    index in the list of the one operation of the OTHER queue that has to finish first,
 *           or -1: a fill waits for the reduce that used its buffer before (bucket - 2), a reduce
 *           for its own fill.  Operations of one queue run in list order.
 * So bucket b+1 is copied while bucket b is reduced and at most two buckets are resident.
 *   out     HOST array of `capacity` entries, or NULL to query *n_ops (= 2 * n_buckets) only
 */
enum { ES_SWAP_FILL = 0, ES_SWAP_REDUCE = 1 };
typedef struct es_swap_op {
    uint32_t kind;
    uint32_t bucket;
    uint32_t half;
    int32_t  wait;
} es_swap_op;
int es_plan_swap_in(uint32_t n_buckets, es_swap_op* out, uint64_t capacity, uint64_t* n_ops);

/*
 * Host-only planning helper (touches no device): the work decomposition of the
 * ring-ordered reduce for a layout.  Each tile is a range of the flat parameter
 * space that lies inside ONE ring chunk of one bucket; start_rank is the virtual
 * rank whose gradient opens the fold for every element of the tile (= the chunk
 * index, see es_ring_order_reduce).  The first *n_big tiles are big tiles of
 * 256 * big_unroll * 4 elements (full, offset a multiple of 4); all others have
 * at most tile_elems elements.  A chunk that starts inside a 128-byte line (32
 * elements; 16 bytes if tile_elems is not a multiple of 32) opens with a shorter
 * tile that ends on a line boundary, so every later tile of the chunk starts on
 * one.  Tiles are disjoint and cover [0, n_params).
 *   out       HOST array of `capacity` entries, or NULL to query the counts only
 * Returns ES_EINVAL for an invalid layout or option value, or capacity too small.
 */
typedef struct es_tile {
    uint64_t offset_elems;
    uint32_t len_elems;
    uint32_t start_rank;
} es_tile;
int es_plan_tiles(uint32_t n_logical, const es_bucket_layout* layout, uint32_t tile_elems,
                  uint32_t big_unroll, es_tile* out, uint64_t capacity, uint64_t* n_tiles,
                  uint64_t* n_big);

/* Sizes the library derived from the layout (HOST out pointers, each may be NULL). */
int es_query(es_handle* h, uint64_t* n_params, uint32_t* n_buckets, uint64_t* ctx_bytes,
             uint32_t* n_workers, uint64_t* n_reduce_tiles);

int         es_last_hip_error(es_handle* h);      /* hipError_t of the last ES_EHIP, else 0 */
const char* es_strerror(int status);
const char* es_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ES_H */
