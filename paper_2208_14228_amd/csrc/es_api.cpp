// Host runtime and C boundary of libes (declared in include/es.h).
//
// Host side only: argument validation, the ring-chunk tile table, the
// rank -> slot pointer table, context piece tables, stream/event wiring and
// per-step bookkeeping.  All data movement and arithmetic is done by the
// kernels in es_kernels.hip.
#include "es.h"
#include "es_internal.h"

#include <algorithm>
#include <cstring>
#include <new>
#include <string>
#include <vector>

using namespace es;

namespace {

constexpr uint64_t kSlotAlignBytes = 256;

struct Worker {
    uint32_t n_slots = 0;
    float* grad_arena = nullptr;        // n_slots * grad_stride floats
    bool grad_on_host = false;          // arena is pinned host memory mapped into the device
    uint8_t* ctx_arena = nullptr;       // n_slots * ctx_stride bytes
    std::vector<void*> live;            // bound live tensors (device addresses)
    Piece* d_pieces = nullptr;
    uint32_t n_pieces = 0;
    bool bound = false;
};

}  // namespace

struct es_handle {
    int device = 0;
    uint32_t N = 0;
    uint64_t P = 0;
    uint32_t A = 1;
    std::vector<es_bucket> buckets;
    std::vector<uint64_t> seg_bytes, seg_off;   // seg_off: byte offset inside a context slot
    uint64_t ctx_bytes = 0;                     // payload of one context slot (16-byte padded segments)
    uint64_t ctx_stride = 0;                    // bytes between context slots
    uint64_t grad_stride = 0;                   // floats between gradient slots

    std::vector<uint32_t> worker_of, slot_of;
    std::vector<Worker> workers;

    Tile* d_tiles = nullptr;
    uint32_t n_tiles = 0;
    uint32_t n_big = 0;                         // leading big tiles (see k_ring_reduce_big)
    const float** d_slots = nullptr;            // N device pointers, by virtual rank
    float* d_partials = nullptr;                // ceil(P / 4096) block partials of es_grad_sq_norm

    // ESTs whose gradients the next reduce reads in place (rank, caller's flat gradient)
    std::vector<uint32_t> in_place_rank;
    std::vector<const float*> in_place_ptr;
    std::vector<uint8_t> accumulated;           // [est * n_buckets + bucket]
    uint64_t n_accumulated = 0;

    hipStream_t s_main = nullptr, s_ctx = nullptr, s_stage = nullptr;
    hipEvent_t ev_main = nullptr, ev_ctx = nullptr, ev_stage = nullptr;
    bool stage_pending = false;                 // staging copies enqueued since the last fence

    // one pass per workgroup: 256 lanes x 2 vectors x 4 floats (measured best on MI355X)
    bool host_slots = false;                    // where the next arena allocation places gradient slots
    int64_t hbm_budget_mib = -1;                // >= 0: gradient arenas beyond this many MiB of HBM go to the host
    uint64_t hbm_grad_bytes = 0;                // HBM held by gradient arenas allocated in the current regrouping
    uint32_t tile_elems = 2048;
    ReduceShape shape{2, 8, 1, 0, 1, 0, -1};

    // Swap-in of host-resident gradient slots (option "swap_in"): at the reduce the buckets come
    // back one at a time into two device buffers, bucket b+1 being copied while bucket b is reduced.
    bool swap_in = false;
    bool swap_ready = false;                    // tables below match the current grouping and tile shape
    hipStream_t s_swap = nullptr;               // the library's own copy queue (default priority)
    hipEvent_t ev_filled[2] = {nullptr, nullptr}, ev_consumed[2] = {nullptr, nullptr};
    float* d_swap_buf = nullptr;                // 2 x N rows of swap_row floats
    uint64_t swap_row = 0;
    Tile* d_swap_tiles = nullptr;               // per-bucket tile tables, back to back
    std::vector<uint64_t> swap_tile_off;        // first tile of bucket b
    std::vector<uint32_t> swap_n_tiles, swap_n_big;
    const float** d_swap_tables = nullptr;      // [half][bucket][rank] gradient base pointers

    // the caller's device allocator (es_bucket_layout), or null: hipMalloc / hipFree
    es_dev_alloc_fn dev_alloc = nullptr;
    es_dev_free_fn dev_free = nullptr;
    void* user = nullptr;

    int last_hip = 0;
};

namespace {

int hip_fail(es_handle* h, hipError_t e)
{
    if (h) h->last_hip = (int)e;
    return ES_EHIP;
}

#define ES_HIP(h, call)                                  \
    do {                                                 \
        hipError_t e__ = (call);                         \
        if (e__ != hipSuccess) return hip_fail((h), e__); \
    } while (0)

uint64_t round_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

// Device memory of the handle: the caller's allocator if one was given, else hipMalloc.
hipError_t dev_malloc(es_handle* h, void** out, size_t bytes)
{
    if (!h->dev_alloc) return hipMalloc(out, bytes);
    void* p = h->dev_alloc(bytes, h->user);
    if (p && (((uintptr_t)p) & (kSlotAlignBytes - 1))) {       // the contract asks for 256-byte alignment
        h->dev_free(p, h->user);
        *out = nullptr;
        return hipErrorInvalidValue;
    }
    *out = p;
    return p ? hipSuccess : hipErrorOutOfMemory;
}

void dev_release(es_handle* h, void* p)
{
    if (!p) return;
    if (h->dev_free) h->dev_free(p, h->user);
    else (void)hipFree(p);
}

float* slot_base(const es_handle* h, uint32_t est)
{
    const Worker& w = h->workers[h->worker_of[est]];
    return w.grad_arena + (uint64_t)h->slot_of[est] * h->grad_stride;
}

uint8_t* ctx_base(const es_handle* h, uint32_t est)
{
    const Worker& w = h->workers[h->worker_of[est]];
    return w.ctx_arena + (uint64_t)h->slot_of[est] * h->ctx_stride;
}

// Under swap-in, gradients of an EST whose slot lives in host memory are staged by asynchronous
// device-to-host copies (the copy engines, which leave the compute units to the next EST) instead
// of a copy kernel that writes through the host link.
bool dma_staging(const es_handle* h, uint32_t est)
{
    return h->swap_in && h->workers[h->worker_of[est]].grad_on_host;
}

void free_worker(es_handle* h, Worker& w)
{
    if (w.grad_arena) {
        if (w.grad_on_host) (void)hipHostFree(w.grad_arena);
        else dev_release(h, w.grad_arena);
    }
    dev_release(h, w.ctx_arena);
    dev_release(h, w.d_pieces);
    w = Worker{};
}

int alloc_worker(es_handle* h, Worker& w, uint32_t n_slots)
{
    w.n_slots = n_slots;
    const uint64_t gbytes = (uint64_t)n_slots * h->grad_stride * sizeof(float);
    const uint64_t cbytes = (uint64_t)n_slots * h->ctx_stride;
    if (gbytes) {
        // host placement: pinned, device-mapped memory; the staging copy and the reduce then
        // reach the gradients over the host link with the same kernels (memory-pressure mode)
        w.grad_on_host = h->host_slots ||
                         (h->hbm_budget_mib >= 0 && h->hbm_grad_bytes + gbytes > ((uint64_t)h->hbm_budget_mib << 20));
        if (!w.grad_on_host) h->hbm_grad_bytes += gbytes;
        hipError_t e = w.grad_on_host
                           ? hipHostMalloc((void**)&w.grad_arena, gbytes, hipHostMallocMapped | hipHostMallocPortable)
                           : dev_malloc(h, (void**)&w.grad_arena, gbytes);
        if (e != hipSuccess) { h->last_hip = (int)e; w.grad_arena = nullptr; return e == hipErrorOutOfMemory ? ES_ENOMEM : ES_EHIP; }
    }
    if (cbytes) {
        hipError_t e = dev_malloc(h, (void**)&w.ctx_arena, cbytes);
        if (e != hipSuccess) { h->last_hip = (int)e; return e == hipErrorOutOfMemory ? ES_ENOMEM : ES_EHIP; }
        e = hipMemset(w.ctx_arena, 0, cbytes);
        if (e != hipSuccess) return hip_fail(h, e);
    }
    return ES_OK;
}

// Ring-chunk tile table.  Chunk c of a bucket of length L covers
// [min(L, c*CL), min(L, (c+1)*CL)), CL = roundup(ceil(L/N), A).  Pure host logic.
void plan_tiles(const std::vector<es_bucket>& buckets, uint32_t N, uint32_t A, uint64_t T,
                uint64_t TB, std::vector<Tile>& big, std::vector<Tile>& small)
{
    for (const es_bucket& b : buckets) {
        const uint64_t L = b.len_elems;
        if (L == 0) continue;
        const uint64_t CL = round_up((L + N - 1) / N, A);
        for (uint32_t c = 0; c < N; ++c) {
            const uint64_t lo = std::min<uint64_t>(L, (uint64_t)c * CL);
            const uint64_t hi = std::min<uint64_t>(L, lo + CL);
            uint64_t a = lo;
            // A chunk that starts inside a 128-byte line opens with a tile that ends on a line
            // boundary: every later tile then starts on one (a line shared by two workgroups
            // is fetched twice, by two compute dies), only the opening tile can have scalar
            // leading elements, and big tiles stay usable.  The opening tile is just the
            // elements up to the boundary when big tiles follow, else a tile a little short of T.
            const uint64_t line = (T % 32 == 0) ? 32 : 4;                 // elements
            const uint64_t mis = (b.offset_elems + lo) & (line - 1);
            if (mis && lo < hi) {
                const uint64_t odd = line - mis;
                Tile t;
                t.off = b.offset_elems + a;
                t.len = (uint32_t)((TB && a + odd + TB <= hi) ? odd : std::min<uint64_t>(hi - a, T - mis));
                t.rank0 = c;
                small.push_back(t);
                a += t.len;
            }
            // full, 16-byte aligned big tiles first; the remainder of the chunk in small tiles
            if (TB && ((b.offset_elems + a) & 3) == 0) {
                for (; a + TB <= hi; a += TB) {
                    Tile t;
                    t.off = b.offset_elems + a;
                    t.len = (uint32_t)TB;
                    t.rank0 = c;
                    big.push_back(t);
                }
            }
            for (; a < hi; a += T) {
                Tile t;
                t.off = b.offset_elems + a;
                t.len = (uint32_t)std::min<uint64_t>(T, hi - a);
                t.rank0 = c;
                small.push_back(t);
            }
        }
    }
}

int build_tiles(es_handle* h)
{
    std::vector<Tile> big, tiles;
    const uint64_t TB = h->shape.big_unroll ? (uint64_t)kReduceBlock * h->shape.big_unroll * 4 : 0;
    plan_tiles(h->buckets, h->N, h->A, h->tile_elems, TB, big, tiles);
    if (big.size() + tiles.size() > 0x7fffffffull) return ES_EINVAL;
    h->swap_ready = false;                       // the per-bucket tile tables of the swap-in path follow the same shape
    h->n_big = (uint32_t)big.size();
    big.insert(big.end(), tiles.begin(), tiles.end());
    tiles.swap(big);
    if (h->d_tiles) { dev_release(h, h->d_tiles); h->d_tiles = nullptr; }
    h->n_tiles = (uint32_t)tiles.size();
    if (h->n_tiles) {
        ES_HIP(h, dev_malloc(h, (void**)&h->d_tiles, tiles.size() * sizeof(Tile)));
        ES_HIP(h, hipMemcpy(h->d_tiles, tiles.data(), tiles.size() * sizeof(Tile), hipMemcpyHostToDevice));
    }
    return ES_OK;
}

int validate_layout(uint32_t n_logical, const es_bucket_layout* lay)
{
    if (!lay || n_logical == 0 || n_logical > 65535) return ES_EINVAL;
    if (lay->chunk_align == 0 || (lay->n_buckets && !lay->buckets)) return ES_EINVAL;
    if (lay->n_state_segs && !lay->state_seg_bytes) return ES_EINVAL;
    if ((lay->dev_alloc == nullptr) != (lay->dev_free == nullptr)) return ES_EINVAL;   // both or neither
    uint64_t pos = 0;
    for (uint32_t b = 0; b < lay->n_buckets; ++b) {
        if (lay->buckets[b].offset_elems != pos) return ES_EINVAL;        // ascending, disjoint, no gaps
        if (lay->buckets[b].len_elems > (1ull << 40)) return ES_EINVAL;
        pos += lay->buckets[b].len_elems;
    }
    if (pos != lay->n_params || pos > (1ull << 40)) return ES_EINVAL;
    for (uint32_t j = 0; j < lay->n_state_segs; ++j)
        if (lay->state_seg_bytes[j] == 0 || lay->state_seg_bytes[j] > (1ull << 32)) return ES_EINVAL;
    return ES_OK;
}

int upload_slot_table(es_handle* h)
{
    std::vector<const float*> ptrs(h->N);
    for (uint32_t e = 0; e < h->N; ++e) ptrs[e] = slot_base(h, e);
    if (!h->d_slots) ES_HIP(h, dev_malloc(h, (void**)&h->d_slots, h->N * sizeof(float*)));
    ES_HIP(h, hipMemcpy((void*)h->d_slots, ptrs.data(), h->N * sizeof(float*), hipMemcpyHostToDevice));
    return ES_OK;
}

bool valid_grouping(uint32_t N, uint32_t n_workers, const uint32_t* wo, const uint32_t* so,
                    std::vector<uint32_t>& counts)
{
    if (n_workers == 0 || n_workers > N) return false;
    counts.assign(n_workers, 0);
    for (uint32_t e = 0; e < N; ++e) {
        if (wo[e] >= n_workers) return false;
        counts[wo[e]]++;
    }
    std::vector<std::vector<uint8_t>> seen(n_workers);
    for (uint32_t w = 0; w < n_workers; ++w) {
        if (counts[w] == 0) return false;
        seen[w].assign(counts[w], 0);
    }
    for (uint32_t e = 0; e < N; ++e) {
        if (so[e] >= counts[wo[e]] || seen[wo[e]][so[e]]) return false;
        seen[wo[e]][so[e]] = 1;
    }
    return true;
}

// Ordering helpers.  `from` must have finished what is enqueued on it so far
// before work enqueued on `to` after this call starts.
int order_after(es_handle* h, hipStream_t to, hipStream_t from, hipEvent_t ev)
{
    if (to == from) return ES_OK;
    ES_HIP(h, hipEventRecord(ev, from));
    ES_HIP(h, hipStreamWaitEvent(to, ev, 0));
    return ES_OK;
}

int sync_all(es_handle* h)
{
    ES_HIP(h, hipStreamSynchronize(h->s_main));
    if (h->s_ctx != h->s_main) ES_HIP(h, hipStreamSynchronize(h->s_ctx));
    if (h->s_stage != h->s_main && h->s_stage != h->s_ctx) ES_HIP(h, hipStreamSynchronize(h->s_stage));
    if (h->s_swap) ES_HIP(h, hipStreamSynchronize(h->s_swap));
    h->stage_pending = false;
    return ES_OK;
}

int check_ctx_call(es_handle* h, uint32_t est)
{
    if (!h || est >= h->N) return ES_EINVAL;
    if (h->seg_bytes.empty()) return ES_OK;
    if (!h->workers[h->worker_of[est]].bound) return ES_ESTATE;
    return ES_OK;
}

int aligned16(const void* p) { return (((uintptr_t)p) & 15) == 0; }

// true if two buffers of `bytes` bytes each share an address (null = absent buffer)
bool overlap(const void* a, const void* b, uint64_t bytes)
{
    if (!a || !b || bytes == 0) return false;
    const uintptr_t x = (uintptr_t)a, y = (uintptr_t)b;
    return x < y + bytes && y < x + bytes;
}

// Makes the handle's device current for the duration of a call and puts the
// caller's device back afterwards (the handle lives on the device that was
// current at es_init).
struct DeviceGuard {
    int prev = -1;
    bool switched = false;
    explicit DeviceGuard(const es_handle* h)
    {
        if (hipGetDevice(&prev) == hipSuccess && prev != h->device)
            switched = hipSetDevice(h->device) == hipSuccess;
    }
    ~DeviceGuard()
    {
        if (switched) (void)hipSetDevice(prev);
    }
    DeviceGuard(const DeviceGuard&) = delete;
    DeviceGuard& operator=(const DeviceGuard&) = delete;
};

// The two-buffer swap-in schedule: what is enqueued, in this order, on the copy queue ("fill")
// and on main ("reduce"), and the one operation of the other queue each has to wait for.
void swap_plan(uint32_t n_buckets, std::vector<es_swap_op>& ops)
{
    ops.clear();
    std::vector<int32_t> reduce_at(n_buckets, -1);
    for (uint32_t b = 0; b < n_buckets; ++b) {
        es_swap_op f;
        f.kind = ES_SWAP_FILL; f.bucket = b; f.half = b & 1;
        f.wait = b >= 2 ? reduce_at[b - 2] : -1;                  // the previous user of this buffer
        ops.push_back(f);
        es_swap_op r;
        r.kind = ES_SWAP_REDUCE; r.bucket = b; r.half = b & 1;
        r.wait = (int32_t)ops.size() - 1;                         // its own fill
        ops.push_back(r);
        reduce_at[b] = (int32_t)ops.size() - 1;
    }
}

void swap_release(es_handle* h)
{
    dev_release(h, h->d_swap_buf);        h->d_swap_buf = nullptr;
    dev_release(h, h->d_swap_tiles);      h->d_swap_tiles = nullptr;
    dev_release(h, (void*)h->d_swap_tables); h->d_swap_tables = nullptr;
    h->swap_ready = false;
}

// Device buffers, per-bucket tile tables and per-bucket pointer tables of the swap-in path.
int swap_prepare(es_handle* h)
{
    if (h->swap_ready) return ES_OK;
    swap_release(h);
    if (!h->s_swap) ES_HIP(h, hipStreamCreateWithFlags(&h->s_swap, hipStreamNonBlocking));
    for (int k = 0; k < 2; ++k) {
        if (!h->ev_filled[k]) ES_HIP(h, hipEventCreateWithFlags(&h->ev_filled[k], hipEventDisableTiming));
        if (!h->ev_consumed[k]) ES_HIP(h, hipEventCreateWithFlags(&h->ev_consumed[k], hipEventDisableTiming));
    }
    const size_t nb = h->buckets.size();
    uint64_t lmax = 0;
    for (const es_bucket& b : h->buckets) lmax = std::max<uint64_t>(lmax, b.len_elems);
    // a row starts as far into a 128-byte line as its bucket does in the flat space, so the tile
    // planner's line alignment holds in the buffer too
    h->swap_row = round_up(lmax + 32, 64);
    if (lmax) ES_HIP(h, dev_malloc(h, (void**)&h->d_swap_buf, 2 * (uint64_t)h->N * h->swap_row * sizeof(float)));
    std::vector<Tile> all;
    h->swap_tile_off.assign(nb, 0);
    h->swap_n_tiles.assign(nb, 0);
    h->swap_n_big.assign(nb, 0);
    const uint64_t TB = h->shape.big_unroll ? (uint64_t)kReduceBlock * h->shape.big_unroll * 4 : 0;
    for (size_t b = 0; b < nb; ++b) {
        std::vector<Tile> big, small;
        plan_tiles(std::vector<es_bucket>(1, h->buckets[b]), h->N, h->A, h->tile_elems, TB, big, small);
        h->swap_tile_off[b] = all.size();
        h->swap_n_big[b] = (uint32_t)big.size();
        h->swap_n_tiles[b] = (uint32_t)(big.size() + small.size());
        all.insert(all.end(), big.begin(), big.end());
        all.insert(all.end(), small.begin(), small.end());
    }
    if (!all.empty()) {
        ES_HIP(h, dev_malloc(h, (void**)&h->d_swap_tiles, all.size() * sizeof(Tile)));
        ES_HIP(h, hipMemcpy(h->d_swap_tiles, all.data(), all.size() * sizeof(Tile), hipMemcpyHostToDevice));
    }
    // rank r, bucket b, buffer `half`: the kernel forms table[r] + (flat offset), so a row's entry
    // is its start minus the bucket's flat offset; a rank whose slot is in HBM is read where it is
    std::vector<const float*> tab(2 * nb * h->N);
    for (int half = 0; half < 2; ++half)
        for (size_t b = 0; b < nb; ++b)
            for (uint32_t r = 0; r < h->N; ++r) {
                const Worker& w = h->workers[h->worker_of[r]];
                const float* entry = slot_base(h, r);
                if (w.grad_on_host) {
                    const uintptr_t row = (uintptr_t)(h->d_swap_buf + ((uint64_t)half * h->N + r) * h->swap_row +
                                                      (h->buckets[b].offset_elems & 31));
                    entry = (const float*)(row - h->buckets[b].offset_elems * sizeof(float));
                }
                tab[((size_t)half * nb + b) * h->N + r] = entry;
            }
    if (!tab.empty()) {
        ES_HIP(h, dev_malloc(h, (void**)&h->d_swap_tables, tab.size() * sizeof(float*)));
        ES_HIP(h, hipMemcpy((void*)h->d_swap_tables, tab.data(), tab.size() * sizeof(float*), hipMemcpyHostToDevice));
    }
    h->swap_ready = true;
    return ES_OK;
}

// The reduce of a job whose gradient slots (some or all) are in host memory, with swap-in.
int swap_reduce(es_handle* h, float* avg, float* p, float* v, float lr, float mu)
{
    int rc = swap_prepare(h);
    if (rc != ES_OK) return rc;
    const size_t nb = h->buckets.size();
    // the copy queue starts after every staging copy of the step and after main (in-place sources)
    if ((rc = order_after(h, h->s_swap, h->s_stage, h->ev_stage)) != ES_OK) return rc;
    if ((rc = order_after(h, h->s_swap, h->s_main, h->ev_main)) != ES_OK) return rc;
    h->stage_pending = false;
    std::vector<const float*> in_place(h->N, nullptr);
    for (size_t k = 0; k < h->in_place_rank.size(); ++k) in_place[h->in_place_rank[k]] = h->in_place_ptr[k];
    std::vector<es_swap_op> ops;
    swap_plan((uint32_t)nb, ops);
    for (const es_swap_op& op : ops) {
        const es_bucket& bk = h->buckets[op.bucket];
        if (op.kind == ES_SWAP_FILL) {
            if (op.wait >= 0) ES_HIP(h, hipStreamWaitEvent(h->s_swap, h->ev_consumed[op.half], 0));
            for (uint32_t r = 0; r < h->N && bk.len_elems; ++r) {
                const Worker& w = h->workers[h->worker_of[r]];
                const float* src = (in_place[r] ? in_place[r] : slot_base(h, r)) + bk.offset_elems;
                float* dst = w.grad_on_host
                                 ? h->d_swap_buf + ((uint64_t)op.half * h->N + r) * h->swap_row + (bk.offset_elems & 31)
                                 : slot_base(h, r) + bk.offset_elems;
                if (src == dst) continue;                       // a rank resident in HBM, read where it is
                ES_HIP(h, hipMemcpyAsync(dst, src, bk.len_elems * sizeof(float), hipMemcpyDefault, h->s_swap));
            }
            ES_HIP(h, hipEventRecord(h->ev_filled[op.half], h->s_swap));
        } else {
            ES_HIP(h, hipStreamWaitEvent(h->s_main, h->ev_filled[op.half], 0));
            ES_HIP(h, launch_ring_reduce(h->s_main, h->d_swap_tiles + h->swap_tile_off[op.bucket],
                                         h->swap_n_tiles[op.bucket], h->swap_n_big[op.bucket],
                                         h->d_swap_tables + ((size_t)op.half * nb + op.bucket) * h->N, h->N,
                                         avg, p, v, lr, mu, h->shape));
            ES_HIP(h, hipEventRecord(h->ev_consumed[op.half], h->s_main));
        }
    }
    return ES_OK;
}

}  // namespace

extern "C" {

int es_init(es_handle** out, uint32_t n_logical, const es_bucket_layout* lay)
{
    if (!out) return ES_EINVAL;
    int vrc = validate_layout(n_logical, lay);
    if (vrc != ES_OK) return vrc;

    es_handle* h = new (std::nothrow) es_handle;
    if (!h) return ES_ENOMEM;
    int rc = ES_OK;
    try {
        h->N = n_logical;
        h->P = lay->n_params;
        h->A = lay->chunk_align;
        h->dev_alloc = lay->dev_alloc;
        h->dev_free = lay->dev_free;
        h->user = lay->user;
        h->buckets.assign(lay->buckets, lay->buckets + lay->n_buckets);
        uint64_t off = 0;
        for (uint32_t j = 0; j < lay->n_state_segs; ++j) {
            h->seg_bytes.push_back(lay->state_seg_bytes[j]);
            h->seg_off.push_back(off);
            off += round_up(lay->state_seg_bytes[j], 16);
        }
        h->ctx_bytes = off;
        h->ctx_stride = round_up(off, kSlotAlignBytes);
        h->grad_stride = round_up(h->P * sizeof(float), kSlotAlignBytes) / sizeof(float);
        h->worker_of.assign(h->N, 0);
        h->slot_of.resize(h->N);
        for (uint32_t e = 0; e < h->N; ++e) h->slot_of[e] = e;
        h->accumulated.assign((size_t)h->N * h->buckets.size(), 0);
        // fewer ranks than the default batch: the largest power of two that fits, so that the
        // opening loads of a fold are still issued together (measured +4 % at N = 5..7)
        while (h->shape.rank_batch > 1 && (uint32_t)h->shape.rank_batch > h->N) h->shape.rank_batch /= 2;
        // many concurrent gradient streams: long contiguous reads per stream pay off (measured)
        if (h->N >= 11) { h->shape.big_unroll = 32; h->shape.big_rank_batch = 1; }
        // parameters + momentum that fit in the Infinity Cache and the L2s stay cacheable between
        // steps (measured crossover at N = 8: between 282 and 290 MiB)
        h->shape.nontemporal_pv = (2 * h->P * sizeof(float) > (284ull << 20)) ? 1 : 0;
        h->workers.resize(1);
        h->workers[0].live.assign(h->seg_bytes.size(), nullptr);
    } catch (const std::bad_alloc&) {
        delete h;
        return ES_ENOMEM;
    }
    hipError_t e = hipGetDevice(&h->device);
    if (e != hipSuccess) { delete h; return ES_EHIP; }
    if ((e = hipEventCreateWithFlags(&h->ev_main, hipEventDisableTiming)) != hipSuccess ||
        (e = hipEventCreateWithFlags(&h->ev_ctx, hipEventDisableTiming)) != hipSuccess ||
        (e = hipEventCreateWithFlags(&h->ev_stage, hipEventDisableTiming)) != hipSuccess) {
        es_destroy(h);
        return ES_EHIP;
    }
    rc = alloc_worker(h, h->workers[0], h->N);
    if (rc == ES_OK) rc = build_tiles(h);
    if (rc == ES_OK) rc = upload_slot_table(h);
    if (rc == ES_OK && h->P) {
        e = dev_malloc(h, (void**)&h->d_partials, ((h->P + 4095) / 4096) * sizeof(float));
        if (e != hipSuccess) rc = hip_fail(h, e);
    }
    if (rc != ES_OK) { es_destroy(h); return rc; }
    *out = h;
    return ES_OK;
}

int es_destroy(es_handle* h)
{
    if (!h) return ES_EINVAL;
    DeviceGuard guard__(h);
    (void)hipStreamSynchronize(h->s_main);
    (void)hipStreamSynchronize(h->s_ctx);
    (void)hipStreamSynchronize(h->s_stage);
    for (Worker& w : h->workers) free_worker(h, w);
    dev_release(h, h->d_tiles);
    dev_release(h, (void*)h->d_slots);
    dev_release(h, h->d_partials);
    if (h->s_swap) (void)hipStreamSynchronize(h->s_swap);
    swap_release(h);
    if (h->s_swap) (void)hipStreamDestroy(h->s_swap);
    for (int k = 0; k < 2; ++k) {
        if (h->ev_filled[k]) (void)hipEventDestroy(h->ev_filled[k]);
        if (h->ev_consumed[k]) (void)hipEventDestroy(h->ev_consumed[k]);
    }
    if (h->ev_main) (void)hipEventDestroy(h->ev_main);
    if (h->ev_ctx) (void)hipEventDestroy(h->ev_ctx);
    if (h->ev_stage) (void)hipEventDestroy(h->ev_stage);
    delete h;
    return ES_OK;
}

int es_set_streams(es_handle* h, void* main, void* ctx, void* stage)
{
    if (!h) return ES_EINVAL;
    DeviceGuard guard__(h);
    int rc = sync_all(h);
    if (rc != ES_OK) return rc;
    h->s_main = (hipStream_t)main;
    h->s_ctx = (hipStream_t)ctx;
    h->s_stage = (hipStream_t)stage;
    return ES_OK;
}

int es_plan_tiles(uint32_t n_logical, const es_bucket_layout* layout, uint32_t tile_elems,
                  uint32_t big_unroll, es_tile* out, uint64_t capacity, uint64_t* n_tiles,
                  uint64_t* n_big)
try {
    int rc = validate_layout(n_logical, layout);
    if (rc != ES_OK) return rc;
    if (tile_elems < 256 || tile_elems > 65536 || (tile_elems & 3)) return ES_EINVAL;
    if (big_unroll != 0 && big_unroll != 8 && big_unroll != 16 && big_unroll != 32) return ES_EINVAL;
    std::vector<es_bucket> buckets(layout->buckets, layout->buckets + layout->n_buckets);
    std::vector<Tile> big, small;
    plan_tiles(buckets, n_logical, layout->chunk_align, tile_elems,
               big_unroll ? (uint64_t)kReduceBlock * big_unroll * 4 : 0, big, small);
    if (n_tiles) *n_tiles = big.size() + small.size();
    if (n_big) *n_big = big.size();
    if (out) {
        if (capacity < big.size() + small.size()) return ES_EINVAL;
        uint64_t k = 0;
        for (const std::vector<Tile>* v : {&big, &small})
            for (const Tile& t : *v) {
                out[k].offset_elems = t.off;
                out[k].len_elems = t.len;
                out[k].start_rank = t.rank0;
                ++k;
            }
    }
    return ES_OK;
} catch (const std::bad_alloc&) {
    return ES_ENOMEM;
}

int es_plan_swap_in(uint32_t n_buckets, es_swap_op* out, uint64_t capacity, uint64_t* n_ops)
try {
    std::vector<es_swap_op> ops;
    swap_plan(n_buckets, ops);
    if (n_ops) *n_ops = ops.size();
    if (out) {
        if (capacity < ops.size()) return ES_EINVAL;
        std::copy(ops.begin(), ops.end(), out);
    }
    return ES_OK;
} catch (const std::bad_alloc&) {
    return ES_ENOMEM;
}

int es_set_grouping(es_handle* h, uint32_t n_workers, const uint32_t* worker_of_est,
                    const uint32_t* slot_of_est)
try {
    if (!h || !worker_of_est || !slot_of_est) return ES_EINVAL;
    DeviceGuard guard__(h);
    std::vector<uint32_t> counts;
    if (!valid_grouping(h->N, n_workers, worker_of_est, slot_of_est, counts)) return ES_EINVAL;
    if (h->n_accumulated != 0) return ES_ESTATE;
    int rc = sync_all(h);
    if (rc != ES_OK) return rc;

    std::vector<Worker> fresh(n_workers);
    const uint64_t hbm_before = h->hbm_grad_bytes;
    h->hbm_grad_bytes = 0;                       // placement is decided anew, worker by worker
    for (uint32_t w = 0; w < n_workers && rc == ES_OK; ++w) {
        fresh[w].live.assign(h->seg_bytes.size(), nullptr);
        rc = alloc_worker(h, fresh[w], counts[w]);
    }
    // carry every EST's small-state context over to its new slot
    if (rc == ES_OK && h->ctx_bytes) {
        for (uint32_t e = 0; e < h->N && rc == ES_OK; ++e) {
            uint8_t* dst = fresh[worker_of_est[e]].ctx_arena + (uint64_t)slot_of_est[e] * h->ctx_stride;
            hipError_t he = launch_copy_bytes(h->s_main, dst, ctx_base(h, e), h->ctx_bytes);
            if (he != hipSuccess) rc = hip_fail(h, he);
        }
        if (rc == ES_OK) {
            hipError_t he = hipStreamSynchronize(h->s_main);
            if (he != hipSuccess) rc = hip_fail(h, he);
        }
    }
    if (rc != ES_OK) {
        for (Worker& w : fresh) free_worker(h, w);
        h->hbm_grad_bytes = hbm_before;          // the previous grouping stays in force, with its placement
        return rc;
    }
    for (Worker& w : h->workers) free_worker(h, w);
    h->workers.swap(fresh);
    h->worker_of.assign(worker_of_est, worker_of_est + h->N);
    h->slot_of.assign(slot_of_est, slot_of_est + h->N);
    h->swap_ready = false;                       // slot addresses and placements have changed
    return upload_slot_table(h);
} catch (const std::bad_alloc&) {
    return ES_ENOMEM;
}

int es_bind_live_state(es_handle* h, uint32_t worker, void* const* live_ptrs)
try {
    if (!h || worker >= h->workers.size()) return ES_EINVAL;
    DeviceGuard guard__(h);
    const size_t ns = h->seg_bytes.size();
    if (ns && !live_ptrs) return ES_EINVAL;
    for (size_t j = 0; j < ns; ++j)
        if (!live_ptrs[j]) return ES_EINVAL;
    for (size_t j = 0; j < ns; ++j)                      // live tensors must not overlap
        for (size_t k = j + 1; k < ns; ++k) {
            const uintptr_t a = (uintptr_t)live_ptrs[j], b = (uintptr_t)live_ptrs[k];
            if (a < b + h->seg_bytes[k] && b < a + h->seg_bytes[j]) return ES_EINVAL;
        }
    int rc = sync_all(h);
    if (rc != ES_OK) return rc;
    Worker& w = h->workers[worker];
    std::vector<Piece> pieces;
    for (size_t j = 0; j < ns; ++j) {
        const uintptr_t p = (uintptr_t)live_ptrs[j];
        const uint64_t nb = h->seg_bytes[j];
        const uint32_t width = ((p | nb) & 15) == 0 ? 16 : ((p | nb) & 3) == 0 ? 4 : 1;
        for (uint64_t o = 0; o < nb; o += kPieceBytes) {
            Piece pc;
            pc.live = (void*)(p + o);
            pc.slot_off = h->seg_off[j] + o;
            pc.nbytes = (uint32_t)std::min<uint64_t>(kPieceBytes, nb - o);
            pc.width = width;
            pieces.push_back(pc);
        }
    }
    // the worker counts as unbound until the new table is in place
    w.bound = false;
    w.n_pieces = 0;
    if (w.d_pieces) { dev_release(h, w.d_pieces); w.d_pieces = nullptr; }
    if (!pieces.empty()) {
        ES_HIP(h, dev_malloc(h, (void**)&w.d_pieces, pieces.size() * sizeof(Piece)));
        ES_HIP(h, hipMemcpy(w.d_pieces, pieces.data(), pieces.size() * sizeof(Piece), hipMemcpyHostToDevice));
    }
    w.n_pieces = (uint32_t)pieces.size();
    w.live.assign(live_ptrs, live_ptrs + ns);
    w.bound = true;
    return ES_OK;
} catch (const std::bad_alloc&) {
    return ES_ENOMEM;
}

int es_ctx_restore(es_handle* h, uint32_t est)
{
    int rc = check_ctx_call(h, est);
    if (rc != ES_OK) return rc;
    DeviceGuard guard__(h);
    if (h->seg_bytes.empty()) return ES_OK;
    const Worker& w = h->workers[h->worker_of[est]];
    if ((rc = order_after(h, h->s_ctx, h->s_main, h->ev_main)) != ES_OK) return rc;
    ES_HIP(h, launch_ctx(h->s_ctx, w.d_pieces, w.n_pieces, ctx_base(h, est), nullptr, kRestore));
    return order_after(h, h->s_main, h->s_ctx, h->ev_ctx);
}

int es_ctx_save(es_handle* h, uint32_t est)
{
    int rc = check_ctx_call(h, est);
    if (rc != ES_OK) return rc;
    DeviceGuard guard__(h);
    if (h->seg_bytes.empty()) return ES_OK;
    const Worker& w = h->workers[h->worker_of[est]];
    if ((rc = order_after(h, h->s_ctx, h->s_main, h->ev_main)) != ES_OK) return rc;
    ES_HIP(h, launch_ctx(h->s_ctx, w.d_pieces, w.n_pieces, ctx_base(h, est), nullptr, kSave));
    return ES_OK;
}

int es_ctx_switch(es_handle* h, uint32_t est_out, uint32_t est_in)
{
    if (!h || est_out >= h->N || est_in >= h->N || est_out == est_in) return ES_EINVAL;
    DeviceGuard guard__(h);
    if (h->worker_of[est_out] != h->worker_of[est_in]) return ES_EINVAL;
    if (h->seg_bytes.empty()) return ES_OK;
    const Worker& w = h->workers[h->worker_of[est_out]];
    if (!w.bound) return ES_ESTATE;
    int rc = order_after(h, h->s_ctx, h->s_main, h->ev_main);
    if (rc != ES_OK) return rc;
    ES_HIP(h, launch_ctx(h->s_ctx, w.d_pieces, w.n_pieces, ctx_base(h, est_out), ctx_base(h, est_in), kSwitch));
    return order_after(h, h->s_main, h->s_ctx, h->ev_ctx);
}

float* es_grad_slot(es_handle* h, uint32_t est, uint32_t bucket)
{
    if (!h || est >= h->N || bucket >= h->buckets.size()) return nullptr;
    return slot_base(h, est) + h->buckets[bucket].offset_elems;
}

int es_accumulate(es_handle* h, uint32_t est, uint32_t bucket, const float* d_grad_bucket)
{
    if (!h || est >= h->N || bucket >= h->buckets.size()) return ES_EINVAL;
    DeviceGuard guard__(h);
    const uint64_t len = h->buckets[bucket].len_elems;
    if (len && (!d_grad_bucket || (((uintptr_t)d_grad_bucket) & 3))) return ES_EINVAL;
    uint8_t& flag = h->accumulated[(size_t)est * h->buckets.size() + bucket];
    if (flag) return ES_ESTATE;
    float* dst = es_grad_slot(h, est, bucket);
    if (len && d_grad_bucket != dst) {
        // a source that overlaps the destination slot without being it cannot be copied in one pass
        const uintptr_t a = (uintptr_t)d_grad_bucket, b = (uintptr_t)dst, n = len * sizeof(float);
        if (a < b + n && b < a + n) return ES_EINVAL;
        int rc = order_after(h, h->s_stage, h->s_main, h->ev_main);
        if (rc != ES_OK) return rc;
        if (dma_staging(h, est))
            ES_HIP(h, hipMemcpyAsync(dst, d_grad_bucket, len * sizeof(float), hipMemcpyDeviceToHost, h->s_stage));
        else
            ES_HIP(h, launch_copy_f32(h->s_stage, dst, d_grad_bucket, len));
        h->stage_pending = true;
    }
    flag = 1;
    h->n_accumulated++;
    return ES_OK;
}

namespace {

// A batch of buckets of one EST, checked as a whole: a failing call enqueues nothing and marks nothing.
int validate_batch(const es_handle* h, uint32_t est, uint32_t n, const uint32_t* buckets,
                   const float* const* srcs)
{
    if (est >= h->N || (n && (!buckets || !srcs))) return ES_EINVAL;
    const size_t nb = h->buckets.size();
    uint64_t blocks_bound = 0;               // workgroups of the whole batch: a bound on every launch's grid
    for (uint32_t k = 0; k < n; ++k) {
        const uint32_t b = buckets[k];
        if (b >= nb) return ES_EINVAL;
        const uint64_t len = h->buckets[b].len_elems;
        blocks_bound += ((len >> 2) + kCopyBlock - 1) / kCopyBlock + 1;
        if (blocks_bound > 0x7fffffffull) return ES_EINVAL;
        const float* src = srcs[k];
        if (len && (!src || (((uintptr_t)src) & 3))) return ES_EINVAL;
        for (uint32_t j = 0; j < k; ++j)
            if (buckets[j] == b) return ES_ESTATE;
        if (h->accumulated[(size_t)est * nb + b]) return ES_ESTATE;
        const float* dst = slot_base(h, est) + h->buckets[b].offset_elems;
        if (len && src != dst && overlap(src, dst, len * sizeof(float))) return ES_EINVAL;
    }
    return ES_OK;
}

// Staging copies as launches of at most kMaxRuns contiguous runs each.
struct RunBuilder {
    std::vector<CopyRuns> launches;
    void add(float* dst, const float* src, uint64_t len)
    {
        if (launches.empty()) open();
        CopyRuns* r = &launches.back();
        // extend the previous run when source and destination both continue it
        if (r->n_runs && r->src[r->n_runs - 1] + r->n[r->n_runs - 1] == src &&
            r->dst[r->n_runs - 1] + r->n[r->n_runs - 1] == dst &&
            r->first_block[r->n_runs - 1] + blocks_of(r->n[r->n_runs - 1] + len) <= 0x7fffffffull) {
            r->n[r->n_runs - 1] += len;
        } else {
            if (r->n_runs == (uint32_t)kMaxRuns || r->first_block[r->n_runs] + blocks_of(len) > 0x7fffffffull) {
                open();
                r = &launches.back();
            }
            r->dst[r->n_runs] = dst;
            r->src[r->n_runs] = src;
            r->n[r->n_runs] = len;
            ++r->n_runs;
        }
        r->first_block[r->n_runs] = r->first_block[r->n_runs - 1] + (uint32_t)blocks_of(r->n[r->n_runs - 1]);
    }
    static uint64_t blocks_of(uint64_t len)
    {
        const uint64_t blocks = ((len >> 2) + kCopyBlock - 1) / kCopyBlock;
        return blocks ? blocks : 1;
    }
    void open()
    {
        launches.emplace_back();
        CopyRuns& r = launches.back();
        r.n_runs = 0;
        for (int k = 0; k <= kMaxRuns; ++k) r.first_block[k] = 0xFFFFFFFFu;   // "no run starts here"
        r.first_block[0] = 0;
    }
};

void collect_runs(es_handle* h, uint32_t est, uint32_t n, const uint32_t* buckets, const float* const* srcs,
                  RunBuilder& rb)
{
    for (uint32_t k = 0; k < n; ++k) {
        const uint64_t len = h->buckets[buckets[k]].len_elems;
        float* dst = slot_base(h, est) + h->buckets[buckets[k]].offset_elems;
        if (len && srcs[k] != dst) rb.add(dst, srcs[k], len);
    }
}

int enqueue_staging(es_handle* h, const RunBuilder& rb, bool dma, size_t first_launch = 0)
{
    for (size_t k = first_launch; k < rb.launches.size(); ++k) {
        const CopyRuns& r = rb.launches[k];
        if (!dma) {
            ES_HIP(h, launch_copy_runs(h->s_stage, r));
            continue;
        }
        for (uint32_t j = 0; j < r.n_runs; ++j)
            ES_HIP(h, hipMemcpyAsync(r.dst[j], r.src[j], r.n[j] * sizeof(float), hipMemcpyDeviceToHost, h->s_stage));
    }
    return ES_OK;
}

void mark_batch(es_handle* h, uint32_t est, uint32_t n, const uint32_t* buckets)
{
    const size_t nb = h->buckets.size();
    for (uint32_t k = 0; k < n; ++k) h->accumulated[(size_t)est * nb + buckets[k]] = 1;
    h->n_accumulated += n;
}

}  // namespace

int es_accumulate_batch(es_handle* h, uint32_t est, uint32_t n, const uint32_t* buckets,
                        const float* const* d_grad_buckets)
try {
    if (!h) return ES_EINVAL;
    DeviceGuard guard__(h);
    int rc = validate_batch(h, est, n, buckets, d_grad_buckets);
    if (rc != ES_OK) return rc;
    RunBuilder rb;
    collect_runs(h, est, n, buckets, d_grad_buckets, rb);
    if (!rb.launches.empty()) {
        if ((rc = order_after(h, h->s_stage, h->s_main, h->ev_main)) != ES_OK) return rc;
        if ((rc = enqueue_staging(h, rb, dma_staging(h, est))) != ES_OK) return rc;
        h->stage_pending = true;
    }
    mark_batch(h, est, n, buckets);
    return ES_OK;
} catch (const std::bad_alloc&) {
    return ES_ENOMEM;
}

int es_accumulate_many(es_handle* h, uint32_t n_ests, const uint32_t* ests, const float* const* d_flat_grads)
try {
    if (!h || (n_ests && (!ests || !d_flat_grads))) return ES_EINVAL;
    DeviceGuard guard__(h);
    const size_t nb = h->buckets.size();
    const uint64_t vec_bytes = h->P * sizeof(float);
    if (RunBuilder::blocks_of(h->P) > 0x7fffffffull) return ES_EINVAL;
    for (uint32_t k = 0; k < n_ests; ++k) {
        const uint32_t e = ests[k];
        if (e >= h->N) return ES_EINVAL;
        const float* src = d_flat_grads[k];
        if (h->P && (!src || (((uintptr_t)src) & 3))) return ES_EINVAL;
        for (uint32_t j = 0; j < k; ++j)
            if (ests[j] == e) return ES_ESTATE;
        for (size_t b = 0; b < nb; ++b)
            if (h->accumulated[(size_t)e * nb + b]) return ES_ESTATE;
        if (h->P && src != slot_base(h, e) && overlap(src, slot_base(h, e), vec_bytes)) return ES_EINVAL;
    }
    RunBuilder rb, rb_dma;
    for (uint32_t k = 0; k < n_ests; ++k)
        if (h->P && d_flat_grads[k] != slot_base(h, ests[k]))
            (dma_staging(h, ests[k]) ? rb_dma : rb).add(slot_base(h, ests[k]), d_flat_grads[k], h->P);
    if (!rb.launches.empty() || !rb_dma.launches.empty()) {
        int rc = order_after(h, h->s_stage, h->s_main, h->ev_main);
        if (rc == ES_OK) rc = enqueue_staging(h, rb, false);
        if (rc == ES_OK) rc = enqueue_staging(h, rb_dma, true);
        if (rc != ES_OK) return rc;
        h->stage_pending = true;
    }
    for (uint32_t k = 0; k < n_ests; ++k)
        for (size_t b = 0; b < nb; ++b) h->accumulated[(size_t)ests[k] * nb + b] = 1;
    h->n_accumulated += (uint64_t)n_ests * nb;
    return ES_OK;
} catch (const std::bad_alloc&) {
    return ES_ENOMEM;
}

int es_est_boundary(es_handle* h, uint32_t est_out, uint32_t est_in, uint32_t n, const uint32_t* buckets,
                    const float* const* d_grad_buckets)
try {
    if (!h || est_out >= h->N) return ES_EINVAL;
    const bool has_in = est_in != ES_NO_EST;
    if (has_in && (est_in >= h->N || est_in == est_out)) return ES_EINVAL;
    DeviceGuard guard__(h);
    if (has_in && h->worker_of[est_out] != h->worker_of[est_in]) return ES_EINVAL;
    const Worker& w = h->workers[h->worker_of[est_out]];
    if (!h->seg_bytes.empty() && !w.bound) return ES_ESTATE;
    int rc = validate_batch(h, est_out, n, buckets, d_grad_buckets);
    if (rc != ES_OK) return rc;
    RunBuilder rb;
    collect_runs(h, est_out, n, buckets, d_grad_buckets, rb);
    const uint32_t n_pieces = h->seg_bytes.empty() ? 0 : w.n_pieces;
    if (h->s_stage != h->s_main) {
        // Staging has a stream of its own so that the copy overlaps the next EST's compute: one
        // fused launch would make main wait for the whole copy.  The copy goes to the stage
        // stream and the small-state switch where es_ctx_switch puts it; main waits for the
        // switch alone.
        if (!rb.launches.empty()) {
            if ((rc = order_after(h, h->s_stage, h->s_main, h->ev_main)) != ES_OK) return rc;
            if ((rc = enqueue_staging(h, rb, dma_staging(h, est_out))) != ES_OK) return rc;
            h->stage_pending = true;
        }
        mark_batch(h, est_out, n, buckets);
        if (n_pieces) {
            if ((rc = order_after(h, h->s_ctx, h->s_main, h->ev_main)) != ES_OK) return rc;
            ES_HIP(h, launch_ctx(h->s_ctx, w.d_pieces, n_pieces, ctx_base(h, est_out),
                                 has_in ? ctx_base(h, est_in) : nullptr, has_in ? kSwitch : kSave));
            if (has_in && (rc = order_after(h, h->s_main, h->s_ctx, h->ev_ctx)) != ES_OK) return rc;
        }
        return ES_OK;
    }
    if (n_pieces || !rb.launches.empty()) {
        // after the outgoing EST's compute on main and after earlier context traffic on the ctx stream
        if ((rc = order_after(h, h->s_stage, h->s_main, h->ev_main)) != ES_OK) return rc;
        if (h->s_ctx != h->s_main && (rc = order_after(h, h->s_stage, h->s_ctx, h->ev_ctx)) != ES_OK) return rc;
        const bool dma = dma_staging(h, est_out);
        RunBuilder none;
        none.open();
        if (rb.launches.empty()) rb.open();
        ES_HIP(h, launch_est_boundary(h->s_stage, dma ? none.launches[0] : rb.launches[0], w.d_pieces, n_pieces,
                                      ctx_base(h, est_out), has_in ? ctx_base(h, est_in) : nullptr,
                                      has_in ? kSwitch : kSave));
        if ((rc = enqueue_staging(h, rb, dma, dma ? 0 : 1)) != ES_OK) return rc;
        h->stage_pending = true;
    }
    mark_batch(h, est_out, n, buckets);
    // the incoming EST's compute on main must see its restored state
    if (has_in && n_pieces) {
        if ((rc = order_after(h, h->s_main, h->s_stage, h->ev_stage)) != ES_OK) return rc;
        h->stage_pending = false;
    }
    return ES_OK;
} catch (const std::bad_alloc&) {
    return ES_ENOMEM;
}

int es_accumulate_in_place(es_handle* h, uint32_t est, const float* d_flat_grad)
try {
    if (!h || est >= h->N) return ES_EINVAL;
    if (h->P && (!d_flat_grad || !aligned16(d_flat_grad))) return ES_EINVAL;
    const size_t nb = h->buckets.size();
    for (size_t b = 0; b < nb; ++b)
        if (h->accumulated[(size_t)est * nb + b]) return ES_ESTATE;
    h->in_place_rank.push_back(est);
    h->in_place_ptr.push_back(d_flat_grad);
    for (size_t b = 0; b < nb; ++b) h->accumulated[(size_t)est * nb + b] = 1;
    h->n_accumulated += nb;
    return ES_OK;
} catch (const std::bad_alloc&) {
    return ES_ENOMEM;
}

int es_stage_fence(es_handle* h)
{
    if (!h) return ES_EINVAL;
    DeviceGuard guard__(h);
    if (!h->stage_pending) return ES_OK;
    int rc = order_after(h, h->s_main, h->s_stage, h->ev_stage);
    if (rc == ES_OK) h->stage_pending = false;
    return rc;
}

int es_dropout_mask(es_handle* h, uint32_t est, uint32_t state_seg, uint8_t* d_mask, uint64_t n,
                    double p)
{
    if (!h || est >= h->N || state_seg >= h->seg_bytes.size()) return ES_EINVAL;
    DeviceGuard guard__(h);
    if (h->seg_bytes[state_seg] != 16 || (n && !d_mask) || !(p >= 0.0 && p <= 1.0)) return ES_EINVAL;
    const Worker& w = h->workers[h->worker_of[est]];
    if (!w.bound) return ES_ESTATE;
    if (((uintptr_t)w.live[state_seg]) & 7) return ES_EINVAL;
    uint64_t thr = p >= 1.0 ? (1ull << 32) : (uint64_t)(p * 4294967296.0);
    ES_HIP(h, launch_dropout_mask(h->s_main, (uint64_t*)w.live[state_seg], d_mask, n, thr));
    return ES_OK;
}

// Redirects the table entries of the ESTs taken in place, kMaxInPlace per launch: to the
// caller's gradients, or back to the ESTs' own slots.
static hipError_t patch_table(es_handle* h, bool to_caller)
{
    const size_t n = h->in_place_rank.size();
    for (size_t k0 = 0; k0 < n; k0 += kMaxInPlace) {
        InPlace patch{};
        patch.n = (uint32_t)std::min<size_t>(kMaxInPlace, n - k0);
        for (uint32_t k = 0; k < patch.n; ++k) {
            patch.rank[k] = h->in_place_rank[k0 + k];
            patch.ptr[k] = to_caller ? h->in_place_ptr[k0 + k] : slot_base(h, patch.rank[k]);
        }
        const hipError_t e = launch_patch_slots(h->s_main, h->d_slots, patch);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

static int reduce_common(es_handle* h, float* avg, float* p, float* v, float lr, float mu)
{
    if (h->n_accumulated != (uint64_t)h->N * h->buckets.size()) return ES_ESTATE;
    // gradients taken in place must not overlap what this launch writes
    for (size_t k = 0; k < h->in_place_ptr.size(); ++k) {
        const uintptr_t g = (uintptr_t)h->in_place_ptr[k], sz = h->P * sizeof(float);
        for (const float* o : {(const float*)avg, (const float*)p, (const float*)v}) {
            const uintptr_t b = (uintptr_t)o;
            if (o && g < b + sz && b < g + sz) return ES_EINVAL;
        }
    }
    bool any_on_host = false;
    for (const Worker& w : h->workers) any_on_host = any_on_host || w.grad_on_host;
    if (h->swap_in && any_on_host) {
        int src;
        try {
            src = swap_reduce(h, avg, p, v, lr, mu);
        } catch (const std::bad_alloc&) {
            return ES_ENOMEM;
        }
        if (src != ES_OK) return src;
        std::fill(h->accumulated.begin(), h->accumulated.end(), 0);
        h->n_accumulated = 0;
        h->in_place_rank.clear();
        h->in_place_ptr.clear();
        return ES_OK;
    }
    int rc = es_stage_fence(h);
    if (rc != ES_OK) return rc;
    // gradients taken in place: point their ranks at caller memory for this launch only, then
    // back at the slots, whether or not the launches in between worked.  The handle's record
    // of the caller's pointers is left as it is until the whole step has been enqueued, so a
    // reduce that failed can be called again and reads the same gradients.
    hipError_t status = patch_table(h, /*to_caller=*/true);
    if (status == hipSuccess)
        status = launch_ring_reduce(h->s_main, h->d_tiles, h->n_tiles, h->n_big, h->d_slots, h->N,
                                    avg, p, v, lr, mu, h->shape);
    const hipError_t restored = patch_table(h, /*to_caller=*/false);
    ES_HIP(h, status);
    ES_HIP(h, restored);
    std::fill(h->accumulated.begin(), h->accumulated.end(), 0);
    h->n_accumulated = 0;
    h->in_place_rank.clear();
    h->in_place_ptr.clear();
    return ES_OK;
}

int es_ring_order_reduce(es_handle* h, float* d_avg_grad)
{
    if (!h || (h->P && (!d_avg_grad || !aligned16(d_avg_grad)))) return ES_EINVAL;
    DeviceGuard guard__(h);
    return reduce_common(h, d_avg_grad, nullptr, nullptr, 0.f, 0.f);
}

int es_sgd_step(es_handle* h, float* d_param, float* d_momentum, const float* d_avg_grad,
                float lr, float mu)
{
    if (!h) return ES_EINVAL;
    DeviceGuard guard__(h);
    if (h->P && (!d_param || !d_momentum || !d_avg_grad)) return ES_EINVAL;
    if (!aligned16(d_param) || !aligned16(d_momentum) || !aligned16(d_avg_grad)) return ES_EINVAL;
    const uint64_t vec_bytes = h->P * sizeof(float);
    if (overlap(d_param, d_momentum, vec_bytes) || overlap(d_param, d_avg_grad, vec_bytes) ||
        overlap(d_momentum, d_avg_grad, vec_bytes))
        return ES_EINVAL;
    ES_HIP(h, launch_sgd(h->s_main, d_param, d_momentum, d_avg_grad, h->P, lr, mu, h->shape.nontemporal_pv != 0));
    return ES_OK;
}

int es_grad_sq_norm(es_handle* h, const float* d_vec, float* d_out2)
{
    if (!h || !d_out2 || (((uintptr_t)d_out2) & 3)) return ES_EINVAL;
    DeviceGuard guard__(h);
    if (h->P && (!d_vec || !aligned16(d_vec))) return ES_EINVAL;
    ES_HIP(h, launch_sq_norm(h->s_main, d_vec, h->P, h->d_partials, d_out2));
    return ES_OK;
}

int es_clip_sgd_step(es_handle* h, float* d_param, float* d_momentum, const float* d_avg_grad,
                     const float* d_norm2, float max_norm, float eps, float lr, float mu)
{
    if (!h) return ES_EINVAL;
    DeviceGuard guard__(h);
    if (!d_norm2 || (((uintptr_t)d_norm2) & 3) || !(max_norm >= 0.0f) || !(eps >= 0.0f)) return ES_EINVAL;
    if (h->P && (!d_param || !d_momentum || !d_avg_grad)) return ES_EINVAL;
    if (!aligned16(d_param) || !aligned16(d_momentum) || !aligned16(d_avg_grad)) return ES_EINVAL;
    const uint64_t vec_bytes = h->P * sizeof(float);
    if (overlap(d_param, d_momentum, vec_bytes) || overlap(d_param, d_avg_grad, vec_bytes) ||
        overlap(d_momentum, d_avg_grad, vec_bytes))
        return ES_EINVAL;
    ES_HIP(h, launch_sgd_clip(h->s_main, d_param, d_momentum, d_avg_grad, h->P, d_norm2, max_norm, eps, lr, mu,
                              h->shape.nontemporal_pv != 0));
    return ES_OK;
}

uint64_t es_bn_workspace_floats(uint64_t n_images, uint64_t n_channels, uint64_t n_positions)
{
    if (n_images == 0 || n_positions == 0) return 0;
    if (n_images > (1ull << 31) / n_positions) return 0;
    return n_channels * ((n_images * n_positions + 4095) / 4096);
}

int es_bn_batch_stats(const float* d_x, uint64_t n_images, uint64_t n_channels, uint64_t n_positions,
                      float* d_mean, float* d_var, float* d_workspace, uint64_t workspace_floats, void* stream)
{
    if (n_images == 0 || n_positions == 0 || n_channels > 65535) return ES_EINVAL;
    if (n_positions >= (1ull << 31) || n_images > ((1ull << 31) - 1) / n_positions) return ES_EINVAL;
    if (n_channels == 0) return ES_OK;
    if (!d_x || !d_mean || !d_var || !d_workspace) return ES_EINVAL;
    if ((((uintptr_t)d_x) | ((uintptr_t)d_mean) | ((uintptr_t)d_var) | ((uintptr_t)d_workspace)) & 3) return ES_EINVAL;
    if (workspace_floats < es_bn_workspace_floats(n_images, n_channels, n_positions)) return ES_EINVAL;
    return launch_bn_batch_stats((hipStream_t)stream, d_x, (uint32_t)n_images, (uint32_t)n_channels,
                                 (uint32_t)n_positions, d_mean, d_var, d_workspace) == hipSuccess
               ? ES_OK : ES_EHIP;
}

int es_grad_sq_norm_static(const float* d_vec, uint64_t n, float* d_out2, void* stream)
{
    if (!d_out2 || (((uintptr_t)d_out2) & 3)) return ES_EINVAL;
    if (n && (!d_vec || !aligned16(d_vec))) return ES_EINVAL;
    if ((n + 4095) / 4096 > kStaticPartials) return ES_EINVAL;
    return launch_sq_norm_static((hipStream_t)stream, d_vec, n, d_out2) == hipSuccess ? ES_OK : ES_EHIP;
}

int es_reduce_sgd_step(es_handle* h, float* d_param, float* d_momentum, float* d_avg_grad,
                       float lr, float mu)
{
    if (!h) return ES_EINVAL;
    DeviceGuard guard__(h);
    if (h->P && (!d_param || !d_momentum)) return ES_EINVAL;
    if (!aligned16(d_param) || !aligned16(d_momentum) || !aligned16(d_avg_grad)) return ES_EINVAL;
    const uint64_t vec_bytes = h->P * sizeof(float);
    if (overlap(d_param, d_momentum, vec_bytes) || overlap(d_param, d_avg_grad, vec_bytes) ||
        overlap(d_momentum, d_avg_grad, vec_bytes))
        return ES_EINVAL;
    return reduce_common(h, d_avg_grad, d_param, d_momentum, lr, mu);
}

namespace {
constexpr uint64_t kCkptMagic = 0x3130544B50435345ull;   // "ESCPKT01" as little-endian bytes

uint64_t ckpt_bytes(const es_handle* h)
{
    return 8 * sizeof(uint64_t) + h->buckets.size() * sizeof(es_bucket) +
           h->seg_bytes.size() * sizeof(uint64_t) + (uint64_t)h->N * h->ctx_bytes +
           2 * h->P * sizeof(float);
}
}  // namespace

uint64_t es_checkpoint_bytes(es_handle* h) { return h ? ckpt_bytes(h) : 0; }

int es_checkpoint_export(es_handle* h, void* host_blob, uint64_t capacity, const float* d_param,
                         const float* d_momentum, uint64_t global_step)
{
    if (!h || !host_blob || capacity < ckpt_bytes(h)) return ES_EINVAL;
    DeviceGuard guard__(h);
    if (h->P && (!d_param || !d_momentum)) return ES_EINVAL;
    if (h->n_accumulated != 0) return ES_ESTATE;
    int rc = sync_all(h);
    if (rc != ES_OK) return rc;
    uint8_t* out = (uint8_t*)host_blob;
    const uint64_t hdr[8] = {kCkptMagic, h->N, h->P, h->buckets.size(), h->A,
                             h->seg_bytes.size(), h->ctx_bytes, global_step};
    std::memcpy(out, hdr, sizeof(hdr));
    out += sizeof(hdr);
    if (!h->buckets.empty()) std::memcpy(out, h->buckets.data(), h->buckets.size() * sizeof(es_bucket));
    out += h->buckets.size() * sizeof(es_bucket);
    if (!h->seg_bytes.empty()) std::memcpy(out, h->seg_bytes.data(), h->seg_bytes.size() * sizeof(uint64_t));
    out += h->seg_bytes.size() * sizeof(uint64_t);
    if (h->ctx_bytes)
        for (uint32_t e = 0; e < h->N; ++e, out += h->ctx_bytes)
            ES_HIP(h, hipMemcpy(out, ctx_base(h, e), h->ctx_bytes, hipMemcpyDeviceToHost));
    if (h->P) {
        ES_HIP(h, hipMemcpy(out, d_param, h->P * sizeof(float), hipMemcpyDeviceToHost));
        out += h->P * sizeof(float);
        ES_HIP(h, hipMemcpy(out, d_momentum, h->P * sizeof(float), hipMemcpyDeviceToHost));
    }
    return ES_OK;
}

int es_checkpoint_import(es_handle* h, const void* host_blob, uint64_t size, float* d_param,
                         float* d_momentum, uint64_t* global_step)
{
    if (!h || !host_blob || size != ckpt_bytes(h)) return ES_EINVAL;
    DeviceGuard guard__(h);
    if (h->P && (!d_param || !d_momentum)) return ES_EINVAL;
    const uint8_t* in = (const uint8_t*)host_blob;
    uint64_t hdr[8];
    std::memcpy(hdr, in, sizeof(hdr));
    in += sizeof(hdr);
    if (hdr[0] != kCkptMagic || hdr[1] != h->N || hdr[2] != h->P || hdr[3] != h->buckets.size() ||
        hdr[4] != h->A || hdr[5] != h->seg_bytes.size() || hdr[6] != h->ctx_bytes)
        return ES_EINVAL;
    // the recorded bucket mapping and state shape must be the ones this job was created with
    if (!h->buckets.empty() && std::memcmp(in, h->buckets.data(), h->buckets.size() * sizeof(es_bucket)) != 0)
        return ES_EINVAL;
    in += h->buckets.size() * sizeof(es_bucket);
    if (!h->seg_bytes.empty() && std::memcmp(in, h->seg_bytes.data(), h->seg_bytes.size() * sizeof(uint64_t)) != 0)
        return ES_EINVAL;
    in += h->seg_bytes.size() * sizeof(uint64_t);
    if (h->n_accumulated != 0) return ES_ESTATE;
    int rc = sync_all(h);
    if (rc != ES_OK) return rc;
    if (h->ctx_bytes)
        for (uint32_t e = 0; e < h->N; ++e, in += h->ctx_bytes)
            ES_HIP(h, hipMemcpy(ctx_base(h, e), in, h->ctx_bytes, hipMemcpyHostToDevice));
    if (h->P) {
        ES_HIP(h, hipMemcpy(d_param, in, h->P * sizeof(float), hipMemcpyHostToDevice));
        in += h->P * sizeof(float);
        ES_HIP(h, hipMemcpy(d_momentum, in, h->P * sizeof(float), hipMemcpyHostToDevice));
    }
    if (global_step) *global_step = hdr[7];
    return ES_OK;
}

int es_sync(es_handle* h)
{
    if (!h) return ES_EINVAL;
    DeviceGuard guard__(h);
    return sync_all(h);
}

int es_set_option(es_handle* h, const char* name, int64_t value)
try {
    if (!h || !name) return ES_EINVAL;
    DeviceGuard guard__(h);
    const std::string k(name);
    if (k == "reduce_tile_elems") {
        if (value < 256 || value > 65536 || (value & 3)) return ES_EINVAL;
        int rc = sync_all(h);
        if (rc != ES_OK) return rc;
        const uint32_t old = h->tile_elems;
        h->tile_elems = (uint32_t)value;
        rc = build_tiles(h);
        if (rc != ES_OK) { h->tile_elems = old; (void)build_tiles(h); }
        return rc;
    }
    if (k == "reduce_big_unroll" || k == "reduce_big_rank_batch") {
        const bool u = k == "reduce_big_unroll";
        if (u && value != 0 && value != 8 && value != 16 && value != 32) return ES_EINVAL;
        if (!u && value != 1 && value != 2 && value != 4) return ES_EINVAL;
        int rc = sync_all(h);
        if (rc != ES_OK) return rc;
        int& field = u ? h->shape.big_unroll : h->shape.big_rank_batch;
        const int old = field;
        field = (int)value;
        if (h->shape.big_unroll * h->shape.big_rank_batch > 32) { field = old; return ES_EINVAL; }
        rc = build_tiles(h);
        if (rc != ES_OK) { field = old; (void)build_tiles(h); }
        return rc;
    }
    if (k == "reduce_lds_pad_kib") {
        if (value < -1 || value > 160) return ES_EINVAL;
        h->shape.lds_pad_kib = (int)value;
        return ES_OK;
    }
    if (k == "reduce_unroll") {
        if (value != 1 && value != 2 && value != 4) return ES_EINVAL;
        h->shape.unroll = (int)value;
        return ES_OK;
    }
    if (k == "reduce_rank_batch") {
        if (value != 1 && value != 2 && value != 4 && value != 8 && value != 16) return ES_EINVAL;
        h->shape.rank_batch = (int)value;
        return ES_OK;
    }
    if (k == "nontemporal") {
        if (value != 0 && value != 1) return ES_EINVAL;
        h->shape.nontemporal = (int)value;
        return ES_OK;
    }
    if (k == "swap_in") {
        if (value != 0 && value != 1) return ES_EINVAL;
        if (h->n_accumulated != 0) return ES_ESTATE;     // staged gradients would be read the other way
        int rc = sync_all(h);
        if (rc != ES_OK) return rc;
        h->swap_in = value != 0;
        if (!h->swap_in) swap_release(h);
        return ES_OK;
    }
    if (k == "host_slots") {
        if (value != 0 && value != 1) return ES_EINVAL;
        h->host_slots = value != 0;
        return ES_OK;
    }
    if (k == "hbm_slot_budget_mib") {
        if (value < -1 || value > (1ll << 40)) return ES_EINVAL;     // MiB: the byte count must fit 64 bits
        h->hbm_budget_mib = value;
        return ES_OK;
    }
    if (k == "nontemporal_pv") {
        if (value != 0 && value != 1) return ES_EINVAL;
        h->shape.nontemporal_pv = (int)value;
        return ES_OK;
    }
    return ES_EINVAL;
} catch (const std::bad_alloc&) {
    return ES_ENOMEM;
}

int es_get_option(es_handle* h, const char* name, int64_t* value)
{
    if (!h || !name || !value) return ES_EINVAL;
    const std::string k(name);
    if (k == "reduce_tile_elems") *value = h->tile_elems;
    else if (k == "reduce_unroll") *value = h->shape.unroll;
    else if (k == "reduce_rank_batch") *value = h->shape.rank_batch;
    else if (k == "nontemporal") *value = h->shape.nontemporal;
    else if (k == "nontemporal_pv") *value = h->shape.nontemporal_pv;
    else if (k == "reduce_lds_pad_kib") *value = h->shape.lds_pad_kib;
    else if (k == "host_slots") *value = h->host_slots ? 1 : 0;
    else if (k == "swap_in") *value = h->swap_in ? 1 : 0;
    else if (k == "hbm_slot_budget_mib") *value = h->hbm_budget_mib;
    else if (k == "slots_on_host") {             // read-only: ESTs whose gradient slot is in host memory now
        int64_t n = 0;
        for (uint32_t e = 0; e < h->N; ++e) n += h->workers[h->worker_of[e]].grad_on_host ? 1 : 0;
        *value = n;
    }
    else if (k == "reduce_big_unroll") *value = h->shape.big_unroll;
    else if (k == "reduce_big_rank_batch") *value = h->shape.big_rank_batch;
    else return ES_EINVAL;
    return ES_OK;
}

int es_query(es_handle* h, uint64_t* n_params, uint32_t* n_buckets, uint64_t* ctx_bytes,
             uint32_t* n_workers, uint64_t* n_reduce_tiles)
{
    if (!h) return ES_EINVAL;
    if (n_params) *n_params = h->P;
    if (n_buckets) *n_buckets = (uint32_t)h->buckets.size();
    if (ctx_bytes) *ctx_bytes = h->ctx_bytes;
    if (n_workers) *n_workers = (uint32_t)h->workers.size();
    if (n_reduce_tiles) *n_reduce_tiles = h->n_tiles;
    return ES_OK;
}

int es_last_hip_error(es_handle* h) { return h ? h->last_hip : 0; }

const char* es_strerror(int status)
{
    switch (status) {
    case ES_OK:     return "ok";
    case ES_EINVAL: return "invalid argument";
    case ES_ESTATE: return "call not valid in the current state";
    case ES_ENOMEM: return "out of memory";
    case ES_EHIP:   return "HIP call failed";
    default:        return "unknown status";
    }
}

#ifndef ES_SOURCE_HASH
#define ES_SOURCE_HASH "unknown"
#endif
const char* es_version(void) { return "libes 0.2 (gfx950) src:" ES_SOURCE_HASH; }

}  // extern "C"
