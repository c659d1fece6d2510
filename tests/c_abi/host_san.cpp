// Host runtime of libes under AddressSanitizer / UBSan without a GPU: the kernel launchers
// are stubbed out, so only the host logic runs (layout validation, tile planning, argument
// checks).  Test program; exit status 0 = clean.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "es.h"
#include "es_internal.h"
#include "es_sched.h"

namespace es {
hipError_t launch_ring_reduce(hipStream_t, const Tile*, uint32_t, uint32_t, const float* const*, uint32_t,
                              float*, float*, float*, float, float, ReduceShape) { return hipSuccess; }
hipError_t launch_sgd(hipStream_t, float*, float*, const float*, uint64_t, float, float, bool) { return hipSuccess; }
hipError_t launch_copy_f32(hipStream_t, float*, const float*, uint64_t) { return hipSuccess; }
hipError_t launch_copy_runs(hipStream_t, const CopyRuns&) { return hipSuccess; }
hipError_t launch_patch_slots(hipStream_t, const float**, const InPlace&) { return hipSuccess; }
hipError_t launch_ctx(hipStream_t, const Piece*, uint32_t, uint8_t*, const uint8_t*, CtxDir) { return hipSuccess; }
hipError_t launch_est_boundary(hipStream_t, const CopyRuns&, const Piece*, uint32_t, uint8_t*, const uint8_t*, CtxDir) { return hipSuccess; }
hipError_t launch_sgd_clip(hipStream_t, float*, float*, const float*, uint64_t, const float*, float, float, float, float, bool) { return hipSuccess; }
hipError_t launch_bn_batch_stats(hipStream_t, const float*, uint32_t, uint32_t, uint32_t, float*, float*, float*) { return hipSuccess; }
hipError_t launch_copy_bytes(hipStream_t, uint8_t*, const uint8_t*, uint64_t) { return hipSuccess; }
hipError_t launch_sq_norm(hipStream_t, const float*, uint64_t, float*, float*) { return hipSuccess; }
hipError_t launch_sq_norm_static(hipStream_t, const float*, uint64_t, float*) { return hipSuccess; }
hipError_t launch_dropout_mask(hipStream_t, uint64_t*, uint8_t*, uint64_t, uint64_t) { return hipSuccess; }
}  // namespace es

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c); return 1; } } while (0)

int main()
{
    unsigned planned = 0;
    const uint32_t Ns[] = {1, 2, 3, 7, 16, 64, 1000};
    const uint64_t lens[][4] = {{0, 0, 0, 0}, {1, 0, 3, 5}, {4096, 4097, 0, 12}, {100003, 7, 32768 * 3 + 1, 2048},
                                {1u << 20, 3, 0, (1u << 18) + 5}};
    for (uint32_t N : Ns)
        for (const auto& l : lens)
            for (uint32_t A : {1u, 4u, 64u})
                for (uint32_t tile : {256u, 2048u, 65536u})
                    for (uint32_t big : {0u, 8u, 32u}) {
                        es_bucket b[4];
                        uint64_t off = 0;
                        for (int k = 0; k < 4; ++k) { b[k] = {off, l[k]}; off += l[k]; }
                        es_bucket_layout lay = {off, 4, b, A, 0, nullptr, nullptr, nullptr, nullptr};
                        uint64_t nt = 0, nb = 0;
                        CHECK(es_plan_tiles(N, &lay, tile, big, nullptr, 0, &nt, &nb) == ES_OK);
                        std::vector<es_tile> t(nt + 1);
                        CHECK(es_plan_tiles(N, &lay, tile, big, t.data(), nt, &nt, &nb) == ES_OK);
                        uint64_t sum = 0;
                        for (uint64_t k = 0; k < nt; ++k) { sum += t[k].len_elems; CHECK(t[k].start_rank < N); }
                        CHECK(sum == off && nb <= nt);
                        if (nt) CHECK(es_plan_tiles(N, &lay, tile, big, t.data(), nt - 1, &nt, &nb) == ES_EINVAL);
                        ++planned;
                    }
    // argument validation never touches memory it was not given
    es_handle* h = nullptr;
    es_bucket one = {0, 8}, gap[2] = {{0, 4}, {5, 3}};
    es_bucket_layout ok = {8, 1, &one, 1, 0, nullptr, nullptr, nullptr, nullptr}, bad = {8, 2, gap, 1, 0, nullptr, nullptr, nullptr, nullptr};
    CHECK(es_init(nullptr, 2, &ok) == ES_EINVAL);
    CHECK(es_init(&h, 0, &ok) == ES_EINVAL && h == nullptr);
    CHECK(es_init(&h, 2, &bad) == ES_EINVAL && h == nullptr);
    CHECK(es_init(&h, 2, nullptr) == ES_EINVAL);
    int rc = es_init(&h, 2, &ok);            // without a GPU this fails cleanly; with one it succeeds
    CHECK((rc == ES_OK && h) || (rc != ES_OK && !h));
    if (h) CHECK(es_destroy(h) == ES_OK);
    CHECK(es_sync(nullptr) == ES_EINVAL && es_destroy(nullptr) == ES_EINVAL);
    CHECK(es_checkpoint_bytes(nullptr) == 0);
    // the swap-in schedule: every fill waits for the reduce two buckets back, every reduce for its fill
    for (uint32_t nbk : {0u, 1u, 2u, 3u, 37u, 1000u}) {
        uint64_t n_ops = 0;
        CHECK(es_plan_swap_in(nbk, nullptr, 0, &n_ops) == ES_OK && n_ops == 2ull * nbk);
        std::vector<es_swap_op> ops(n_ops + 1);
        CHECK(es_plan_swap_in(nbk, ops.data(), n_ops, &n_ops) == ES_OK);
        for (uint64_t k = 0; k < n_ops; ++k) {
            CHECK(ops[k].bucket == k / 2 && ops[k].half == (k / 2) % 2 && ops[k].kind == (k % 2 ? ES_SWAP_REDUCE : ES_SWAP_FILL));
            CHECK(ops[k].wait == (k % 2 ? (int32_t)k - 1 : (k >= 4 ? (int32_t)k - 3 : -1)));
        }
        if (n_ops) CHECK(es_plan_swap_in(nbk, ops.data(), n_ops - 1, &n_ops) == ES_EINVAL);
    }
    // handle-free entry points reject bad sizes before any device work
    CHECK(es_bn_workspace_floats(32, 64, 12544) == 64 * 98 && es_bn_workspace_floats(0, 1, 1) == 0);
    CHECK(es_bn_workspace_floats(1ull << 20, 2, 1ull << 12) == 0);
    CHECK(es_bn_batch_stats(nullptr, 2, 2, 8, nullptr, nullptr, nullptr, 0, nullptr) == ES_EINVAL);
    CHECK(es_grad_sq_norm_static(nullptr, (1ull << 30) + 1, nullptr, nullptr) == ES_EINVAL);
    // scheduler-side planner: bit-set edges, clipped caps, ranking buffer of every size
    unsigned searched = 0;
    const double C[3] = {9.5, 4.25, 0.75};
    for (uint32_t max_p : {1u, 2u, 63u, 64u, 65u, 129u, 1000u, (unsigned)ES_SCHED_MAX_P})
        for (uint32_t top_k : {1u, 2u, 7u, 64u}) {
            const uint32_t avail[3] = {3, 2, 2};
            std::vector<es_sched_plan> plans(top_k);
            uint32_t n = 0;
            CHECK(es_sched_enumerate(3, C, avail, max_p, top_k, plans.data(), &n) == ES_OK && n <= top_k);
            for (uint32_t k = 0; k < n; ++k) {
                CHECK(plans[k].n_est >= max_p && plans[k].n_gpus >= 1 && plans[k].n_gpus <= max_p);
                std::vector<uint32_t> wo(max_p), so(max_p);
                uint32_t nw = 0;
                CHECK(es_sched_grouping(3, &plans[k], max_p, wo.data(), so.data(), &nw) == ES_OK);
                CHECK(nw == plans[k].n_gpus && wo[max_p - 1] == nw - 1);
                es_sched_plan again;
                CHECK(es_sched_evaluate(3, C, plans[k].n_used, plans[k].est_per_gpu, max_p,
                                        ES_SCHED_WASTE_PER_GPU, &again) == ES_OK);
                CHECK(again.throughput == plans[k].throughput && again.n_est == plans[k].n_est);
                ++searched;
            }
        }
    CHECK(searched > 0);
    std::printf("host runtime sanitizer run: %u plans clean\n", planned);
    return 0;
}
