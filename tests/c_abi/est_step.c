/*
 * The EST step driven through the C boundary alone: no Python, no PyTorch.
 * A plain C host program allocates device memory with HIP, feeds seeded
 * gradients to libes, runs two global steps (staging, ring-ordered reduce,
 * SGD-momentum; second step fused and with the last EST taken in place) and
 * compares every output bit with the CPU oracle linked into the same program.
 * Test program: exit status 0 = bit-exact.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "es.h"

int  eso_ring_order_reduce(float *buf, uint64_t L, uint32_t N, uint32_t A, float *out);
void eso_sgd_momentum(float *p, float *v, const float *g, uint64_t n, float lr, float mu);

#define HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
    fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define ES(x) do { int s_ = (x); if (s_ != ES_OK) { \
    fprintf(stderr, "libes: %s (%d) at line %d\n", es_strerror(s_), s_, __LINE__); return 3; } } while (0)

static uint64_t rng_state = 0x5EED0C0DEull;
static float next_value(void)            /* xorshift64*, mapped to a wide range of magnitudes */
{
    rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
    uint64_t z = rng_state * 0x2545F4914F6CDD1Dull;
    int32_t m = (int32_t)(z >> 40) - (1 << 23);
    int e = (int)((z >> 8) & 15) - 8;
    return (float)m * (1.0f / (1 << 23)) * (float)(1 << (e + 8)) * (1.0f / 256.0f);
}

int main(void)
{
    enum { N = 5, NB = 4 };
    const es_bucket buckets[NB] = { {0, 3 * 4096 + 37}, {3 * 4096 + 37, 0}, {3 * 4096 + 37, 1001},
                                    {3 * 4096 + 37 + 1001, 40000} };
    const uint64_t P = 3 * 4096 + 37 + 1001 + 40000;
    const uint32_t A = 4;
    const float lr = 0.1f, mu = 0.9f;
    es_bucket_layout lay = { P, NB, buckets, A, 0, NULL, NULL, NULL, NULL };

    es_handle *h = NULL;
    ES(es_init(&h, N, &lay));

    float *hg = (float *)malloc(sizeof(float) * N * P);      /* this step's gradients, rank-major */
    float *hp = (float *)malloc(sizeof(float) * P), *hv = (float *)calloc(P, sizeof(float));
    float *ref_avg = (float *)malloc(sizeof(float) * P), *out = (float *)malloc(sizeof(float) * P);
    for (uint64_t i = 0; i < P; ++i) hp[i] = next_value();

    float *dg, *dp, *dv, *davg;
    HIP(hipMalloc((void **)&dg, sizeof(float) * N * P));
    HIP(hipMalloc((void **)&dp, sizeof(float) * P));
    HIP(hipMalloc((void **)&dv, sizeof(float) * P));
    HIP(hipMalloc((void **)&davg, sizeof(float) * P));
    HIP(hipMemcpy(dp, hp, sizeof(float) * P, hipMemcpyHostToDevice));
    HIP(hipMemset(dv, 0, sizeof(float) * P));

    for (int step = 0; step < 2; ++step) {
        for (uint64_t i = 0; i < (uint64_t)N * P; ++i) hg[i] = next_value();
        HIP(hipMemcpy(dg, hg, sizeof(float) * N * P, hipMemcpyHostToDevice));

        /* library */
        /* the ways of handing gradients over: several ESTs in one launch, one EST boundary in one
           launch, one bucket at a time, and in place */
        uint32_t first = 0;
        if (step == 0) {
            const uint32_t two[2] = { 0, 1 };
            const float *flat[2] = { dg, dg + P };
            ES(es_accumulate_many(h, 2, two, flat));
            first = 2;
        } else {
            uint32_t idx[NB];
            const float *src[NB];
            for (uint32_t b = 0; b < NB; ++b) { idx[b] = b; src[b] = dg + buckets[b].offset_elems; }
            ES(es_est_boundary(h, 0, ES_NO_EST, NB, idx, src));
            first = 1;
        }
        for (uint32_t e = first; e < N; ++e) {
            if (step == 1 && e == N - 1) { ES(es_accumulate_in_place(h, e, dg + (uint64_t)e * P)); continue; }
            for (uint32_t b = 0; b < NB; ++b)
                ES(es_accumulate(h, e, b, dg + (uint64_t)e * P + buckets[b].offset_elems));
        }
        if (step == 0) {
            ES(es_ring_order_reduce(h, davg));
            ES(es_sgd_step(h, dp, dv, davg, lr, mu));
        } else {
            ES(es_reduce_sgd_step(h, dp, dv, davg, lr, mu));
        }
        ES(es_sync(h));

        /* oracle: per bucket, ring all-reduce among N ranks, /N; then the update */
        for (uint32_t b = 0; b < NB; ++b) {
            const uint64_t L = buckets[b].len_elems, off = buckets[b].offset_elems;
            if (!L) continue;
            float *ranks = (float *)malloc(sizeof(float) * N * L);
            for (uint32_t r = 0; r < N; ++r) memcpy(ranks + r * L, hg + (uint64_t)r * P + off, sizeof(float) * L);
            if (eso_ring_order_reduce(ranks, L, N, A, ref_avg + off)) { fprintf(stderr, "oracle failed\n"); return 4; }
            free(ranks);
        }
        eso_sgd_momentum(hp, hv, ref_avg, P, lr, mu);

        struct { const char *name; const float *dev, *ref; } cmp[3] = {
            {"averaged gradient", davg, ref_avg}, {"parameters", dp, hp}, {"momentum", dv, hv} };
        for (int k = 0; k < 3; ++k) {
            HIP(hipMemcpy(out, cmp[k].dev, sizeof(float) * P, hipMemcpyDeviceToHost));
            if (memcmp(out, cmp[k].ref, sizeof(float) * P) != 0) {
                fprintf(stderr, "step %d: %s differs from the oracle\n", step, cmp[k].name);
                return 1;
            }
        }
    }
    ES(es_destroy(h));
    printf("c-abi: 2 global steps, N=%d, P=%llu: bit-exact with the oracle (%s)\n", N,
           (unsigned long long)P, es_version());
    return 0;
}
