/* Runs the C oracle over awkward sizes under AddressSanitizer / UBSan (host only). */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void eso_chunk_bounds(uint64_t L, uint32_t N, uint32_t A, uint32_t c, uint64_t *lo, uint64_t *hi);
int eso_ring_order_reduce(float *buf, uint64_t L, uint32_t N, uint32_t A, float *out);
void eso_sgd_momentum(float *p, float *v, const float *g, uint64_t n, float lr, float mu);
void eso_dropout_mask(uint64_t state[2], uint8_t *mask, uint64_t n, uint64_t threshold);
float eso_tree_sumsq(const float *x, uint64_t n);

int main(void)
{
    const uint32_t Ns[] = {1, 2, 3, 5, 8, 17, 64};
    const uint64_t Ls[] = {0, 1, 2, 3, 4, 5, 7, 8, 63, 64, 65, 127, 1000, 4099};
    const uint32_t As[] = {1, 2, 4, 64};
    unsigned checked = 0;
    for (unsigned a = 0; a < sizeof(Ns) / sizeof(*Ns); ++a)
        for (unsigned b = 0; b < sizeof(Ls) / sizeof(*Ls); ++b)
            for (unsigned c = 0; c < sizeof(As) / sizeof(*As); ++c) {
                const uint32_t N = Ns[a], A = As[c];
                const uint64_t L = Ls[b];
                float *buf = (float *)malloc(sizeof(float) * (N * L + 1));   /* exact size: overruns trip ASan */
                float *out = (float *)malloc(sizeof(float) * (L + 1));
                for (uint64_t i = 0; i < N * L; ++i) buf[i] = (float)((i * 2654435761u) % 1000) - 500.0f;
                if (eso_ring_order_reduce(buf, L, N, A, out)) return 1;
                uint64_t lo, hi, prev = 0;
                for (uint32_t k = 0; k < N; ++k) {
                    eso_chunk_bounds(L, N, A, k, &lo, &hi);
                    if (lo != prev || hi < lo || hi > L) return 2;
                    prev = hi;
                }
                if (prev != L) return 3;
                float *p = (float *)calloc(L + 1, sizeof(float)), *v = (float *)calloc(L + 1, sizeof(float));
                eso_sgd_momentum(p, v, out, L, 0.1f, 0.9f);
                uint8_t *mask = (uint8_t *)malloc(L + 1);
                uint64_t st[2] = {N * 7919u + L, (uint64_t)-3};              /* offset wraps 64 bits */
                eso_dropout_mask(st, mask, L, (uint64_t)429496729);
                (void)eso_tree_sumsq(out, L);
                free(buf); free(out); free(p); free(v); free(mask);
                ++checked;
            }
    float *big = (float *)malloc(sizeof(float) * (256 * 4096 + 5));
    for (int i = 0; i < 256 * 4096 + 5; ++i) big[i] = 1.0f;
    if (eso_tree_sumsq(big, 256 * 4096 + 5) != (float)(256 * 4096 + 5)) return 4;
    free(big);
    printf("oracle sanitizer run: %u geometries clean\n", checked);
    return 0;
}
