/*
 * CPU oracle for the EasyScaleThread (EST) step.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, single-threaded C in IEEE binary32 (the precision the method
 * fixes).  It exists to say what the right bits are; the product (the HIP
 * library) never links, loads or calls it, and it shares no code with it.
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math (no FMA contraction, no
 * flush-to-zero), see oracle/__init__.py.
 *
 * What it follows
 *   - paper §3.2: every EST produces its own gradients; a global step ends
 *     when the gradients of all N ESTs are aggregated and the one shared
 *     replica of the parameters is updated.
 *   - paper §3.3 (D1): every EST has a constant virtual communication rank and
 *     the gradient->bucket mapping is fixed, so the aggregation is the one an
 *     N-rank DDP job would do, bucket by bucket.
 *   - the benchmark spec fixes what the paper leaves open: the all-reduce is
 *     the textbook ring (reduce-scatter then all-gather), the sum is divided
 *     by N afterwards, the update is SGD with momentum, the RNG is
 *     Philox4x32-10 (Salmon et al., SC'11).
 *
 * The ring is simulated as message passing: N rank-private buffers, explicit
 * per-step messages that are snapshotted before any receiver applies them.
 * Nothing here is blocked, fused or reordered.
 *
 * The "omp parallel for" pragmas are ignored by the default build (no -fopenmp),
 * which is the oracle the tests pin.  A second build of this same file with
 * -fopenmp exists only so that bench.py can also time it on all host cores: in
 * each ring step the N ranks post, and then consume, independently of one another
 * (that is what the message snapshot is for), and elementwise loops have no order,
 * so threads over ranks or elements change no operation and no operand.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ *
 * Chunk geometry of one bucket of L elements split among N ranks.
 * The paper is silent; reading: chunk length CL = ceil(L/N) rounded up to a
 * multiple of A, chunk c = [min(L,c*CL), min(L,(c+1)*CL)) (trailing chunks
 * may be short or empty).
 * ------------------------------------------------------------------ */
void eso_chunk_bounds(uint64_t L, uint32_t N, uint32_t A, uint32_t c,
                      uint64_t *lo, uint64_t *hi)
{
    uint64_t cl = (L + N - 1) / N;
    cl = (cl + A - 1) / A * A;
    uint64_t a = (uint64_t)c * cl, b = a + cl;
    *lo = a < L ? a : L;
    *hi = b < L ? b : L;
}

static uint32_t mod_n(int64_t x, uint32_t N)
{
    int64_t m = x % (int64_t)N;
    return (uint32_t)(m < 0 ? m + N : m);
}

/*
 * Ring all-reduce (sum) among N simulated ranks over one bucket.
 * buf holds the N rank-private copies back to back (rank r at buf + r*L) and
 * is updated in place; afterwards every rank holds the complete sums.
 *
 * Reduce-scatter, step s = 0..N-2: rank r sends its current chunk (r-s) mod N
 * to rank r+1; the receiver adds the message into its own copy of that chunk.
 * After the last step rank r owns the finished chunk (r+1) mod N.
 * All-gather, step s = 0..N-2: rank r sends chunk (r+1-s) mod N to rank r+1,
 * which overwrites its copy.
 *
 * Returns 0, or -1 on allocation failure.
 */
int eso_ring_allreduce(float *buf, uint64_t L, uint32_t N, uint32_t A)
{
    if (N <= 1 || L == 0)
        return 0;
    uint64_t lo, hi;
    eso_chunk_bounds(L, N, A, 0, &lo, &hi);
    uint64_t cl = hi - lo;                  /* chunk 0 is the longest */
    float *msg = (float *)malloc((size_t)N * cl * sizeof(float));
    if (!msg)
        return -1;

    for (int phase = 0; phase < 2; ++phase) {
        for (uint32_t s = 0; s + 1 < N; ++s) {
            /* every rank posts its message first ... */
            #pragma omp parallel for schedule(static)
            for (uint32_t r = 0; r < N; ++r) {
                uint64_t lo, hi;
                uint32_t c = mod_n((int64_t)r - s + phase, N);
                eso_chunk_bounds(L, N, A, c, &lo, &hi);
                memcpy(msg + (size_t)r * cl, buf + (size_t)r * L + lo, (hi - lo) * sizeof(float));
            }
            /* ... then every rank consumes the message of its left neighbour */
            #pragma omp parallel for schedule(static)
            for (uint32_t r = 0; r < N; ++r) {
                uint64_t lo, hi;
                uint32_t from = mod_n((int64_t)r - 1, N);
                uint32_t c = mod_n((int64_t)from - s + phase, N);
                eso_chunk_bounds(L, N, A, c, &lo, &hi);
                const float *in = msg + (size_t)from * cl;
                float *mine = buf + (size_t)r * L + lo;
                if (phase == 0) {
                    for (uint64_t i = 0; i < hi - lo; ++i)
                        mine[i] = in[i] + mine[i];
                } else {
                    memcpy(mine, in, (hi - lo) * sizeof(float));
                }
            }
        }
    }
    free(msg);
    return 0;
}

/*
 * One bucket of the EST-aware gradient all-reduce: ranks = virtual ranks of
 * the ESTs (paper §3.3 D1).  buf as above (clobbered).  Writes the averaged
 * gradient, sum / (float)N with one IEEE division per element, to out[L].
 * Returns 0; -1 on allocation failure; -2 if the N ranks do not end with
 * bit-identical buffers (would mean the simulation itself is broken).
 */
int eso_ring_order_reduce(float *buf, uint64_t L, uint32_t N, uint32_t A, float *out)
{
    int rc = eso_ring_allreduce(buf, L, N, A);
    if (rc)
        return rc;
    int differ = 0;
    #pragma omp parallel for schedule(static) reduction(|:differ)
    for (uint32_t r = 1; r < N; ++r)
        if (memcmp(buf, buf + (size_t)r * L, L * sizeof(float)) != 0)
            differ |= 1;
    if (differ)
        return -2;
    float n = (float)N;
    #pragma omp parallel for schedule(static)
    for (uint64_t i = 0; i < L; ++i)
        out[i] = buf[i] / n;
    return 0;
}

/*
 * SGD with momentum on the single shared replica (paper §3.2: parameters and
 * optimizer state are updated once per global step).  No dampening, no
 * Nesterov, no weight decay; v starts at zero and the same two lines are used
 * at every step; every multiply and add is rounded on its own (no FMA).
 *     v <- mu*v + g ;  p <- p - lr*v
 */
void eso_sgd_momentum(float *p, float *v, const float *g, uint64_t n, float lr, float mu)
{
    #pragma omp parallel for schedule(static)
    for (uint64_t i = 0; i < n; ++i) {
        float mv = mu * v[i];
        float vn = mv + g[i];
        float step = lr * vn;
        v[i] = vn;
        p[i] = p[i] - step;
    }
}

/* ------------------------------------------------------------------ *
 * Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as
 * easy as 1, 2, 3", SC'11): ten rounds; each round multiplies counter words
 * 0 and 2 by two fixed 32-bit constants, mixes the high halves with words 1
 * and 3 and the key, and the key is bumped by two Weyl constants between
 * rounds.
 * ------------------------------------------------------------------ */
void eso_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* keep-threshold for drop probability p: floor(p * 2^32), clamped to [0, 2^32] */
uint64_t eso_dropout_threshold(double p)
{
    if (!(p > 0.0))
        return 0;
    if (p >= 1.0)
        return (uint64_t)1 << 32;
    return (uint64_t)(p * 4294967296.0);
}

/*
 * Dropout keep-mask drawn from an EST's RNG state (the paper lists RNG state
 * as part of the EST context and Dropout as its consumer, §3.2-§3.3; the
 * mapping below is this build's own, not any framework's).
 * state = {seed, offset}.  Mask byte j is 1 (keep) iff word (j mod 4) of
 *   Philox(key = seed as (lo,hi), counter = (offset + j/4 as (lo,hi), 0, 0))
 * is >= threshold.  Afterwards offset += ceil(n/4).
 */
void eso_dropout_mask(uint64_t state[2], uint8_t *mask, uint64_t n, uint64_t threshold)
{
    uint32_t key[2] = { (uint32_t)state[0], (uint32_t)(state[0] >> 32) };
    uint64_t blocks = (n + 3) / 4;
    for (uint64_t b = 0; b < blocks; ++b) {
        uint64_t pos = state[1] + b;
        uint32_t ctr[4] = { (uint32_t)pos, (uint32_t)(pos >> 32), 0u, 0u };
        uint32_t w[4];
        eso_philox4x32_10(ctr, key, w);
        for (int k = 0; k < 4; ++k) {
            uint64_t j = 4 * b + k;
            if (j < n)
                mask[j] = (uint64_t)w[k] >= threshold ? 1 : 0;
        }
    }
    state[1] += blocks;
}

/* ------------------------------------------------------------------ *
 * Fixed-tree sum of squares of a flat vector (for a global gradient norm).
 * The paper's level D2 (section 3.3) asks for reductions whose result does not
 * depend on the GPU they run on; the paper fixes thread counts of existing
 * kernels, this build fixes the summation tree as a function of the data
 * size alone.  The tree (this build's own definition):
 *   - the vector is cut into blocks of 4096 elements, missing tail elements
 *     count as +0;
 *   - in a block, lane t (0..255) adds, starting from +0, the squares of the
 *     elements 4*(256*q + t) + c for q = 0..3 (outer) and c = 0..3 (inner);
 *   - the 256 lane sums are combined by v[t] = v[t] + v[t+s] for t < s,
 *     s = 128, 64, ..., 1; v[0] is the block's partial;
 *   - the block partials are combined the same way by one more block: lane t
 *     adds, from +0, partials t, t+256, t+512, ..., then the same tree.
 * Every square and every add is rounded to fp32 on its own.
 * ------------------------------------------------------------------ */
static float eso_tree256(float v[256])
{
    for (int s = 128; s >= 1; s >>= 1)
        for (int t = 0; t < s; ++t)
            v[t] = v[t] + v[t + s];
    return v[0];
}

float eso_tree_sumsq(const float *x, uint64_t n)
{
    uint64_t nblk = (n + 4095) / 4096;
    float *part = (float *)malloc((nblk ? nblk : 1) * sizeof(float));
    float v[256];
    for (uint64_t b = 0; b < nblk; ++b) {
        for (int t = 0; t < 256; ++t) {
            float s = 0.0f;
            for (int q = 0; q < 4; ++q)
                for (int c = 0; c < 4; ++c) {
                    uint64_t i = b * 4096 + 4 * (uint64_t)(256 * q + t) + c;
                    float e = i < n ? x[i] : 0.0f;
                    float sq = e * e;
                    s = s + sq;
                }
            v[t] = s;
        }
        part[b] = eso_tree256(v);
    }
    for (int t = 0; t < 256; ++t) {
        float s = 0.0f;
        for (uint64_t k = t; k < nblk; k += 256)
            s = s + part[k];
        v[t] = s;
    }
    float total = eso_tree256(v);
    free(part);
    return total;
}

/* ------------------------------------------------------------------ *
 * Gradient clipping by the global norm, folded into the update.  The paper
 * does not discuss clipping; this is the usual convention of training
 * frameworks, stated in full: the whole averaged gradient is multiplied by
 *     coef = min(1, max_norm / (norm + eps))
 * where norm is the square root of the fixed-tree sum of squares above; the
 * sum, the division and the product are each rounded to fp32.  With coef = 1
 * the product g * 1 is g itself, so an unclipped step equals eso_sgd_momentum.
 * ------------------------------------------------------------------ */
float eso_clip_coef(float norm, float max_norm, float eps)
{
    float d = norm + eps;
    float c = max_norm / d;
    return c < 1.0f ? c : 1.0f;
}

void eso_sgd_momentum_scaled(float *p, float *v, const float *g, uint64_t n, float lr, float mu, float coef)
{
    #pragma omp parallel for schedule(static)
    for (uint64_t i = 0; i < n; ++i) {
        float gs = coef * g[i];
        float mv = mu * v[i];
        float vn = mv + gs;
        float step = lr * vn;
        v[i] = vn;
        p[i] = p[i] - step;
    }
}

/* ------------------------------------------------------------------ *
 * BatchNorm batch statistics along the fixed tree (the paper's level D2,
 * section 3.3, asks of "reduce" that its result not depend on the GPU; BatchNorm
 * is the operator of section 3.3 whose statistics every EST tracks).
 * x is laid out [B][C][HW] (images, channels, spatial positions).  For channel
 * ch the M = B*HW values in the order (image, position) form a vector
 * y[m] = x[(m / HW) * C + ch][m % HW].  With T(f) the tree of eso_tree_sumsq
 * applied to the terms f(y[m]) instead of squares (blocks of 4096 terms, 256
 * lanes x (q outer, c inner), stride-halving, second stage over the block
 * partials; terms beyond M count as +0):
 *     mean[ch] = T(y) / (float)M
 *     var[ch]  = T((y - mean[ch])^2) / (float)M        (the biased variance)
 * every subtraction, square, add and division rounded to fp32.
 * ------------------------------------------------------------------ */
static float eso_tree_channel(const float *x, uint64_t C, uint64_t HW, uint64_t M, uint64_t ch,
                              int squared_deviation, float center)
{
    uint64_t nblk = (M + 4095) / 4096;
    float *part = (float *)malloc((nblk ? nblk : 1) * sizeof(float));
    float v[256];
    for (uint64_t b = 0; b < nblk; ++b) {
        for (int t = 0; t < 256; ++t) {
            float s = 0.0f;
            for (int q = 0; q < 4; ++q)
                for (int c = 0; c < 4; ++c) {
                    uint64_t m = b * 4096 + 4 * (uint64_t)(256 * q + t) + c;
                    float term = 0.0f;
                    if (m < M) {
                        float y = x[((m / HW) * C + ch) * HW + m % HW];
                        if (squared_deviation) {
                            float d = y - center;
                            term = d * d;
                        } else {
                            term = y;
                        }
                    }
                    s = s + term;
                }
            v[t] = s;
        }
        part[b] = eso_tree256(v);
    }
    for (int t = 0; t < 256; ++t) {
        float s = 0.0f;
        for (uint64_t k = t; k < nblk; k += 256)
            s = s + part[k];
        v[t] = s;
    }
    float total = eso_tree256(v);
    free(part);
    return total;
}

void eso_bn_batch_stats(const float *x, uint64_t B, uint64_t C, uint64_t HW, float *mean, float *var)
{
    uint64_t M = B * HW;
    float fm = (float)M;
    for (uint64_t ch = 0; ch < C; ++ch) {
        float mu = eso_tree_channel(x, C, HW, M, ch, 0, 0.0f) / fm;
        mean[ch] = mu;
        var[ch] = eso_tree_channel(x, C, HW, M, ch, 1, mu) / fm;
    }
}
