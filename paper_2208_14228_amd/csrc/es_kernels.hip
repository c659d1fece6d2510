// gfx950 (CDNA4) kernels of the EST step.  Wave size 64; 256-lane workgroups except
// the staging copies, which run one wave per workgroup.
//
// Bit-exactness rules that hold for every kernel in this file:
//  - fp32 IEEE arithmetic, denormals kept, no fused multiply-add (the file is
//    compiled with -ffp-contract=off), division correctly rounded;
//  - no atomics; no arithmetic across lanes: a sum over N ranks is a chain of
//    N-1 adds in one lane in program order, so neither the grid shape nor the
//    order in which loads return can change a bit;
//  - loads may be issued early and in any order, only the add chain is ordered.
#include "es_internal.h"

#include <mutex>

namespace es {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

// Tables that every lane of a workgroup reads at the same index live in the
// constant address space so the reads are scalar loads shared by the wave.
#define ES_CONST_AS __attribute__((address_space(4)))
#pragma clang diagnostic ignored "-Wold-style-cast"

template <bool NT>
__device__ __forceinline__ f4 ld4(const float* p)
{
    const f4* q = reinterpret_cast<const f4*>(p);
    if constexpr (NT)
        return __builtin_nontemporal_load(q);
    else
        return *q;
}

__device__ __forceinline__ void st4(float* p, f4 x) { *reinterpret_cast<f4*>(p) = x; }

// Parameter / momentum traffic of the update, and the store of the averaged
// gradient.  Touched once per global step: when the vectors fit in the 256 MB
// Infinity Cache they are left cacheable and come back from it (parameters and
// momentum in the next step, measured +13 % at P = 25.6 M; the averaged gradient
// in the update kernel that follows an unfused reduce); when they do not,
// streaming accesses are faster (fused: +6 % at P = 109 M; the unfused reduce:
// +11 % at P = 109 M, N = 16 and +13 % at P = 355 M, N = 64 from the store of the
// averaged gradient alone).
template <bool NTPV>
__device__ __forceinline__ f4 ld4_pv(const float* p)
{
    if constexpr (NTPV) return __builtin_nontemporal_load(reinterpret_cast<const f4*>(p));
    else return *reinterpret_cast<const f4*>(p);
}
template <bool NTPV>
__device__ __forceinline__ void st4_pv(float* p, f4 x)
{
    if constexpr (NTPV) __builtin_nontemporal_store(x, reinterpret_cast<f4*>(p));
    else *reinterpret_cast<f4*>(p) = x;
}

// ---------------------------------------------------------------------------
// Ring-ordered N-way reduce (paper §3.3 D1: aggregation order fixed by the
// ESTs' constant virtual ranks), optionally fused with the SGD-momentum update
// of the shared replica (paper §3.2).
//
// One workgroup = one Tile (a range inside one ring chunk).  Chunk c's sum is
// the left fold over ranks c, c+1, ..., c+N-1 (mod N): what the reduce-scatter
// of an N-rank ring computes when rank r sends to r+1 and first sends its own
// chunk.  Each lane keeps U independent 16-byte accumulators and loads NB ranks
// ahead of the adds.
// ---------------------------------------------------------------------------
template <int U, int NB, int NT, bool FIRST>
__device__ __forceinline__ void fold_batch(const float* const ES_CONST_AS* slots, uint32_t N,
                                           uint32_t r0, const uint64_t (&e)[U], f4 (&acc)[U])
{
    // ranks r0 .. r0+NB-1 (mod N): all loads first, then the adds in rank order
    f4 x[NB][U];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        uint32_t r = r0 + j;
        if (r >= N) r -= N;
        const float* g = slots[r];
#pragma unroll
        for (int u = 0; u < U; ++u) x[j][u] = ld4<(NT & 1) != 0>(g + e[u]);
    }
    // keep every load of the batch ahead of the first add: the batch is the
    // wave's bytes in flight
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < NB; ++j) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (FIRST && j == 0)
                acc[u] = x[0][u];                          // the fold opens with rank c itself
            else
                acc[u] = acc[u] + x[j][u];
        }
    }
}

// The last N - k < 2*NBX ranks of a fold, in batches of NBX, NBX/2, .. 1 (same order of adds).
template <int U, int NBX, int NT>
__device__ __forceinline__ void fold_rest(const float* const ES_CONST_AS* slots, uint32_t N, uint32_t rank0,
                                          uint32_t& k, const uint64_t (&e)[U], f4 (&acc)[U])
{
    if constexpr (NBX >= 1) {
        if (k + NBX <= N) {
            uint32_t r0 = rank0 + k;
            if (r0 >= N) r0 -= N;
            fold_batch<U, NBX, NT, false>(slots, N, r0, e, acc);
            k += NBX;
        }
        fold_rest<U, NBX / 2, NT>(slots, N, rank0, k, e, acc);
    }
}

template <bool SGD>
__device__ __forceinline__ void finish_scalar(float acc, float fN, uint64_t e, float* avg,
                                              float* p, float* v, float lr, float mu)
{
    const float a = acc / fN;
    if (avg) avg[e] = a;
    if constexpr (SGD) {
        const float mv = mu * v[e];
        const float vn = mv + a;
        const float st = lr * vn;
        v[e] = vn;
        p[e] = p[e] - st;
    }
}

template <bool SGD>
__device__ __forceinline__ void fold_scalar(const float* const ES_CONST_AS* slots, uint32_t N,
                                            uint32_t rank0, float fN, uint64_t e, float* avg,
                                            float* p, float* v, float lr, float mu)
{
    uint32_t r = rank0;
    float acc = slots[r][e];
    for (uint32_t k = 1; k < N; ++k) {
        r = (r + 1 == N) ? 0 : r + 1;
        acc = acc + slots[r][e];
    }
    finish_scalar<SGD>(acc, fN, e, avg, p, v, lr, mu);
}

template <int U, int NB, int NT, bool SGD>
__device__ __forceinline__ void small_tile(const float* const ES_CONST_AS* slots, uint32_t N,
                                           uint64_t off, uint32_t len, uint32_t rank0,
                                           float* __restrict__ avg, float* __restrict__ p,
                                           float* __restrict__ v, float lr, float mu)
{
    const float fN = (float)N;

    // 16-byte vectors need element offsets that are multiples of 4 (all slot,
    // avg, p and v bases are 16-byte aligned): up to 3 leading and 3 trailing
    // elements of a tile take the scalar path.
    uint32_t head = (uint32_t)((4 - (off & 3)) & 3);
    if (head > len) head = len;
    const uint32_t nvec = (len - head) >> 2;
    const uint64_t vbase = off + head;
    const uint32_t tail = len - head - 4 * nvec;

    for (uint32_t i0 = threadIdx.x; i0 < nvec; i0 += kReduceBlock * U) {
        uint64_t e[U];
        bool ok[U];
        f4 acc[U], pp[U], vv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t i = i0 + u * kReduceBlock;
            ok[u] = i < nvec;
            // a lane without work in this pass re-reads the tile's last vector
            // (in bounds, result dropped) so that no load needs a predicate
            e[u] = vbase + 4ull * (ok[u] ? i : nvec - 1);
        }
        if constexpr (SGD) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                pp[u] = ld4_pv<(NT & 2) != 0>(p + e[u]);
                vv[u] = ld4_pv<(NT & 2) != 0>(v + e[u]);
            }
        }
        // N = q*NB + rem ranks: q full batches, then the rest in batches of NB/2, NB/4, .. 1
        // (a remainder taken one rank at a time leaves the wave with a single rank's loads in
        // flight: measured -10 % at N = 12 when one workgroup has a CU to itself)
        uint32_t k;
        if (N >= (uint32_t)NB) {
            fold_batch<U, NB, NT, true>(slots, N, rank0, e, acc);
            k = NB;
        } else {
            fold_batch<U, 1, NT, true>(slots, N, rank0, e, acc);
            k = 1;
        }
        for (; k + NB <= N; k += NB) {
            uint32_t r0 = rank0 + k;
            if (r0 >= N) r0 -= N;
            fold_batch<U, NB, NT, false>(slots, N, r0, e, acc);
        }
        fold_rest<U, NB / 2, NT>(slots, N, rank0, k, e, acc);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (!ok[u]) continue;
            const f4 a = acc[u] / fN;
            if (avg) st4_pv<(NT & 2) != 0>(avg + e[u], a);
            if constexpr (SGD) {
                const f4 mv = mu * vv[u];
                const f4 vn = mv + a;
                const f4 st = lr * vn;
                st4_pv<(NT & 2) != 0>(v + e[u], vn);
                st4_pv<(NT & 2) != 0>(p + e[u], pp[u] - st);
            }
        }
    }
    if (threadIdx.x < head)
        fold_scalar<SGD>(slots, N, rank0, fN, off + threadIdx.x, avg, p, v, lr, mu);
    if (threadIdx.x < tail)
        fold_scalar<SGD>(slots, N, rank0, fN, vbase + 4ull * nvec + threadIdx.x, avg, p, v, lr, mu);
}

template <int U, int NB, int NT, bool SGD>
__global__ __launch_bounds__(kReduceBlock) void k_ring_reduce(const Tile* tiles_g,
                                                        const float* const* slots_g, uint32_t N,
                                                        float* __restrict__ avg,
                                                        float* __restrict__ p,
                                                        float* __restrict__ v, float lr, float mu)
{
    const Tile ES_CONST_AS* tiles = (const Tile ES_CONST_AS*)tiles_g;
    const float* const ES_CONST_AS* slots = (const float* const ES_CONST_AS*)slots_g;
    small_tile<U, NB, NT, SGD>(slots, N, tiles[blockIdx.x].off, tiles[blockIdx.x].len,
                               tiles[blockIdx.x].rank0, avg, p, v, lr, mu);
}

// ---------------------------------------------------------------------------
// Big-tile form of the same kernel for large N.  Measured on MI355X: with many
// concurrent gradient streams HBM delivers more when each workgroup reads a long
// contiguous span per stream (128 KiB at UB = 32: 6.2 TB/s at N = 64 against
// 5.4 TB/s for 8 KiB spans).  A big tile is always full and 16-byte aligned, so
// addresses are base + constants and nothing is predicated; each wave owns UB
// consecutive KiB of every stream.  The first n_big workgroups take big tiles,
// the rest run the small-tile path (chunk remainders, ragged and unaligned
// pieces) with U = 2, NB = 8.
// ---------------------------------------------------------------------------
template <int UB, int NB, int NT, bool FIRST>
__device__ __forceinline__ void fold_batch_lin(const float* const ES_CONST_AS* slots, uint32_t N,
                                               uint32_t r0, uint64_t e0, f4 (&acc)[UB])
{
    f4 x[NB][UB];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        uint32_t r = r0 + j;
        if (r >= N) r -= N;
        const float* g = slots[r] + e0;
#pragma unroll
        for (int u = 0; u < UB; ++u) x[j][u] = ld4<(NT & 1) != 0>(g + 256 * u);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < NB; ++j) {
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            if (FIRST && j == 0)
                acc[u] = x[0][u];
            else
                acc[u] = acc[u] + x[j][u];
        }
    }
}

template <int UB, int NBB, int NT, bool SGD>
__global__ __launch_bounds__(kReduceBlock) void k_ring_reduce_big(const Tile* tiles_g, uint32_t n_big,
                                                            const float* const* slots_g, uint32_t N,
                                                            float* __restrict__ avg,
                                                            float* __restrict__ p,
                                                            float* __restrict__ v, float lr, float mu)
{
    const Tile ES_CONST_AS* tiles = (const Tile ES_CONST_AS*)tiles_g;
    const float* const ES_CONST_AS* slots = (const float* const ES_CONST_AS*)slots_g;
    const uint64_t off = tiles[blockIdx.x].off;
    const uint32_t len = tiles[blockIdx.x].len;
    const uint32_t rank0 = tiles[blockIdx.x].rank0;
    if (blockIdx.x >= n_big) {
        small_tile<2, 8, NT, SGD>(slots, N, off, len, rank0, avg, p, v, lr, mu);
        return;
    }
    const float fN = (float)N;
    const uint32_t w = threadIdx.x >> 6, l = threadIdx.x & 63;
    const uint64_t e0 = off + 4ull * ((uint64_t)(w * UB) * 64 + l);
    f4 acc[UB];
    uint32_t k;
    if (N >= (uint32_t)NBB) {
        fold_batch_lin<UB, NBB, NT, true>(slots, N, rank0, e0, acc);
        k = NBB;
    } else {
        fold_batch_lin<UB, 1, NT, true>(slots, N, rank0, e0, acc);
        k = 1;
    }
    for (; k + NBB <= N; k += NBB) {
        uint32_t r0 = rank0 + k;
        if (r0 >= N) r0 -= N;
        fold_batch_lin<UB, NBB, NT, false>(slots, N, r0, e0, acc);
    }
    for (; k < N; ++k) {
        uint32_t r0 = rank0 + k;
        if (r0 >= N) r0 -= N;
        fold_batch_lin<UB, 1, NT, false>(slots, N, r0, e0, acc);
    }
    // Epilogue kBigEpilogue vectors at a time, in the registers the rank loads have left free:
    // 2 * 16 loads of parameters and momentum in flight, then their stores (measured against
    // groups of 4: +3 % at N = 16, +2 % at N = 64; parameter and momentum accesses alternating
    // as here beat all of one, then all of the other).
    constexpr int EG = (kBigEpilogue < UB) ? kBigEpilogue : UB;
#pragma unroll
    for (int u0 = 0; u0 < UB; u0 += EG) {
        f4 pp[EG], vv[EG];
        if constexpr (SGD) {
#pragma unroll
            for (int q = 0; q < EG; ++q) {
                pp[q] = ld4_pv<(NT & 2) != 0>(p + e0 + 256 * (u0 + q));
                vv[q] = ld4_pv<(NT & 2) != 0>(v + e0 + 256 * (u0 + q));
            }
        }
#pragma unroll
        for (int q = 0; q < EG; ++q) {
            const uint64_t e = e0 + 256 * (u0 + q);
            const f4 a = acc[u0 + q] / fN;
            if (avg) st4_pv<(NT & 2) != 0>(avg + e, a);
            if constexpr (SGD) {
                const f4 mv = mu * vv[q];
                const f4 vn = mv + a;
                const f4 st = lr * vn;
                st4_pv<(NT & 2) != 0>(v + e, vn);
                st4_pv<(NT & 2) != 0>(p + e, pp[q] - st);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <int U, int NB>
static hipError_t launch_reduce_unb(hipStream_t s, const Tile* tiles, uint32_t n_tiles,
                                    const float* const* slots, uint32_t N, float* avg, float* p,
                                    float* v, float lr, float mu, int nt, uint32_t lds_pad)
{
    const bool sgd = p != nullptr;
    dim3 grid(n_tiles), block(kReduceBlock);
#define ES_LAUNCH(NTV, SGDV) \
    hipLaunchKernelGGL((k_ring_reduce<U, NB, NTV, SGDV>), grid, block, lds_pad, s, tiles, slots, N, avg, p, v, lr, mu)
    if (!sgd) {
        switch (nt & 3) {
        case 0: ES_LAUNCH(0, false); break;
        case 1: ES_LAUNCH(1, false); break;
        case 2: ES_LAUNCH(2, false); break;
        default: ES_LAUNCH(3, false); break;
        }
    } else {
        switch (nt & 3) {
        case 0: ES_LAUNCH(0, true); break;
        case 1: ES_LAUNCH(1, true); break;
        case 2: ES_LAUNCH(2, true); break;
        default: ES_LAUNCH(3, true); break;
        }
    }
#undef ES_LAUNCH
    return hipGetLastError();
}

template <int U>
static hipError_t launch_reduce_u(hipStream_t s, const Tile* tiles, uint32_t n_tiles,
                                  const float* const* slots, uint32_t N, float* avg, float* p,
                                  float* v, float lr, float mu, ReduceShape sh)
{
    const int nt = (sh.nontemporal ? 1 : 0) | (sh.nontemporal_pv ? 2 : 0);
    switch (sh.rank_batch) {
    case 1:  return launch_reduce_unb<U, 1>(s, tiles, n_tiles, slots, N, avg, p, v, lr, mu, nt, reduce_lds_pad(sh.lds_pad_kib, N, sh.nontemporal_pv != 0 && p != nullptr, p != nullptr));
    case 2:  return launch_reduce_unb<U, 2>(s, tiles, n_tiles, slots, N, avg, p, v, lr, mu, nt, reduce_lds_pad(sh.lds_pad_kib, N, sh.nontemporal_pv != 0 && p != nullptr, p != nullptr));
    case 4:  return launch_reduce_unb<U, 4>(s, tiles, n_tiles, slots, N, avg, p, v, lr, mu, nt, reduce_lds_pad(sh.lds_pad_kib, N, sh.nontemporal_pv != 0 && p != nullptr, p != nullptr));
    case 8:  return launch_reduce_unb<U, 8>(s, tiles, n_tiles, slots, N, avg, p, v, lr, mu, nt, reduce_lds_pad(sh.lds_pad_kib, N, sh.nontemporal_pv != 0 && p != nullptr, p != nullptr));
    case 16: return launch_reduce_unb<U, 16>(s, tiles, n_tiles, slots, N, avg, p, v, lr, mu, nt, reduce_lds_pad(sh.lds_pad_kib, N, sh.nontemporal_pv != 0 && p != nullptr, p != nullptr));
    default: return hipErrorInvalidValue;
    }
}

template <int UB, int NBB>
static hipError_t launch_reduce_big(hipStream_t s, const Tile* tiles, uint32_t n_tiles, uint32_t n_big,
                                    const float* const* slots, uint32_t N, float* avg, float* p,
                                    float* v, float lr, float mu, int nt)
{
    const bool sgd = p != nullptr;
    dim3 grid(n_tiles), block(kReduceBlock);
#define ES_LAUNCH(NTV, SGDV) \
    hipLaunchKernelGGL((k_ring_reduce_big<UB, NBB, NTV, SGDV>), grid, block, 0, s, tiles, n_big, slots, N, avg, p, v, lr, mu)
    if (!sgd) {
        switch (nt & 3) {
        case 0: ES_LAUNCH(0, false); break;
        case 1: ES_LAUNCH(1, false); break;
        case 2: ES_LAUNCH(2, false); break;
        default: ES_LAUNCH(3, false); break;
        }
    } else {
        switch (nt & 3) {
        case 0: ES_LAUNCH(0, true); break;
        case 1: ES_LAUNCH(1, true); break;
        case 2: ES_LAUNCH(2, true); break;
        default: ES_LAUNCH(3, true); break;
        }
    }
#undef ES_LAUNCH
    return hipGetLastError();
}

template <int UB>
static hipError_t launch_reduce_big_u(hipStream_t s, const Tile* tiles, uint32_t n_tiles, uint32_t n_big,
                                      const float* const* slots, uint32_t N, float* avg, float* p,
                                      float* v, float lr, float mu, ReduceShape sh)
{
    const int nt = (sh.nontemporal ? 1 : 0) | (sh.nontemporal_pv ? 2 : 0);
    // only shapes whose loads in flight fit the register file exist: UB * batch <= 32
    if (sh.big_rank_batch == 1)
        return launch_reduce_big<UB, 1>(s, tiles, n_tiles, n_big, slots, N, avg, p, v, lr, mu, nt);
    if constexpr (UB <= 16) {
        if (sh.big_rank_batch == 2)
            return launch_reduce_big<UB, 2>(s, tiles, n_tiles, n_big, slots, N, avg, p, v, lr, mu, nt);
    }
    if constexpr (UB <= 8) {
        if (sh.big_rank_batch == 4)
            return launch_reduce_big<UB, 4>(s, tiles, n_tiles, n_big, slots, N, avg, p, v, lr, mu, nt);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_ring_reduce(hipStream_t s, const Tile* tiles, uint32_t n_tiles, uint32_t n_big,
                              const float* const* slots, uint32_t N, float* avg, float* p,
                              float* v, float lr, float mu, ReduceShape sh)
{
    if (n_tiles == 0) return hipSuccess;
    if (sh.big_unroll) {
        switch (sh.big_unroll) {
        case 8:  return launch_reduce_big_u<8>(s, tiles, n_tiles, n_big, slots, N, avg, p, v, lr, mu, sh);
        case 16: return launch_reduce_big_u<16>(s, tiles, n_tiles, n_big, slots, N, avg, p, v, lr, mu, sh);
        case 32: return launch_reduce_big_u<32>(s, tiles, n_tiles, n_big, slots, N, avg, p, v, lr, mu, sh);
        default: return hipErrorInvalidValue;
        }
    }
    switch (sh.unroll) {
    case 1: return launch_reduce_u<1>(s, tiles, n_tiles, slots, N, avg, p, v, lr, mu, sh);
    case 2: return launch_reduce_u<2>(s, tiles, n_tiles, slots, N, avg, p, v, lr, mu, sh);
    case 4: return launch_reduce_u<4>(s, tiles, n_tiles, slots, N, avg, p, v, lr, mu, sh);
    default: return hipErrorInvalidValue;
    }
}

// Redirect a few entries of the rank -> gradient-base table in stream order.
__global__ void k_patch_slots(const float** table, const InPlace patch)
{
    if (blockIdx.x == 0 && threadIdx.x < patch.n) table[patch.rank[threadIdx.x]] = patch.ptr[threadIdx.x];
}

hipError_t launch_patch_slots(hipStream_t s, const float** table, const InPlace& patch)
{
    if (patch.n == 0) return hipSuccess;
    hipLaunchKernelGGL(k_patch_slots, dim3(1), dim3(64), 0, s, table, patch);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// SGD with momentum on the shared replica (paper §3.2), unfused form.
// ---------------------------------------------------------------------------
constexpr int kSgdU = 4;

template <bool NTPV>
__global__ __launch_bounds__(kBlock) void k_sgd(float* __restrict__ p, float* __restrict__ v,
                                                const float* __restrict__ g, uint64_t n,
                                                float lr, float mu)
{
    const uint64_t nvec = n >> 2;
    const uint64_t base = (uint64_t)blockIdx.x * (kBlock * kSgdU) + threadIdx.x;
    f4 pp[kSgdU], vv[kSgdU], gg[kSgdU];
#pragma unroll
    for (int u = 0; u < kSgdU; ++u) {
        const uint64_t i = base + (uint64_t)u * kBlock;
        if (i < nvec) {
            gg[u] = ld4<true>(g + 4 * i);
            pp[u] = ld4_pv<NTPV>(p + 4 * i);
            vv[u] = ld4_pv<NTPV>(v + 4 * i);
        }
    }
#pragma unroll
    for (int u = 0; u < kSgdU; ++u) {
        const uint64_t i = base + (uint64_t)u * kBlock;
        if (i < nvec) {
            const f4 mv = mu * vv[u];
            const f4 vn = mv + gg[u];
            const f4 st = lr * vn;
            st4_pv<NTPV>(v + 4 * i, vn);
            st4_pv<NTPV>(p + 4 * i, pp[u] - st);
        }
    }
    if (blockIdx.x == 0) {
        const uint64_t e = 4 * nvec + threadIdx.x;
        if (e < n) {
            const float mv = mu * v[e];
            const float vn = mv + g[e];
            const float st = lr * vn;
            v[e] = vn;
            p[e] = p[e] - st;
        }
    }
}

hipError_t launch_sgd(hipStream_t s, float* p, float* v, const float* g, uint64_t n, float lr,
                      float mu, bool stream_pv)
{
    if (n == 0) return hipSuccess;
    const uint64_t nvec = n >> 2;
    uint64_t blocks = (nvec + kBlock * kSgdU - 1) / (kBlock * kSgdU);
    if (blocks == 0) blocks = 1;
    if (stream_pv)
        hipLaunchKernelGGL(k_sgd<true>, dim3((uint32_t)blocks), dim3(kBlock), kAuxLdsPad, s, p, v, g, n, lr, mu);
    else
        hipLaunchKernelGGL(k_sgd<false>, dim3((uint32_t)blocks), dim3(kBlock), kAuxLdsPad, s, p, v, g, n, lr, mu);
    return hipGetLastError();
}

// The same update with the gradient clipped by its global norm first: every lane forms
//     coef = min(1, max_norm / (norm + eps))
// from the norm es_grad_sq_norm left in device memory (no host round trip) and scales its
// gradient elements by it; coef * g is rounded on its own before it enters the momentum.
template <bool NTPV>
__global__ __launch_bounds__(kBlock) void k_sgd_clip(float* __restrict__ p, float* __restrict__ v,
                                                     const float* __restrict__ g, uint64_t n,
                                                     const float* __restrict__ norm2, float max_norm,
                                                     float eps, float lr, float mu)
{
    const float d = norm2[1] + eps;
    const float q = max_norm / d;
    const float coef = q < 1.0f ? q : 1.0f;
    const uint64_t nvec = n >> 2;
    const uint64_t base = (uint64_t)blockIdx.x * (kBlock * kSgdU) + threadIdx.x;
    f4 pp[kSgdU], vv[kSgdU], gg[kSgdU];
#pragma unroll
    for (int u = 0; u < kSgdU; ++u) {
        const uint64_t i = base + (uint64_t)u * kBlock;
        if (i < nvec) {
            gg[u] = ld4<true>(g + 4 * i);
            pp[u] = ld4_pv<NTPV>(p + 4 * i);
            vv[u] = ld4_pv<NTPV>(v + 4 * i);
        }
    }
#pragma unroll
    for (int u = 0; u < kSgdU; ++u) {
        const uint64_t i = base + (uint64_t)u * kBlock;
        if (i < nvec) {
            const f4 gs = coef * gg[u];
            const f4 mv = mu * vv[u];
            const f4 vn = mv + gs;
            const f4 st = lr * vn;
            st4_pv<NTPV>(v + 4 * i, vn);
            st4_pv<NTPV>(p + 4 * i, pp[u] - st);
        }
    }
    if (blockIdx.x == 0) {
        const uint64_t e = 4 * nvec + threadIdx.x;
        if (e < n) {
            const float gs = coef * g[e];
            const float mv = mu * v[e];
            const float vn = mv + gs;
            const float st = lr * vn;
            v[e] = vn;
            p[e] = p[e] - st;
        }
    }
}

hipError_t launch_sgd_clip(hipStream_t s, float* p, float* v, const float* g, uint64_t n,
                           const float* norm2, float max_norm, float eps, float lr, float mu, bool stream_pv)
{
    if (n == 0) return hipSuccess;
    const uint64_t nvec = n >> 2;
    uint64_t blocks = (nvec + kBlock * kSgdU - 1) / (kBlock * kSgdU);
    if (blocks == 0) blocks = 1;
    if (stream_pv)
        hipLaunchKernelGGL(k_sgd_clip<true>, dim3((uint32_t)blocks), dim3(kBlock), kAuxLdsPad, s, p, v, g, n, norm2,
                           max_norm, eps, lr, mu);
    else
        hipLaunchKernelGGL(k_sgd_clip<false>, dim3((uint32_t)blocks), dim3(kBlock), kAuxLdsPad, s, p, v, g, n, norm2,
                           max_norm, eps, lr, mu);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Fixed-tree sum of squares of a flat vector (global gradient norm).  In the
// spirit of the paper's level D2 (section 3.3: reductions must not depend on
// the GPU they run on) the summation tree is a function of the vector length
// alone: blocks of 4096 elements; lane t adds the squares of elements
// 4*(256*q + t) + c, q = 0..3 outer, c = 0..3 inner, starting from +0; the 256
// lane sums combine as v[t] += v[t+s], s = 128 .. 1; block partials combine the
// same way in one more workgroup (lane t adds partials t, t+256, ... first).
// No atomics; wave shuffles (and LDS in the last stage) carry the tree.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float tree256(float s, float* lds)
{
    const uint32_t t = threadIdx.x;
    lds[t] = s;
    __syncthreads();
    if (t < 128) {
        s = s + lds[t + 128];
        lds[t] = s;
    }
    __syncthreads();
    if (t < 64) {
        s = s + lds[t + 64];
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) s = s + __shfl_down(s, d, 64);
    }
    return s;                                           // valid in lane 0
}

// One WAVE per 4096-element block: hardware lane h plays the tree's lanes h, h+64,
// h+128 and h+192, so the strides 128 and 64 are adds between its own registers,
// 32 .. 1 are wave shuffles, and no LDS or barrier is needed; all 16 loads of a
// lane are in flight before the first add.
__global__ __launch_bounds__(kBlock) void k_sq_partials(const float* __restrict__ x, uint64_t n,
                                                        uint64_t nblk, float* __restrict__ part)
{
    const uint32_t h = threadIdx.x & 63;
    const uint64_t blk = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (blk >= nblk) return;                            // whole wave leaves together
    const uint64_t base = blk * 4096;
    f4 v[4][4];                                         // [tree lane h + 64 j][q]
    if (base + 4096 <= n) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j][q] = ld4<true>(x + base + 4ull * (256 * q + 64 * j + h));
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint64_t i = base + 4ull * (256 * q + 64 * j + h);
                f4 e;
                e.x = (i + 0 < n) ? x[i + 0] : 0.0f;
                e.y = (i + 1 < n) ? x[i + 1] : 0.0f;
                e.z = (i + 2 < n) ? x[i + 2] : 0.0f;
                e.w = (i + 3 < n) ? x[i + 3] : 0.0f;
                v[j][q] = e;
            }
    }
    __builtin_amdgcn_sched_barrier(0);
    float s[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float a = 0.0f;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f4 e = v[j][q];
            a = a + e.x * e.x;
            a = a + e.y * e.y;
            a = a + e.z * e.z;
            a = a + e.w * e.w;
        }
        s[j] = a;
    }
    float r0 = s[0] + s[2];                             // stride 128: lanes h and h+64
    float r1 = s[1] + s[3];
    float r = r0 + r1;                                  // stride 64
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) r = r + __shfl_down(r, d, 64);
    if (h == 0) part[blk] = r;
}

__global__ __launch_bounds__(kBlock) void k_sq_final(const float* __restrict__ part, uint64_t nblk,
                                                     float* __restrict__ out)
{
    __shared__ float lds[kBlock];
    float s = 0.0f;
    // lane t adds partials t, t+256, ... in that order; eight loads are issued ahead of the adds
    for (uint64_t k0 = threadIdx.x; k0 < nblk; k0 += 8 * kBlock) {
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint64_t k = k0 + (uint64_t)j * kBlock;
            v[j] = part[k < nblk ? k : nblk - 1];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (k0 + (uint64_t)j * kBlock < nblk) s = s + v[j];
    }
    s = tree256(s, lds);
    if (threadIdx.x == 0) {
        out[0] = s;
        out[1] = sqrtf(s);
    }
}

hipError_t launch_sq_norm(hipStream_t s, const float* x, uint64_t n, float* part, float* out)
{
    const uint64_t nblk = (n + 4095) / 4096;
    if (nblk) hipLaunchKernelGGL(k_sq_partials, dim3((uint32_t)((nblk + 3) / 4)), dim3(kBlock), kAuxLdsPad, s, x, n, nblk, part);
    hipLaunchKernelGGL(k_sq_final, dim3(1), dim3(kBlock), 0, s, part, nblk, out);
    return hipGetLastError();
}

// Block partials of the allocation-free norm: one array per GPU, part of the code
// object, held until the process ends.  `scratch` is a host-side stand-in for the
// symbol, not a device address: host code only ever uses the address that
// hipGetSymbolAddress returned for the device in question.
static __device__ __align__(256) float scratch[kStaticPartials];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float* g_scratch_ptr[kMaxDevices] = {};          // per device: where that GPU's copy of `scratch` lives
}

// Device address of the current device's `scratch` (looked up once per device).
static hipError_t static_partials(float** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        float* p = nullptr;
        e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

hipError_t launch_sq_norm_static(hipStream_t s, const float* x, uint64_t n, float* out)
{
    if ((n + 4095) / 4096 > kStaticPartials) return hipErrorInvalidValue;
    float* part = nullptr;
    const hipError_t e = static_partials(&part);
    if (e != hipSuccess) return e;
    // k_sq_partials writes partials [0, nblk) before k_sq_final reads exactly those, so what
    // an earlier call left in the array is never read and nothing has to be cleared
    return launch_sq_norm(s, x, n, part, out);
}

// ---------------------------------------------------------------------------
// Gradient staging: copy one bucket into an EST's context slot (paper §3.2).
// ---------------------------------------------------------------------------
// One 16-byte vector per lane and streaming hints on both sides measured fastest
// on MI355X (about 6.5 TB/s read+write; four vectors per lane: 4.6 TB/s).
//
// Neither side needs 16-byte alignment.  Each wave moves 1 KiB that starts on a 128-byte
// line of the destination (a piece that starts inside a line shares that line with the
// neighbouring workgroup on another compute die, and the line travels twice: measured
// -13 % for buckets at offsets that are not multiples of 128 bytes).  The elements up to
// the first such line and the 0-3 after the last whole vector are copied one by one by the
// first workgroup.  Loads are 16 bytes wide at whatever 4-byte-aligned address that gives
// on the source side (global memory needs dword alignment only): when source and
// destination are equally far off a line - the usual case, a bucket at the same offset in
// a flat gradient and in the slot - they are aligned alike.
typedef float f4_dword_aligned __attribute__((ext_vector_type(4), aligned(4)));

__device__ __forceinline__ void copy_span(float* __restrict__ dst, const float* __restrict__ src,
                                          uint64_t n, uint32_t block, uint32_t lane, uint32_t lanes)
{
    constexpr uintptr_t kAlign = 128;                    // 1 KiB alignment measured no better
    uint64_t head = ((kAlign - (reinterpret_cast<uintptr_t>(dst) & (kAlign - 1))) & (kAlign - 1)) >> 2;
    if (head > n) head = n;
    const float* __restrict__ sb = src + head;
    float* __restrict__ db = dst + head;
    const uint64_t nb = n - head;
    const uint64_t nvec = nb >> 2;
    const uint64_t i = (uint64_t)block * lanes + lane;
    if (i < nvec) {
        const f4 x = __builtin_nontemporal_load(reinterpret_cast<const f4_dword_aligned*>(sb + 4 * i));
        __builtin_nontemporal_store(x, reinterpret_cast<f4*>(db + 4 * i));
    }
    if (block == 0) {
        for (uint64_t e = lane; e < head; e += lanes) dst[e] = src[e];
        const uint64_t e = 4 * nvec + lane;
        if (lane < 4 && e < nb) db[e] = sb[e];
    }
}

__global__ __launch_bounds__(kCopyBlock) void k_copy_f4(float* __restrict__ dst,
                                                    const float* __restrict__ src, uint64_t n)
{
    copy_span(dst, src, n, blockIdx.x, threadIdx.x, kCopyBlock);
}

hipError_t launch_copy_f32(hipStream_t s, float* dst, const float* src, uint64_t n)
{
    if (n == 0) return hipSuccess;
    uint64_t blocks = ((n >> 2) + kCopyBlock - 1) / kCopyBlock;
    if (blocks == 0) blocks = 1;
    hipLaunchKernelGGL(k_copy_f4, dim3((uint32_t)blocks), dim3(kCopyBlock), 0, s, dst, src, n);
    return hipGetLastError();
}

// Batched staging: the runs arrive as a kernel argument (no table upload); a
// workgroup finds its run from the prefix sums (wave-uniform, scalar).
template <int BS>
__global__ __launch_bounds__(BS) void k_copy_runs(const CopyRuns runs)
{
    // the run of this workgroup = how many later runs start at or before it.  All prefix sums
    // are fetched at once (independent scalar loads of the kernel argument) and compared in
    // registers: a dependent load per run would be most of this short workgroup's life.
    // (Entries past the last run hold 0xFFFFFFFF, so the count needs no bound.)  A single run -
    // one flat gradient vector, the common case - skips the lookup: it costs 2.7 % there.
    uint32_t r = 0;
    if (runs.n_runs > 1) {
#pragma unroll
        for (int k = 1; k < kMaxRuns; ++k) r += blockIdx.x >= runs.first_block[k] ? 1u : 0u;
    }
    copy_span(runs.dst[r], runs.src[r], runs.n[r], blockIdx.x - runs.first_block[r], threadIdx.x, BS);
}

hipError_t launch_copy_runs(hipStream_t s, const CopyRuns& runs)
{
    if (runs.n_runs == 0) return hipSuccess;
    const uint32_t blocks = runs.first_block[runs.n_runs];
    if (blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(k_copy_runs<kCopyBlock>, dim3(blocks), dim3(kCopyBlock), 0, s, runs);
    return hipGetLastError();
}

__global__ __launch_bounds__(kBlock) void k_copy_bytes(uint8_t* __restrict__ dst,
                                                       const uint8_t* __restrict__ src, uint64_t n16)
{
    const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n16) reinterpret_cast<u4*>(dst)[i] = reinterpret_cast<const u4*>(src)[i];
}

// dst, src 16-byte aligned, n a multiple of 16
hipError_t launch_copy_bytes(hipStream_t s, uint8_t* dst, const uint8_t* src, uint64_t n)
{
    if (n == 0) return hipSuccess;
    const uint64_t n16 = n >> 4;
    const uint64_t blocks = (n16 + kBlock - 1) / kBlock;
    hipLaunchKernelGGL(k_copy_bytes, dim3((uint32_t)blocks), dim3(kBlock), 0, s, dst, src, n16);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Small-state context switch (paper §3.2): scattered live tensors <-> one
// contiguous slot, all segments in one launch.  One workgroup per Piece.
// In kSwitch every lane reads its live bytes, then overwrites them with the
// incoming EST's bytes: outgoing and incoming state never meet across lanes.
// ---------------------------------------------------------------------------
template <typename T, uint32_t BS = kBlock>
__device__ __forceinline__ void ctx_move(T* live, T* sa, const T* sb, uint32_t n, int dir)
{
    for (uint32_t i = threadIdx.x; i < n; i += BS) {
        if (dir == kSave) {
            sa[i] = live[i];
        } else if (dir == kRestore) {
            live[i] = sa[i];
        } else {
            const T out = live[i];
            const T in = sb[i];
            sa[i] = out;
            live[i] = in;
        }
    }
}

template <uint32_t BS>
__device__ __forceinline__ void ctx_piece(const Piece ES_CONST_AS* pieces, uint32_t k, uint8_t* slot_a,
                                          const uint8_t* slot_b, int dir)
{
    uint8_t* live = (uint8_t*)pieces[k].live;
    const uint64_t so = pieces[k].slot_off;
    const uint32_t nb = pieces[k].nbytes;
    const uint32_t w = pieces[k].width;
    uint8_t* sa = slot_a + so;
    const uint8_t* sb = slot_b ? slot_b + so : nullptr;
    if (w == 16)
        ctx_move<u4, BS>((u4*)live, (u4*)sa, (const u4*)sb, nb >> 4, dir);
    else if (w == 4)
        ctx_move<uint32_t, BS>((uint32_t*)live, (uint32_t*)sa, (const uint32_t*)sb, nb >> 2, dir);
    else
        ctx_move<uint8_t, BS>(live, sa, sb, nb, dir);
}

__global__ __launch_bounds__(kBlock) void k_ctx(const Piece* pieces_g, uint8_t* slot_a,
                                                const uint8_t* slot_b, int dir)
{
    ctx_piece<kBlock>((const Piece ES_CONST_AS*)pieces_g, blockIdx.x, slot_a, slot_b, dir);
}

// An EST boundary in one launch (paper section 3.2: at a mini-batch boundary the outgoing EST's
// context is saved, its gradients are copied aside, and the incoming EST's context is restored):
// the first n_pieces workgroups move small-state pieces (save, or save + restore per byte in one
// lane), all others are the staging copy of the outgoing EST's gradient runs.  The two parts touch
// disjoint memory, so no ordering between them is needed inside the launch.
__global__ __launch_bounds__(kCopyBlock) void k_est_boundary(const CopyRuns runs, const Piece* pieces_g,
                                                             uint32_t n_pieces, uint8_t* slot_a,
                                                             const uint8_t* slot_b, int dir)
{
    if (blockIdx.x < n_pieces) {
        ctx_piece<kCopyBlock>((const Piece ES_CONST_AS*)pieces_g, blockIdx.x, slot_a, slot_b, dir);
        return;
    }
    const uint32_t blk = blockIdx.x - n_pieces;
    uint32_t r = 0;
    if (runs.n_runs > 1) {
#pragma unroll
        for (int k = 1; k < kMaxRuns; ++k) r += blk >= runs.first_block[k] ? 1u : 0u;
    }
    copy_span(runs.dst[r], runs.src[r], runs.n[r], blk - runs.first_block[r], threadIdx.x, kCopyBlock);
}

hipError_t launch_est_boundary(hipStream_t s, const CopyRuns& runs, const Piece* pieces, uint32_t n_pieces,
                               uint8_t* slot_a, const uint8_t* slot_b, CtxDir dir)
{
    const uint32_t copy_blocks = runs.n_runs ? runs.first_block[runs.n_runs] : 0;
    if (n_pieces + copy_blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(k_est_boundary, dim3(n_pieces + copy_blocks), dim3(kCopyBlock), 0, s, runs, pieces,
                       n_pieces, slot_a, slot_b, (int)dir);
    return hipGetLastError();
}

hipError_t launch_ctx(hipStream_t s, const Piece* pieces, uint32_t n_pieces, uint8_t* slot_a,
                      const uint8_t* slot_b, CtxDir dir)
{
    if (n_pieces == 0) return hipSuccess;
    hipLaunchKernelGGL(k_ctx, dim3(n_pieces), dim3(kBlock), 0, s, pieces, slot_a, slot_b, (int)dir);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Dropout keep-mask from an EST's live RNG state (paper §3.3: Dropout depends
// on RNG state, which is therefore EST context).  Philox4x32-10 after Salmon,
// Moraes, Dror, Shaw (SC'11): ten rounds of two 32x32->64 multiplies whose
// high halves are mixed with the other two counter words and the key; the key
// advances by two Weyl constants per round.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t a = (uint64_t)0xD2511F53u * c0;
        const uint64_t b = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(b >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(a >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)b;
        c3 = (uint32_t)a;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Each lane draws 4 counter values = 16 mask bytes.
__global__ __launch_bounds__(kBlock) void k_dropout_mask(const uint64_t* __restrict__ state,
                                                         uint8_t* __restrict__ mask, uint64_t n,
                                                         uint64_t threshold, int aligned16)
{
    const uint64_t seed = state[0];
    const uint64_t offset = state[1];
    const uint64_t t = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    const uint64_t j0 = 16 * t;
    if (j0 >= n) return;
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    uint32_t packed[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint64_t pos = offset + 4 * t + q;
        uint32_t w[4];
        philox4x32_10((uint32_t)pos, (uint32_t)(pos >> 32), 0u, 0u, k0, k1, w);
        uint32_t word = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            word |= ((uint64_t)w[k] >= threshold ? 1u : 0u) << (8 * k);
        packed[q] = word;
    }
    if (aligned16 && j0 + 16 <= n) {
        u4 o = {packed[0], packed[1], packed[2], packed[3]};
        *reinterpret_cast<u4*>(mask + j0) = o;
    } else {
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (j0 + i < n) mask[j0 + i] = (uint8_t)((packed[i >> 2] >> (8 * (i & 3))) & 0xFF);
    }
}

__global__ void k_philox_advance(uint64_t* state, uint64_t blocks)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) state[1] = state[1] + blocks;
}

hipError_t launch_dropout_mask(hipStream_t s, uint64_t* state, uint8_t* mask, uint64_t n,
                               uint64_t threshold)
{
    if (n == 0) return hipSuccess;
    const uint64_t lanes = (n + 15) / 16;
    const uint64_t blocks = (lanes + kBlock - 1) / kBlock;
    const int aligned16 = (((uintptr_t)mask) & 15) == 0;
    hipLaunchKernelGGL(k_dropout_mask, dim3((uint32_t)blocks), dim3(kBlock), 0, s, state, mask, n,
                       threshold, aligned16);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_philox_advance, dim3(1), dim3(64), 0, s, state, (n + 3) / 4);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// BatchNorm batch statistics along the fixed tree (the paper's level D2, section 3.3: a
// reduce whose result does not depend on the GPU; BatchNorm is the operator whose statistics
// every EST tracks).  x is [B][C][HW].  For channel ch the M = B*HW values in the order
// (image, position) form a vector y; its terms f(y[m]) are summed along the tree of the norm
// (blocks of 4096 terms; lane t adds terms 4*(256*q + t) + c, q outer, c inner, from +0;
// stride halving over 256 lanes; block partials combined the same way, lane t first adding
// partials t, t+256, ...).  mean = T(y) / M, var = T((y - mean)^2) / M.
//
// First stage: one WAVE per block of one channel; hardware lane h plays tree lanes h, h+64,
// h+128, h+192 (strides 128 and 64 are adds between its own registers, 32..1 wave shuffles).
// Second stage: one workgroup per channel with an LDS stage.  No atomics.
// ---------------------------------------------------------------------------
template <bool SQDEV>
__global__ __launch_bounds__(kBlock) void k_bn_partials(const float* __restrict__ x, uint32_t C, uint32_t HW,
                                                        uint32_t M, uint32_t nblk,
                                                        const float* __restrict__ mean,
                                                        float* __restrict__ part)
{
    const uint32_t h = threadIdx.x & 63;
    const uint32_t blk = blockIdx.x * 4 + (threadIdx.x >> 6);
    const uint32_t ch = blockIdx.y;
    if (blk >= nblk) return;                            // whole wave leaves together
    const float center = SQDEV ? mean[ch] : 0.0f;
    const uint32_t base = blk * 4096;
    f4 t[4][4];                                         // [tree lane h + 64 j][q]: four consecutive terms
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t m0 = base + 4u * (256 * q + 64 * j + h);
            const uint32_t img = m0 / HW, pos = m0 - img * HW;
            f4 e;
            if (m0 + 3 < M && pos + 3 < HW) {           // four terms of one image, all present
                // plain (cacheable) load: the second pass reads the same values again
                e = *reinterpret_cast<const f4_dword_aligned*>(x + ((uint64_t)img * C + ch) * HW + pos);
                if constexpr (SQDEV) {
                    const f4 d = e - center;
                    e = d * d;
                }
            } else {
                float el[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const uint32_t m = m0 + c;
                    float term = 0.0f;                  // terms beyond M count as +0
                    if (m < M) {
                        const uint32_t im = m / HW;
                        const float y = x[((uint64_t)im * C + ch) * HW + (m - im * HW)];
                        if constexpr (SQDEV) {
                            const float d = y - center;
                            term = d * d;
                        } else {
                            term = y;
                        }
                    }
                    el[c] = term;
                }
                e = f4{el[0], el[1], el[2], el[3]};
            }
            t[j][q] = e;
        }
    float s[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float a = 0.0f;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f4 e = t[j][q];
            a = a + e.x;
            a = a + e.y;
            a = a + e.z;
            a = a + e.w;
        }
        s[j] = a;
    }
    const float r0 = s[0] + s[2];                       // stride 128
    const float r1 = s[1] + s[3];
    float r = r0 + r1;                                  // stride 64
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) r = r + __shfl_down(r, d, 64);
    if (h == 0) part[(uint64_t)ch * nblk + blk] = r;
}

__global__ __launch_bounds__(kBlock) void k_bn_final(const float* __restrict__ part, uint32_t nblk, float fM,
                                                     float* __restrict__ out)
{
    __shared__ float lds[kBlock];
    const float* pc = part + (uint64_t)blockIdx.x * nblk;
    float s = 0.0f;
    for (uint32_t k = threadIdx.x; k < nblk; k += kBlock) s = s + pc[k];      // partials t, t+256, ... in order
    s = tree256(s, lds);
    if (threadIdx.x == 0) out[blockIdx.x] = s / fM;
}

hipError_t launch_bn_batch_stats(hipStream_t s, const float* x, uint32_t B, uint32_t C, uint32_t HW,
                                 float* mean, float* var, float* part)
{
    const uint32_t M = B * HW;
    const uint32_t nblk = (M + 4095) / 4096;
    if (C == 0) return hipSuccess;
    const dim3 grid((nblk + 3) / 4, C);
    const float fM = (float)M;
    if (nblk) hipLaunchKernelGGL(k_bn_partials<false>, grid, dim3(kBlock), 0, s, x, C, HW, M, nblk, mean, part);
    hipLaunchKernelGGL(k_bn_final, dim3(C), dim3(kBlock), 0, s, part, nblk, fM, mean);
    if (nblk) hipLaunchKernelGGL(k_bn_partials<true>, grid, dim3(kBlock), 0, s, x, C, HW, M, nblk, mean, part);
    hipLaunchKernelGGL(k_bn_final, dim3(C), dim3(kBlock), 0, s, part, nblk, fM, var);
    return hipGetLastError();
}

}  // namespace es
