// Internal interface between the host runtime (es_api.cpp) and the gfx950
// kernels (es_kernels.hip).  Not part of the public boundary.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace es {

// One workgroup's share of the ring-ordered reduction: a contiguous range of
// the flat parameter space that lies inside a single ring chunk, so the rank
// the fold starts at is the same for every element of the tile.
struct Tile {
    uint64_t off;      // first element (flat parameter space)
    uint32_t len;      // elements
    uint32_t rank0;    // virtual rank whose gradient opens the fold (= chunk index)
};
static_assert(sizeof(Tile) == 16, "Tile is read with one 16-byte scalar load");

// One workgroup's share of a small-state context copy.
struct Piece {
    void*    live;       // device address inside a live state tensor
    uint64_t slot_off;   // byte offset inside the EST's context slot
    uint32_t nbytes;     // <= kPieceBytes
    uint32_t width;      // 16, 4 or 1: widest access both sides are aligned for
};
static_assert(sizeof(Piece) == 24, "Piece layout");

constexpr uint32_t kPieceBytes = 4096;
constexpr uint32_t kBlock = 256;
#ifndef ES_COPY_BLOCK
#define ES_COPY_BLOCK 64
#endif
#ifndef ES_REDUCE_BLOCK
#define ES_REDUCE_BLOCK 256
#endif
constexpr uint32_t kReduceBlock = ES_REDUCE_BLOCK;   // lanes per workgroup of the ring-ordered reduce
constexpr int kBigEpilogue = 16;                     // vectors per lane per pass of a big tile's update epilogue

// Occupancy caps.  Measured on MI355X: the streaming kernels reach more of the HBM rate with few
// workgroups resident per CU (more resident workgroups = more DRAM regions open at once), as long
// as each has a few tens of KiB of loads in flight.  A launch reserves LDS it never touches so that
// only 160 KiB / reserve workgroups fit a CU.  Small-tile reduce: 2 per CU (3 below 4 ranks, where a
// workgroup has fewer loads in flight): +4-8 % at N = 2..10 on 26 M and 109 M parameters with
// nothing cache-resident; 1 per CU when every batch of the fold is full or nearly so (N = 8,
// N >= 10) and parameters and momentum stream (another +3-7 %; with parameters and momentum coming
// from the Infinity Cache one workgroup per CU is 7 % slower than two).  Update and norm kernels:
// 2 per CU, +4 % at 355 M parameters.
constexpr uint32_t kAuxLdsPad = 64u << 10;
inline uint32_t reduce_lds_pad(int option_kib, uint32_t n_ranks, bool streaming_pv, bool fused)
{
    if (option_kib >= 0) return (uint32_t)option_kib << 10;
    // below 4 ranks the unfused reduce is close to a copy and wants more waves still (5 per CU:
    // 57 -> 77 % of the HBM peak at N = 1, 70 -> 80 % at N = 3 on 109 M parameters)
    if (n_ranks < 4) return fused ? 53u << 10 : 32u << 10;
    if (streaming_pv && (n_ranks == 8 || n_ranks >= 10)) return 160u << 10;
    return 64u << 10;
}
constexpr uint32_t kCopyBlock = ES_COPY_BLOCK;   // lanes per workgroup of the batched staging copy

// Entries of the rank -> gradient-base table that are redirected for one reduce
// (gradients taken in place from caller memory, no staging copy).
constexpr uint32_t kMaxInPlace = 16;            // entries one patch launch carries
struct InPlace {
    uint32_t     n;
    uint32_t     rank[kMaxInPlace];
    const float* ptr[kMaxInPlace];      // flat parameter order, 16-byte aligned
};
// table[patch.rank[k]] <- patch.ptr[k], stream-ordered (the values travel as a kernel argument)
hipError_t launch_patch_slots(hipStream_t s, const float** table, const InPlace& patch);

struct ReduceShape {
    int unroll;        // 16-byte vectors per lane per rank
    int rank_batch;    // ranks loaded before adds are issued
    int nontemporal;   // streaming hint on gradient loads
    int big_unroll;    // 0, or vectors per lane of a big tile (8, 16, 32): see k_ring_reduce_big
    int big_rank_batch;
    int nontemporal_pv; // streaming hint on parameter / momentum traffic of the update and on the store of the
                        // averaged gradient
    int lds_pad_kib = -1; // KiB of LDS reserved (and never touched) per workgroup of the small-tile kernel, to cap the
                          // workgroups resident per CU; -1 = default for the rank count (see reduce_lds_pad)
};

// ring-ordered N-way reduce (+ optional fused SGD-momentum).
//  slots: device table of N slot base pointers indexed by virtual rank.
//  avg may be null only when p and v are given.
//  With shape.big_unroll != 0 the first n_big tiles must be full big tiles
//  (kBlock * big_unroll * 4 elements, offset a multiple of 4) and all others
//  at most 2048 elements.
hipError_t launch_ring_reduce(hipStream_t s, const Tile* tiles, uint32_t n_tiles, uint32_t n_big,
                              const float* const* slots, uint32_t N,
                              float* avg, float* p, float* v, float lr, float mu,
                              ReduceShape shape);

// stream_pv: streaming accesses to p and v (vectors too large to stay in the caches between steps)
hipError_t launch_sgd(hipStream_t s, float* p, float* v, const float* g, uint64_t n,
                      float lr, float mu, bool stream_pv);

// dst[0..n) <- src[0..n) floats (any 4-byte alignment)
hipError_t launch_copy_f32(hipStream_t s, float* dst, const float* src, uint64_t n);

// Several contiguous runs copied by one launch (batched gradient staging).
constexpr int kMaxRuns = 16;                // the prefix sums then travel in one 64-byte scalar load
struct CopyRuns {
    float*       dst[kMaxRuns];
    const float* src[kMaxRuns];
    uint64_t     n[kMaxRuns];               // floats; dst and src 4-byte aligned
    uint32_t     first_block[kMaxRuns + 1]; // prefix sums of workgroups per run; [n_runs] = total,
                                            // entries after it 0xFFFFFFFF
    uint32_t     n_runs;
};
hipError_t launch_copy_runs(hipStream_t s, const CopyRuns& runs);

enum CtxDir { kSave = 0, kRestore = 1, kSwitch = 2 };
// kSave:    slot_a <- live;  kRestore: live <- slot_a;
// kSwitch:  slot_a <- live, then live <- slot_b (per byte, same lane)
hipError_t launch_ctx(hipStream_t s, const Piece* pieces, uint32_t n_pieces,
                      uint8_t* slot_a, const uint8_t* slot_b, CtxDir dir);

// One launch for an EST boundary: the small-state pieces (kSave or kSwitch) and the staging
// copy of the outgoing EST's runs.  runs.n_runs may be 0, n_pieces may be 0.  The unused
// prefix-sum entries of `runs` must hold 0xFFFFFFFF as for launch_copy_runs.
hipError_t launch_est_boundary(hipStream_t s, const CopyRuns& runs, const Piece* pieces, uint32_t n_pieces,
                               uint8_t* slot_a, const uint8_t* slot_b, CtxDir dir);

// generic byte copy used when contexts move between arenas
hipError_t launch_copy_bytes(hipStream_t s, uint8_t* dst, const uint8_t* src, uint64_t n);

// out[0] = fixed-tree sum of squares of x[0..n), out[1] = its square root;
// part: scratch of ceil(n / 4096) floats
hipError_t launch_sq_norm(hipStream_t s, const float* x, uint64_t n, float* part, float* out);

// The same with the block partials in a file-scope device array of kStaticPartials floats
// (1 MiB per GPU): no allocation; n <= kStaticPartials * 4096, else hipErrorInvalidValue.
// Runs on the current device.
constexpr uint64_t kStaticPartials = 1ull << 18;
hipError_t launch_sq_norm_static(hipStream_t s, const float* x, uint64_t n, float* out);

// v <- mu*v + coef*g ; p <- p - lr*v with coef = min(1, max_norm / (norm2[1] + eps)) formed on the device
hipError_t launch_sgd_clip(hipStream_t s, float* p, float* v, const float* g, uint64_t n,
                           const float* norm2, float max_norm, float eps, float lr, float mu, bool stream_pv);

// Per-channel mean and biased variance of x[B][C][HW] along the fixed tree; B * HW < 2^31,
// C <= 65535; part: scratch of C * ceil(B * HW / 4096) floats
hipError_t launch_bn_batch_stats(hipStream_t s, const float* x, uint32_t B, uint32_t C, uint32_t HW,
                                 float* mean, float* var, float* part);

hipError_t launch_dropout_mask(hipStream_t s, uint64_t* state, uint8_t* mask, uint64_t n,
                               uint64_t threshold);

}  // namespace es
