// Key tiles for the bf16 MFMA kernels (d = 128): coalesced global loads, a padded
// LDS tile, and reads in the operand layout of v_mfma_f32_32x32x16_bf16.
//
// A 32x32x16 MFMA wants from lane (l32 = lane % 32, hh = lane / 32) eight bf16
// of row l32 per k-step.  Loading that straight from global memory makes every
// load instruction touch 32 different rows, 32 bytes each, and the texture
// addresser then caps the stream far below HBM speed.  Instead a workgroup
// copies tiles of 128 consecutive key rows (32 KiB) with fully coalesced
// 16-byte loads (one wave instruction = 1 KiB contiguous), parks them in LDS
// with a row pitch of 272 bytes (the 16 bytes of padding spread the rows over
// the banks), and each wave reads its 32 rows back with ds_read_b128.  Tiles are
// double buffered: the global loads of tile t+1 are in flight while tile t is
// multiplied, and one barrier per tile separates writers from readers.
#pragma once
#include "common.hpp"

namespace gkv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // 16 bytes, a plain vector register group

constexpr int kD = 128;          // head dimension
constexpr int kSteps = 8;        // k-steps of 16 per 128
constexpr int kBlk = 32;         // rows per MFMA block
constexpr int kTileKeys = 128;   // key rows per LDS tile: 4 streams of 32
constexpr int kPitch = 272;      // bytes per key row in LDS (256 + 16 of padding)
constexpr int kTileBytes = kTileKeys * kPitch;
constexpr int kTileChunks = kTileKeys * 16;   // 16-byte pieces per tile

__device__ __forceinline__ bf16x8 load8(const uint16_t *p)
{
    return *reinterpret_cast<const bf16x8 *>(p);
}

// Row of the 32x32 MFMA result held in accumulator register i of a lane in
// half-wave hh (the column is lane % 32).
__device__ __forceinline__ int acc_row(int i, int hh) { return 8 * (i >> 2) + 4 * hh + (i & 3); }

// A thread of an NT-thread workgroup moves ceil(TK * 16 / NT) 16-byte pieces per tile of TK key
// rows (TK = 128 unless a kernel says otherwise).  When NT does not divide the tile (768 threads:
// three pieces each, 2304 slots for 2048 pieces) the threads whose last slot is past the tile
// move their first piece once more: the same bytes to the same place, so that every thread runs
// the same unconditional code.
template <int NT, int TK = kTileKeys> constexpr int tile_pieces() { return (TK * 16 + NT - 1) / NT; }
template <int NT, int TK = kTileKeys> __device__ __forceinline__ int tile_piece(int tid, int u)
{
    const int g = tid + u * NT;
    return ((TK * 16) % NT == 0 || g < TK * 16) ? g : tid;
}

// Global -> registers.  Tile row t is key (first + t) * stride, clamped to
// last_key (rows past the range are loaded from a valid address and masked later).
template <int NT, int TK = kTileKeys, int PER>
__device__ __forceinline__ void tile_load(const uint16_t *Kh, int first, int last_key, int stride,
                                          int tid, u32x4 (&r)[PER])
{
    static_assert(PER == tile_pieces<NT, TK>(), "pieces per thread");
    // (a head's keys span less than 4 GiB -- the MFMA kernels take fewer than 2^24 rows -- so the
    // byte offset fits 32 bits and the load can take the head's base from scalar registers)
    const char *base = reinterpret_cast<const char *>(Kh);
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int g = tile_piece<NT, TK>(tid, u), row = g >> 4, c = g & 15;
        const uint32_t off = (uint32_t)(min(first + row, last_key) * stride) * (uint32_t)(kD * 2) + (uint32_t)c * 16u;
        r[u] = *reinterpret_cast<const u32x4 *>(base + off);
    }
}

// Registers -> LDS tile.
template <int NT, int TK = kTileKeys, int PER>
__device__ __forceinline__ void tile_store(unsigned char *buf, int tid, const u32x4 (&r)[PER])
{
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int g = tile_piece<NT, TK>(tid, u), row = g >> 4, c = g & 15;
        *reinterpret_cast<u32x4 *>(buf + row * kPitch + c * 16) = r[u];
    }
}

// LDS tile -> MFMA operand registers of rows 32*stream .. 32*stream+31.
__device__ __forceinline__ void tile_read(const unsigned char *buf, int stream, int l32, int hh,
                                          bf16x8 (&kc)[kSteps])
{
    const unsigned char *p = buf + (kBlk * stream + l32) * kPitch + 16 * hh;
#pragma unroll
    for (int s = 0; s < kSteps; ++s) kc[s] = *reinterpret_cast<const bf16x8 *>(p + 32 * s);
}

// x of this lane plus x of the lane 32 places away (the other half of the wave), without a
// trip through the LDS crossbar: gfx950's v_permlane32_swap exchanges the upper half of one
// register with the lower half of another, so two copies of x become (low half twice) and
// (high half twice), whose sum is low + high in every lane.  The sums sit between the matrix
// instructions of every tile; a ds_bpermute there would make each wave wait for a turn in the
// LDS queue behind the other waves' tile reads.
__device__ __forceinline__ float add_other_half(float x)
{
    const unsigned u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// 1/|k| from |k|^2 with the hardware reciprocal square root (1 ulp), 0 for a zero key.
// Every MFMA-path edge uses this one function, so the sampled bound and the filtered
// edges are computed bit for bit alike.
__device__ __forceinline__ float inv_norm(float sq)
{
    return sq == 0.f ? 0.f : __builtin_amdgcn_rsqf(sq);
}

// Sum of squares of the 64 elements a lane holds of its row (8 k-steps x 8),
// two bf16 products per instruction, fp32 accumulation.
__device__ __forceinline__ float half_row_sumsq(const bf16x8 (&r)[kSteps])
{
    float a = 0.f;
#pragma unroll
    for (int s = 0; s < kSteps; ++s)
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const bf16x2 v = {r[s][e], r[s][e + 1]};
            a = __builtin_amdgcn_fdot2_f32_bf16(v, v, a, false);
        }
    return a;
}

// The tile loop shared by the streaming kernels.  Tile t is multiplied out of LDS
// while tiles t+1 and t+2 are on their way from HBM in two sets of staging
// registers: two tiles (64 KiB) in flight per workgroup (a third set brought no
// gain when measured).  One barrier per tile separates the writers of an LDS
// buffer from its readers.  `body(buf, t)` multiplies tile t; AFTER_TILE runs
// right after each tile's barrier with `tile_done` = number of tiles finished (it
// may contain barriers: every thread reaches it).  The loop is unrolled twice so
// that the LDS buffer and the register set of a tile are compile-time choices.
//
// The prefetch loads are issued unconditionally, also past the last tile (rows are
// clamped to `clamp_`, the last row the workgroup needs, so those loads hit one
// cached row): the compiler can then count the loads in flight exactly and the
// wait in front of each LDS store leaves the newer tile's loads outstanding.
// With conditional loads it has to assume they were skipped and waits for
// everything.
#define GKV_TILE_PIPELINE_TK(TK_, NT_, Kh_, first_, clamp_, stride_, ntile_, body, AFTER_TILE)         \
    do {                                                                                               \
        constexpr int tile_bytes_ = (TK_) * kPitch;                                                    \
        u32x4 stage_a[tile_pieces<NT_, TK_>()], stage_b[tile_pieces<NT_, TK_>()];                      \
        tile_load<NT_, TK_>(Kh_, first_, clamp_, stride_, tid, stage_a);                               \
        tile_store<NT_, TK_>(kt, tid, stage_a);                                                        \
        tile_load<NT_, TK_>(Kh_, first_ + (TK_), clamp_, stride_, tid, stage_a);                       \
        tile_load<NT_, TK_>(Kh_, first_ + 2 * (TK_), clamp_, stride_, tid, stage_b);                   \
        __syncthreads();                                                                               \
        for (int t_ = 0; t_ < ntile_; t_ += 2) {                                                       \
            body(kt, t_);                                                                              \
            tile_store<NT_, TK_>(kt + tile_bytes_, tid, stage_a);                                      \
            tile_load<NT_, TK_>(Kh_, first_ + (TK_) * (t_ + 3), clamp_, stride_, tid, stage_a);        \
            __syncthreads();                                                                           \
            { const int tile_done = t_ + 1; (void)tile_done; AFTER_TILE; }                             \
            if (t_ + 1 >= ntile_) break;                                                               \
            body(kt + tile_bytes_, t_ + 1);                                                            \
            tile_store<NT_, TK_>(kt, tid, stage_b);                                                    \
            tile_load<NT_, TK_>(Kh_, first_ + (TK_) * (t_ + 4), clamp_, stride_, tid, stage_b);        \
            __syncthreads();                                                                           \
            { const int tile_done = t_ + 2; (void)tile_done; AFTER_TILE; }                             \
        }                                                                                              \
    } while (0)

// The same loop for kernels that overlap the matrix products of one tile with the vector work on
// the tile before it (a wave issues instructions in order: vector work placed between the matrix
// instructions runs while the matrix core is busy, vector work placed after them waits for all of
// them to be issued).  Such a kernel keeps two sets of accumulators.  `head(buf)` multiplies tile
// 0 into set 0; `body(buf, t, set)` multiplies tile t into `set` and finishes tile t - 1 from the
// other set; `tail(t, set)` finishes the last tile.  `set` is a literal at every call, so the
// accumulator sets stay in registers.
#define GKV_TILE_PIPELINE_OVERLAPPED(TK_, NT_, Kh_, first_, clamp_, stride_, ntile_, head, body, tail)  \
    do {                                                                                               \
        constexpr int tile_bytes_ = (TK_) * kPitch;                                                    \
        u32x4 stage_a[tile_pieces<NT_, TK_>()], stage_b[tile_pieces<NT_, TK_>()];                      \
        tile_load<NT_, TK_>(Kh_, first_, clamp_, stride_, tid, stage_a);                               \
        tile_store<NT_, TK_>(kt, tid, stage_a);                                                        \
        tile_load<NT_, TK_>(Kh_, first_ + (TK_), clamp_, stride_, tid, stage_a);                       \
        tile_load<NT_, TK_>(Kh_, first_ + 2 * (TK_), clamp_, stride_, tid, stage_b);                   \
        __syncthreads();                                                                               \
        head(kt);                                                                                      \
        tile_store<NT_, TK_>(kt + tile_bytes_, tid, stage_a);                                          \
        tile_load<NT_, TK_>(Kh_, first_ + 3 * (TK_), clamp_, stride_, tid, stage_a);                   \
        __syncthreads();                                                                               \
        int t_ = 1;                                                                                    \
        for (; t_ < ntile_; t_ += 2) {                                                                 \
            body(kt + tile_bytes_, t_, 1);                                                             \
            tile_store<NT_, TK_>(kt, tid, stage_b);                                                    \
            tile_load<NT_, TK_>(Kh_, first_ + (TK_) * (t_ + 3), clamp_, stride_, tid, stage_b);        \
            __syncthreads();                                                                           \
            if (t_ + 1 >= ntile_) break;                                                               \
            body(kt, t_ + 1, 0);                                                                       \
            tile_store<NT_, TK_>(kt + tile_bytes_, tid, stage_a);                                      \
            tile_load<NT_, TK_>(Kh_, first_ + (TK_) * (t_ + 4), clamp_, stride_, tid, stage_a);        \
            __syncthreads();                                                                           \
        }                                                                                              \
        if ((ntile_ - 1) & 1) tail(ntile_ - 1, 1); else tail(ntile_ - 1, 0);                           \
    } while (0)

#define GKV_TILE_PIPELINE(NT_, Kh_, first_, clamp_, stride_, ntile_, body, AFTER_TILE) \
    GKV_TILE_PIPELINE_TK(kTileKeys, NT_, Kh_, first_, clamp_, stride_, ntile_, body, AFTER_TILE)

}  // namespace gkv
