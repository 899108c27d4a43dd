// Eq. 1 and Eq. 3 on the matrix cores: cosine of every source key against every
// prefix key (bf16 inputs, d = 128, fp32 accumulation), and each source's m
// largest edges without ever storing the S x P edge block.
//
// Up to 96 source rows (three 32-row MFMA blocks, one per row group of waves) are
// held in registers; keys stream from HBM through LDS tiles into MFMA operand
// registers, as in the scoring kernels.  The squared norm of each streamed key is
// accumulated from the very registers that feed the MFMA, so the keys are read once.
//
// Neighbourhoods in one streaming pass:
//   1. a first pass over an evenly strided sample of the keys (every 8th) counts
//      each source's edges into a histogram and takes a bound from it: the sampled
//      edge of rank r, where r < m is chosen so that all but about one source in 10^7
//      have at least m edges above it (mfma_bound_rank; r = m would make that certain,
//      a subset's m-th largest can only be smaller, but lets 8 m keys through
//      where r lets 8 r);
//   2. the streaming pass keeps only the edges that reach the bound (a couple of
//      hundred per source), staged in LDS and appended to per-source lists;
//   3. an exact (value desc, index asc) top-m over each short list -- exact whenever
//      the list holds m entries or more, since it then holds every edge that is at
//      least the bound and the m largest are among those.
// A source whose list overflows (masses of equal edges, adversarial order) or comes
// out short of m entries sets a per-head flag and that head is redone exactly, row by
// row (redo_rows in select.hip).
//
// A neighbourhood depends on the keys alone, so a source that comes back in a later
// round keeps its list.  The first round's passes also take a third 32-row group per
// workgroup: the nodes ranked right behind the sources, which are the likeliest new
// sources of the following rounds (the decay only lowers scores, so whoever moves up
// comes from just below the cut).  Their candidate lists are kept, and a later round
// runs the exact select on them when they are promoted; only a new source without a
// kept list goes through the bound and filter passes again (a per-head count of rows
// in use; heads without such a source return at once).
#include "common.hpp"
#include "kernels.hpp"
#include "mfma_tile.hpp"

#include <math.h>

namespace gkv {

namespace {

constexpr int kSB = 2;            // source blocks of 32 per workgroup = row groups of waves
constexpr int kRows = kSB * kBlk; // source rows per workgroup
constexpr int kThreads = 256 * kSB;

// The per-row buffers (tau, cand, cand_cnt) hold `pitch` rows per head; the rows of one launch's
// source list start at row `row0` of them.
struct FilterArgs {
    const int32_t *n_src;  // [Hkv] rows of the head's source list in use; null: all S
    const float *tau;      // [Hkv, pitch] the bound pass's value per row: edges below it are dropped
    uint2 *cand;           // [Hkv, pitch, chunks, slice_cap] (edge bits, key index): one slice per key chunk
    int32_t *cand_cnt;     // [Hkv, pitch, chunks] entries in each slice
    int32_t *overflow;     // [Hkv]
    int slice_cap;
    int drain_every;       // tiles between two scheduled drains of the rings
    int sgroups;           // workgroups (groups of source rows) per key chunk
    int src_pitch;         // entries per head of the source list
    int pitch, row0;
};

// Both kernels below: a workgroup has 4 key streams (wave & 3) and 2 source row
// groups (wave >> 2): wave (stream, g) multiplies source rows 32g .. 32g+31 of its
// 64-row group with rows 32*stream .. +31 of every key tile.  Two waves share a
// SIMD and overlap each other's MFMA and vector work.  The edge is
// e = (dot * 1/|k_j|) * 1/|k_i| in both, so the sample pass and the filter pass
// produce the same bits.

// Sources are rows of Ac, the streamed rows are rows of Kc (both [Hkv, N, 128]); for
// Eq. 1 both are the keys, the other pairings of the paper's Discussion pass two tensors.
// This wave's 32 source rows -> MFMA operand registers (slots beyond S repeat the
// last source); 1/|k_i| and the source index of the workgroup's rows go to LDS.
__device__ __forceinline__ void load_sources(const uint16_t *Ah, const int32_t *src_h, int S,
                                             int s_base, int grp, int stream, int l32, int hh,
                                             bf16x8 (&q)[kSteps], float *inv_s, int32_t *idx_s)
{
    const int slot = min(s_base + kBlk * grp + l32, S - 1);
    const int32_t i = src_h[slot];
    const uint16_t *p = Ah + (long)i * kD + 8 * hh;
#pragma unroll
    for (int s = 0; s < kSteps; ++s) q[s] = load8(p + 16 * s);
    float sq = half_row_sumsq(q);
    sq = add_other_half(sq);
    if (stream == 0 && hh == 0) {
        inv_s[kBlk * grp + l32] = inv_norm(sq);
        idx_s[kBlk * grp + l32] = i;
    }
}

// Dense block: E[h, slot, c] = e for column c = key c * key_stride (key_stride = 1:
// every key), -inf where the key is the source itself.  If fa.overflow is set, the first
// workgroup of a head also clears the head's overflow flag for the filter pass that follows.
__global__ __launch_bounds__(kThreads) void cosine_dense_kernel(
    const uint16_t *__restrict__ Ac, const uint16_t *__restrict__ Kc, int N, int n_cols, int key_stride, int S,
    const int32_t *__restrict__ src, int chunk_cols, float *__restrict__ E, FilterArgs fa,
    const int32_t *__restrict__ gate)
{
    __shared__ float inv_s[kRows];
    __shared__ int32_t idx_s[kRows];
    extern __shared__ __align__(16) unsigned char smem[];   // two key tiles
    unsigned char *kt = smem;

    const int h = blockIdx.y, chunk = blockIdx.x, s_base = blockIdx.z * kRows;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, hh = lane >> 5;
    const int stream = wv & 3, grp = wv >> 2;
    if (gate && gate[h] == 0) return;
    const uint16_t *Kh = Kc + (long)h * N * kD;
    const int c0 = chunk * chunk_cols, c1 = min(n_cols, c0 + chunk_cols);
    if (c0 >= n_cols) return;

    if (fa.overflow && chunk == 0 && blockIdx.z == 0 && tid == 0) fa.overflow[h] = 0;

    bf16x8 q[kSteps];
    load_sources(Ac + (long)h * N * kD, src + (long)h * S, S, s_base, grp, stream, l32, hh, q, inv_s, idx_s);
    __syncthreads();
    float inv_src[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) inv_src[i] = inv_s[kBlk * grp + acc_row(i, hh)];

    const int ntile = (c1 - c0 + kTileKeys - 1) / kTileKeys;
    auto multiply_tile = [&](const unsigned char *buf, int t) {
        bf16x8 kc[kSteps];
        tile_read(buf, stream, l32, hh, kc);
        f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
        for (int s = 0; s < kSteps; ++s)   // rows = sources, columns = keys
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q[s], kc[s], acc, 0, 0, 0);

        float sq = half_row_sumsq(kc);
        sq = add_other_half(sq);
        const float inv_k = inv_norm(sq);
        const int col = c0 + kTileKeys * t + kBlk * stream + l32;
        const int key = col * key_stride;
        if (col < c1) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int slot = s_base + kBlk * grp + acc_row(i, hh);
                if (slot < S) {
                    float e = (acc[i] * inv_k) * inv_src[i];
                    if (key == idx_s[kBlk * grp + acc_row(i, hh)]) e = -INFINITY;
                    E[((long)h * S + slot) * n_cols + col] = e;
                }
            }
        }
    };
    GKV_TILE_PIPELINE(kThreads, Kh, c0, c1 - 1, key_stride, ntile, multiply_tile, (void)0);
}

// Bound pass: for every source a value that at least m of its edges reach (short of about one
// source in 10^7, which the select catches), from the edges to a strided sample of the keys
// (column c = key c * key_stride).  `m` below is the rank in the sample that the host chose
// (mfma_bound_rank).  One workgroup takes the whole
// sample of a (head, source group): the edges never leave the registers, they are
// counted into a 256-bin histogram over [-1, 1] per source in LDS, and the bound is
// the lower edge of the bin in which the count from the top reaches m: at most 1/128
// below the m-th largest sampled edge.  (The pass is bound by the vector instructions
// that turn an edge into a bin: a plain counter per bin needs five of them per edge;
// packed 16-bit counters in twice as many bins needed eleven and made this pass 15 %
// slower for a bound that saves the filter pass 1 %.  Bins over [0, 1] only, with all
// negative edges in the lowest bin, are no option: half the updates then hit one LDS
// word.  An edge a rounding error below a bin edge may be counted into the bin above;
// the filter pass lowers every bound by far more than that.)  The source's own column
// is taken out of the counts at the end (Eq. 3: j != i).  Also clears the head's
// overflow flag for the filter pass that follows.
// One wave, one source: lane L holds the counters of bins 4L .. 4L+3 in w4 (zeros beyond the
// last bin).  Finds the bin in which the count from the top reaches m and writes its lower edge.
template <int BINS>
__device__ __forceinline__ void bound_from_histogram(const uint4 w4, int m, int lane, float *tau_row)
{
    const uint32_t c[4] = {w4.x, w4.y, w4.z, w4.w};
    uint32_t mine = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) mine += c[k];
    uint32_t from_top = mine;   // count in this lane's bins and all higher ones
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t v = __shfl_down(from_top, o, kWave);
        if (lane + o < 64) from_top += v;
    }
    const uint32_t above = from_top - mine;
    if (above < (uint32_t)m && from_top >= (uint32_t)m) {
        uint32_t cum = above;
        int k = 3;
        for (; k > 0; --k) {
            if (cum + c[k] >= (uint32_t)m) break;
            cum += c[k];
        }
        *tau_row = (float)(4 * lane + k) * (2.0f / BINS) - 1.0f;
    }
    if (lane == 0 && from_top < (uint32_t)m) *tau_row = -INFINITY;   // fewer than m sampled edges: no bound
}

// Lane L's four counters of one histogram row (BINS words).
template <int BINS>
__device__ __forceinline__ uint4 histogram_words(const uint32_t *row, int lane)
{
    return lane < BINS / 4 ? *reinterpret_cast<const uint4 *>(row + 4 * lane) : make_uint4(0, 0, 0, 0);
}

// SB 32-row groups of sources per workgroup (4 SB waves); BINS bins over [-1, 1]: 256 for two
// groups, 224 for three (the histograms of 96 rows and the two key tiles must fit the LDS), so
// the bound is at most 2 / BINS below the m-th largest sampled edge.
template <int SB, int BINS>
__global__ __launch_bounds__(256 * SB) void cosine_bound_kernel(
    const uint16_t *__restrict__ Ac, const uint16_t *__restrict__ Kc, int N, int n_cols, int key_stride,
    int S, int src_pitch, const int32_t *__restrict__ src, const int32_t *__restrict__ n_src, int m,
    int chunk_cols, uint32_t *__restrict__ hist_part, float *__restrict__ tau, int pitch, int row0,
    int32_t *__restrict__ overflow)
{
    constexpr int ROWS = SB * kBlk, NT = 256 * SB;
    __shared__ float inv_s[ROWS];
    __shared__ int32_t idx_s[ROWS];
    extern __shared__ __align__(16) unsigned char smem[];   // two key tiles, then the histograms
    unsigned char *kt = smem;
    uint32_t *hist = reinterpret_cast<uint32_t *>(smem + 2 * kTileBytes);   // [ROWS][BINS]

    // with few heads the sample is cut into chunks (blockIdx.z) whose histograms are added up
    // by bound_merge_kernel: otherwise a handful of workgroups would walk the sample alone
    const int h = blockIdx.y, s_base = blockIdx.x * ROWS, chunk = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, hh = lane >> 5;
    const int stream = wv & 3, grp = wv >> 2;
    const uint16_t *Kh = Kc + (long)h * N * kD;
    const int c0 = chunk * chunk_cols, c1 = min(n_cols, c0 + chunk_cols);
    if (blockIdx.x == 0 && chunk == 0 && tid == 0) overflow[h] = 0;
    // rows of this head's source list in use
    const int Sh = n_src ? n_src[h] : S;
    if (s_base >= Sh) return;

    bf16x8 q[kSteps];
    load_sources(Ac + (long)h * N * kD, src + (long)h * src_pitch, Sh, s_base, grp, stream, l32, hh, q, inv_s, idx_s);
    for (int u = tid; u < ROWS * BINS; u += NT) hist[u] = 0;
    __syncthreads();
    float inv_src[16];   // 1/|k_i| times half the number of bins: edge -> bin in one multiply-add
#pragma unroll
    for (int i = 0; i < 16; ++i) inv_src[i] = inv_s[kBlk * grp + acc_row(i, hh)] * (0.5f * BINS);

    const int ntile = c1 > c0 ? (c1 - c0 + kTileKeys - 1) / kTileKeys : 0;
    auto multiply_tile = [&](const unsigned char *buf, int t) {
        bf16x8 kc[kSteps];
        tile_read(buf, stream, l32, hh, kc);
        f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
        for (int s = 0; s < kSteps; ++s)   // rows = sources, columns = keys
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q[s], kc[s], acc, 0, 0, 0);

        float sq = half_row_sumsq(kc);
        sq = add_other_half(sq);
        const float inv_k = inv_norm(sq);
        const int col = c0 + kTileKeys * t + kBlk * stream + l32;
        if (col < c1) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                // (e + 1) BINS / 2 with e = (dot / |k_j|) / |k_i|, the dense kernel's edge up to rounding
                int b = (int)fmaf(acc[i] * inv_k, inv_src[i], 0.5f * BINS);
                b = b < 0 ? 0 : (b > BINS - 1 ? BINS - 1 : b);
                atomicAdd(&hist[(kBlk * grp + acc_row(i, hh)) * BINS + b], 1u);
            }
        }
    };
    if (ntile > 0) GKV_TILE_PIPELINE(NT, Kh, c0, c1 - 1, key_stride, ntile, multiply_tile, (void)0);
    __syncthreads();
    // The source's own column is no neighbour (Eq. 3: j != i).  If it is one of the sampled
    // keys of this workgroup it was counted into the top bin (its edge is 1 up to rounding;
    // a zero source, all of whose edges are 0, has nothing there): take it out again.
    if (tid < ROWS) {
        const int32_t i = idx_s[tid];
        const int col = i / key_stride;
        if (i % key_stride == 0 && col >= c0 && col < c1) {
            uint32_t &top = hist[tid * BINS + BINS - 1];
            if (top > 0u) top -= 1u;
        }
    }
    __syncthreads();

    if (gridDim.z > 1) {   // this chunk's counts go to global memory
        uint4 *out = reinterpret_cast<uint4 *>(
            hist_part + ((((long)h * gridDim.x + blockIdx.x) * gridDim.z + chunk) * ROWS) * BINS);
        const uint4 *in = reinterpret_cast<const uint4 *>(hist);
        for (int u = tid; u < ROWS * BINS / 4; u += NT) out[u] = in[u];
        return;
    }
    // Wave w scans the histograms of rows 8w .. 8w+7 from the top; lane L holds bins 8L .. 8L+7.
    for (int r = 0; r < 8; ++r) {
        const int row = wv * 8 + r;
        const uint4 w4 = histogram_words<BINS>(&hist[row * BINS], lane);
        if (s_base + row < Sh) bound_from_histogram<BINS>(w4, m, lane, &tau[(long)h * pitch + row0 + s_base + row]);
    }
}

// Adds up the histograms of the sample's chunks and takes the bound.  One
// wave per source.
template <int SB, int BINS>
__global__ __launch_bounds__(256) void bound_merge_kernel(const uint32_t *__restrict__ hist_part,
                                                          int chunks, int sgroups, int S,
                                                          const int32_t *__restrict__ n_src, int m,
                                                          float *__restrict__ tau, int pitch, int row0)
{
    constexpr int ROWS = SB * kBlk;
    const int lane = threadIdx.x & 63;
    const int slot = blockIdx.x * 4 + (threadIdx.x >> 6), h = blockIdx.y;
    if (slot >= (n_src ? n_src[h] : S)) return;
    const int sg = slot / ROWS, row = slot % ROWS;
    uint4 w4 = make_uint4(0, 0, 0, 0);
    for (int c = 0; c < chunks; ++c) {
        const uint4 v = histogram_words<BINS>(
            hist_part + ((((long)h * sgroups + sg) * chunks + c) * ROWS + row) * BINS, lane);
        w4.x += v.x; w4.y += v.y; w4.z += v.z; w4.w += v.w;
    }
    bound_from_histogram<BINS>(w4, m, lane, &tau[(long)h * pitch + row0 + slot]);
}

// Filter pass over all keys.  A lane holds, per key block, the 16 dots of its key
// with 16 of the wave's sources.  It tests them all at once against the sources'
// bounds (dot >= bound_i * |k_j|, bounds a hair lowered so that rounding can never
// lose an edge) with 16 fused multiply-adds and a max tree; the few lanes that
// have a hit park their 16 dots, the key's squared norm and the key index in an
// LDS ring.  Every half-wave has a ring of its own and positions are a prefix
// count over the hit lanes, so parking needs no atomic and waits for nothing.
// Every few tiles (a schedule the host derives from the expected hit rate, so
// that most of a half-wave's 32 lanes get a row) all waves drain their rings at
// the same time -- a drain is a chain of LDS round trips, and a wave that drains
// alone would keep the others waiting at the tile barrier.  A half-wave
// drains its own ring, so the 16 sources of a parked row are the draining lane's
// own 16 sources and their bounds sit in registers: the same test picks the row's
// hits, their dots become exact edges (the dense kernel's formula, bit for bit),
// and they are appended to the workgroup's own slice of each source's global
// candidate list (one slice per key chunk, so no workgroup ever waits for
// another: positions come from LDS counters).  A ring holds RING rows (64 with two
// row groups per workgroup, 32 with three: the rings share the LDS with the key
// tiles); before a tile's rows are parked a wave drains on its own if a ring could
// not take them.  The source's own column may be among the candidates:
// the exact select drops it.  If a slice (or one of the short LDS lists that take
// a row's hits beyond its fourth) overflows, the head's overflow flag is raised and
// the head is redone exactly, row by row.
constexpr int kStagePitch = 80;    // bytes per parked row: 16 dots, |k|^2, key (72, padded)
constexpr int kLaterCap = 128;     // entries of each of the two LDS lists of hits beyond a row's fourth

template <int SB, int RING>
__global__ __launch_bounds__(256 * SB) void cosine_filter_kernel(
    const uint16_t *__restrict__ Ac, const uint16_t *__restrict__ Kc, int N, int n_cols, int S,
    const int32_t *__restrict__ src, int chunk_cols, FilterArgs fa)
{
    constexpr int ROWS = SB * kBlk, NT = 256 * SB;
    static_assert(RING == 32 || RING == 64, "a ring takes a tile's 32 rows and is indexed with a mask");
    __shared__ float inv_s[ROWS], det_s[ROWS];
    __shared__ int32_t idx_s[ROWS];
    __shared__ int32_t row_pos[ROWS];   // entries written to each source's slice
    __shared__ int32_t idle_pos[kWave];  // takes the additions of 0 of hits that are not there
    // (edge bits, key, source row) of the hits beyond a row's fourth: one list for even and one
    // for odd drain periods, each emptied right after the barrier that ends its period
    __shared__ uint4 later[2][kLaterCap];
    __shared__ int32_t n_later[2], later_lost;   // entries ever listed (never reset)
    extern __shared__ __align__(16) unsigned char smem[];   // two key tiles, then the rings
    unsigned char *kt = smem;
    unsigned char *stage_mem = smem + 2 * kTileBytes;

    // The workgroups that stream the same keys (the source groups of a key chunk) should run at
    // about the same time on the same XCD, so that all but the first find the keys in that XCD's
    // L2.  Workgroups go to the 8 XCDs round robin in the order of their linear number, so the
    // groups of one (head, chunk) unit sit 8 apart: 8 units x all their groups take 8 x sgroups
    // consecutive numbers.  (Unit counts that are no multiple of 8 keep the plain order.)
    const int n_chunks = gridDim.x / fa.sgroups;
    int h = blockIdx.y, chunk = blockIdx.x / fa.sgroups, s_base = (blockIdx.x % fa.sgroups) * ROWS;
    if (fa.sgroups > 1 && ((long)gridDim.y * n_chunks) % 8 == 0) {
        const long lin = (long)blockIdx.y * gridDim.x + blockIdx.x;
        const long grp8 = lin / (8 * fa.sgroups);
        const int r = (int)(lin % (8 * fa.sgroups));
        const long unit = grp8 * 8 + (r & 7);
        h = (int)(unit / n_chunks);
        chunk = (int)(unit % n_chunks);
        s_base = (r >> 3) * ROWS;
    }
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, hh = lane >> 5;
    const int stream = wv & 3, grp = wv >> 2;
    const uint16_t *Kh = Kc + (long)h * N * kD;
    const int c0 = chunk * chunk_cols, c1 = min(n_cols, c0 + chunk_cols);
    if (c0 >= n_cols) return;
    const int Sh = fa.n_src ? fa.n_src[h] : S;
    if (s_base >= Sh) return;
    const long buf_row0 = (long)h * fa.pitch + fa.row0 + s_base;   // this workgroup's first row of the per-row buffers

    bf16x8 q[kSteps];
    load_sources(Ac + (long)h * N * kD, src + (long)h * fa.src_pitch, Sh, s_base, grp, stream, l32, hh, q, inv_s, idx_s);
    if (tid < ROWS) row_pos[tid] = 0;
    if (tid < 2) n_later[tid] = 0;
    if (tid == 0) later_lost = 0;
    __syncthreads();
    if (tid < ROWS) {
        // det: what dot / |k_j| must reach for the edge to be listed, i.e. the source's bound,
        // lowered by twice the slack, divided by 1/|k_i|.  Rows past the last source and
        // impossible bounds never hit; a zero source (all edges 0) hits everywhere.
        const int slot = s_base + tid;
        const float t = fa.tau[buf_row0 + min(tid, Sh - 1 - s_base)];
        const float slack = 4e-6f + 1e-5f * fabsf(t);
        const float inv = inv_s[tid];
        const float lo2 = t - 2.f * slack;
        det_s[tid] = slot >= Sh ? INFINITY : (inv > 0.f ? lo2 / inv : (lo2 <= 0.f ? -INFINITY : INFINITY));
    }
    __syncthreads();
    // this lane's 16 sources: row acc_row(i, hh) of row group grp
    float det[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) det[i] = det_s[kBlk * grp + acc_row(i, hh)];

    unsigned char *ring = stage_mem + (2 * wv + hh) * (RING * kStagePitch);
    const uint64_t half_before = (hh ? 0xffffffff00000000ull : 0x00000000ffffffffull) & ((1ull << lane) - 1ull);
    uint2 *slice0 = fa.cand + (buf_row0 * n_chunks + chunk) * fa.slice_cap;
    const long slice_row_stride = (long)n_chunks * fa.slice_cap;
    // rows ever parked / ever drained by the lower and the upper half-wave (same in every lane)
    int tail0 = 0, tail1 = 0, head0 = 0, head1 = 0;

    // Each half-wave turns up to 32 waiting rows of its ring into list entries, one per lane.
    // No loop in here holds a global store: after such a loop the compiler can no longer
    // count the memory operations in flight and would make the next LDS store of a key tile
    // wait for every outstanding prefetch.  A row's first four hits are stored by straight-
    // line code; further ones (keys that are close to many sources at once) go to the LDS
    // list of the current tile's parity.
    auto drain = [&](int par) {
        const int n0 = min(tail0 - head0, kBlk), n1 = min(tail1 - head1, kBlk);
        if (l32 < (hh ? n1 : n0)) {
            const unsigned char *row_mem = ring + (((hh ? head1 : head0) + l32) & (RING - 1)) * kStagePitch;
            const float4 *vals = reinterpret_cast<const float4 *>(row_mem);
            const float2 extra = *reinterpret_cast<const float2 *>(row_mem + 64);   // |k|^2, key
            const float inv_k = inv_norm(extra.x);   // the dense kernel's formula
            const float norm_k = __builtin_amdgcn_sqrtf(extra.x);
            const uint32_t key = __float_as_uint(extra.y);
            // the test that parked the row, source by source: bit i of `hits` = (dot_i - det_i |k|
            // is not negative), gathered from the sign bits, source 15 first
            uint32_t neg = 0;
#pragma unroll
            for (int v = 3; v >= 0; --v) {
                const float4 dv = vals[v];
                const float d4[4] = {dv.x, dv.y, dv.z, dv.w};
#pragma unroll
                for (int u = 3; u >= 0; --u)
                    neg = __builtin_amdgcn_alignbit(neg, __float_as_uint(fmaf(-det[4 * v + u], norm_k, d4[u])), 31);
            }
            uint32_t hits = ~neg & 0xffffu;
            // The row's first four hits without a branch, so that their LDS reads and list
            // positions are asked for together and waited for once: a hit that is not there
            // reads dot 0 and adds 0 to a counter nobody reads (one per lane).
            int rowk[4];
            int32_t atk[4];
            float dotk[4], invk[4];
            uint32_t validk = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const bool valid = hits != 0;
                const int i = valid ? __ffs(hits) - 1 : 0;
                hits &= hits - 1;
                validk |= valid ? 1u << k : 0u;
                rowk[k] = kBlk * grp + acc_row(i, hh);
                dotk[k] = reinterpret_cast<const float *>(row_mem)[i];
                invk[k] = inv_s[rowk[k]];
                atk[k] = atomicAdd(valid ? &row_pos[rowk[k]] : &idle_pos[lane], valid ? 1 : 0);
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) asm volatile("" : "+v"(dotk[k]), "+v"(invk[k]), "+v"(atk[k]));
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (((validk >> k) & 1u) && atk[k] < fa.slice_cap)
                    slice0[rowk[k] * slice_row_stride + atk[k]] =
                        make_uint2(__float_as_uint((dotk[k] * inv_k) * invk[k]), key);
            while (hits) {
                const int i = __ffs(hits) - 1;
                hits &= hits - 1;
                const int row = kBlk * grp + acc_row(i, hh);
                const float e = (reinterpret_cast<const float *>(row_mem)[i] * inv_k) * inv_s[row];
                const int at = atomicAdd(&n_later[par], 1);
                later[par][at & (kLaterCap - 1)] = make_uint4(__float_as_uint(e), key, (uint32_t)row, 0u);
            }
        }
        head0 += n0;
        head1 += n1;
    };

    const int ntile = (c1 - c0 + kTileKeys - 1) / kTileKeys;
    // The host's schedule is for lanes whose 16 rows are all sources; with fewer (a short
    // list fills the rows in order, four to a lane at a time) the rings fill that much slower.
    const int lane_rows = min(16, 4 * ((min(Sh - s_base, kBlk) + 7) / 8));
    const int de = fa.drain_every * 16 / lane_rows;
    // Tiles come in periods of `de`, the last tile of a period being the one with the scheduled
    // drain.  Hits beyond a row's fourth go to the LDS list of the period's parity, which is stored
    // once the period has ended, while the next period fills the other list.
    int period = 0, period_end = de - 1;   // (the same in every thread)
    // a row group without sources only helps to move the key tiles
    const bool idle = s_base + kBlk * grp >= Sh;
    // Entries listed during the period that just ended are final behind its last barrier, and the
    // next period lists into the other list: one thread per entry stores them.  A list holds
    // kLaterCap entries; more than that in one period and the head is redone exactly.  The list of
    // a period is stored during the first tile of the next one, inside the tile's work and in
    // front of its prefetch loads: a store behind the tile barrier would sit between the loads of
    // two tiles, and the compiler then makes every other tile wait for all loads in flight
    // instead of leaving the newer tile's outstanding.  (Threads 0 .. 127 do it: they belong to
    // the first row group, which always has sources.)
    int later_seen[2] = {0, 0};
    auto store_later = [&](int par) {
        const int n = n_later[par];
        const int x = later_seen[par] + tid;
        if (n - later_seen[par] > kLaterCap && tid == 0) later_lost = 1;
        later_seen[par] = n;
        if (x < n) {
            const uint4 r = later[par][x & (kLaterCap - 1)];
            const int at = atomicAdd(&row_pos[r.z], 1);
            if (at < fa.slice_cap) slice0[(long)r.z * slice_row_stride + at] = make_uint2(r.x, r.y);
        }
    };
    auto multiply_tile = [&](const unsigned char *buf, int t) {
        if (idle) return;
        if (period > 0 && t == period_end - de + 1) store_later((period - 1) & 1);
        bf16x8 kc[kSteps];
        tile_read(buf, stream, l32, hh, kc);
        f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
        for (int s = 0; s < kSteps; ++s)   // rows = sources, columns = keys
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q[s], kc[s], acc, 0, 0, 0);

        float sq = half_row_sumsq(kc);
        sq = add_other_half(sq);
        const float norm_k = __builtin_amdgcn_sqrtf(sq);
        float d[16];   // dot - bound * |k_j|: >= 0 means the edge may reach the bound
#pragma unroll
        for (int i = 0; i < 16; ++i) d[i] = fmaf(-det[i], norm_k, acc[i]);
        float best = d[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) best = fmaxf(best, d[i]);
        const int key = c0 + kTileKeys * t + kBlk * stream + l32;
        const bool hit = best >= 0.f && key < c1;
        const uint64_t hit_lanes = __ballot(hit);
        const int add0 = (int)__popcll(hit_lanes & 0x00000000ffffffffull), add1 = (int)__popcll(hit_lanes >> 32);
        // a ring that could not take this tile's rows is drained first: one pass takes up to
        // 32 rows out, after which the (at most 32) new rows fit
        if (tail0 - head0 + add0 > RING || tail1 - head1 + add1 > RING) drain(period & 1);
        if (hit) {
            const int at = (hh ? tail1 : tail0) + (int)__popcll(hit_lanes & half_before);
            unsigned char *row_mem = ring + (at & (RING - 1)) * kStagePitch;
#pragma unroll
            for (int v = 0; v < 4; ++v)
                *reinterpret_cast<float4 *>(row_mem + 16 * v) =
                    make_float4(acc[4 * v], acc[4 * v + 1], acc[4 * v + 2], acc[4 * v + 3]);
            *reinterpret_cast<float2 *>(row_mem + 64) = make_float2(sq, __int_as_float(key));
        }
        tail0 += add0;
        tail1 += add1;
        // A scheduled drain empties the rings (a pass takes 32 rows per half-wave).  It sits
        // here, in front of the tile's prefetch loads: the drain's stores are then older than
        // those loads, and the wait in front of the next LDS store of a key tile -- a count of
        // memory operations still in flight -- lets the loads stay in flight.
        if (t == period_end) {
            drain(period & 1);
            if (RING > kBlk) drain(period & 1);
        }
    };
    auto end_of_tile = [&](int tile_done) {
        if (tile_done - 1 == period_end) {
            ++period;
            period_end += de;
        }
    };
    GKV_TILE_PIPELINE(NT, Kh, c0, c1 - 1, 1, ntile, multiply_tile, end_of_tile(tile_done));
    drain(period & 1);
    drain(period & 1);
    __syncthreads();
    if (!idle) {
        store_later(0);
        store_later(1);
    }
    __syncthreads();      // every candidate is counted
    if (tid < ROWS && s_base + tid < Sh) {
        const int c = row_pos[tid];
        fa.cand_cnt[(buf_row0 + tid) * n_chunks + chunk] = c < fa.slice_cap ? c : fa.slice_cap;
        if (c > fa.slice_cap || later_lost) fa.overflow[h] = 1;
    }
}

constexpr int kTieRoom = 64;   // entries tied at the cut that a select lists beyond the m winners

__device__ __forceinline__ uint32_t ord_key_u(uint32_t bits)
{
    float f = __uint_as_float(bits) + 0.0f;
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Inverse of the map above (the bits of the float a key stands for).
__device__ __forceinline__ uint32_t ord_key_inv(uint32_t k)
{
    return (k & 0x80000000u) ? (k ^ 0x80000000u) : ~k;
}

// Exact top-m of one source's candidate list by (edge desc, key index asc),
// written in ascending key order.  The workgroups of a head share its sources in
// turn (a workgroup's next list is asked for while it works on the current one);
// heads whose overflow flag is set are left to the exact fallback.
//
// The m-th largest edge value is found by a radix select over the order-
// preserving keys of the (short) list, as in the row top-k; entries above it are
// in, and of the entries equal to it the `need` lowest key indices are in.  The
// winners' output position is their rank by key index among themselves.
//
// The x-th selection of a head takes candidate row sel.row[h, x] of the per-row buffers
// (`pitch` rows per head) and writes the list of source slot sel.pos[h, x] of this round
// (src [Hkv, S]); without those lists row x goes to slot x.
__global__ __launch_bounds__(256) void nbr_select_kernel(const uint2 *__restrict__ cand,
                                                         const int32_t *__restrict__ cand_cnt,
                                                         int32_t *__restrict__ overflow,
                                                         const int32_t *__restrict__ src, int S, int pitch,
                                                         int chunks, int slice_cap, int cap, int m,
                                                         SelectRows sel, int32_t *__restrict__ nbr,
                                                         float *__restrict__ nbr_e)
{
    extern __shared__ __align__(8) uint32_t dyn[];
    __shared__ uint32_t hist[256];   // 8-bit digits: the lists are short
    __shared__ uint32_t s_bin, s_need, s_min[4], s_max[4];
    __shared__ int32_t n_win;
    __shared__ int32_t end_s[256], wave_tot[4], s_pos;   // end_s[c]: entries in slices 0 .. c
    __shared__ uint32_t s_self;
    const int h = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int n_rows = sel.n_rows ? sel.n_rows[h] : S;
    if (overflow[h]) return;
    // Only the edge keys of a list stay in LDS (half the footprint, twice the workgroups per
    // compute unit); the key indices of the winners, and of entries tied at the cut, are fetched
    // from the slices again once those are known.
    uint32_t *ek = dyn;                 // [cap] order-preserving edge keys (0 = dropped)
    uint64_t *win = reinterpret_cast<uint64_t *>(dyn + cap + (cap & 1));   // [m + kTieRoom] winners
    const int win_cap = m + kTieRoom;

    // candidate row and output slot of a selection, then its slice sizes (thread c: chunk c) and
    // the source's own index: two rounds of independent loads, asked for one selection ahead
    auto ask = [&](int x, int32_t &cnt_r, int32_t &self_r, int32_t &pos_r, int32_t &crow_r) {
        const long at = (long)h * S + x;
        crow_r = sel.row ? sel.row[at] : x;
        pos_r = sel.pos ? sel.pos[at] : x;
        cnt_r = tid < chunks ? cand_cnt[((long)h * pitch + crow_r) * chunks + tid] : 0;
        self_r = src[(long)h * S + pos_r];
    };
    int32_t cnt_r = 0, self_r = 0, pos_r = 0, crow_r = 0;
    int search_steps = 0;   // bisection steps over the slices
    while ((1 << search_steps) < chunks) ++search_steps;
    if ((int)blockIdx.x < n_rows) ask(blockIdx.x, cnt_r, self_r, pos_r, crow_r);

    for (int x = blockIdx.x; x < n_rows; x += gridDim.x) {
        const long row = (long)h * pitch + crow_r;
        int incl = cnt_r;   // running total of the slice sizes
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_up(incl, o, kWave);
            if (lane >= o) incl += v;
        }
        if (lane == 63) wave_tot[wv] = incl;
        if (tid == 0) { s_self = (uint32_t)self_r; s_pos = pos_r; n_win = 0; }
        __syncthreads();
        for (int u = 0; u < wv; ++u) incl += wave_tot[u];
        end_s[tid] = incl;
        __syncthreads();
        if (x + (int)gridDim.x < n_rows) ask(x + gridDim.x, cnt_r, self_r, pos_r, crow_r);
        const int n = end_s[255];
        if (n > cap) {          // more candidates than the select can hold: the head is redone exactly
            if (tid == 0) overflow[h] = 1;
            return;
        }
        const uint32_t self = s_self;
        const long out_row = (long)h * S + s_pos;
        const uint2 *slices = cand + row * chunks * (long)slice_cap;
        // where entry r of the concatenated slices sits: the first slice that ends behind it
        auto locate = [&](int r) {
            int lo = 0, hi = chunks - 1;
            for (int s = 0; s < search_steps; ++s) {
                const int mid = (lo + hi) >> 1;
                if (end_s[mid] > r) hi = mid; else lo = mid + 1;
            }
            lo = min(lo, chunks - 1);
            return (long)lo * slice_cap + (r - (lo ? end_s[lo - 1] : 0));
        };
        uint32_t kmin = 0xffffffffu, kmax = 0u;
        // four entries per thread and turn, their loads in flight together (entries past the
        // end read the last one again and are left out below)
        for (int r0 = tid; r0 < n; r0 += 1024) {
            uint2 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = slices[locate(min(r0 + 256 * u, n - 1))];
#pragma unroll
            for (int u = 0; u < 4; ++u) asm volatile("" : "+v"(v[u].x), "+v"(v[u].y));
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int r = r0 + 256 * u;
                if (r < n) {
                    // the source's own column is no neighbour (Eq. 3: j != i): key 0 sorts below every edge
                    const uint32_t k = v[u].y == self ? 0u : ord_key_u(v[u].x);
                    ek[r] = k;
                    if (k) { kmin = min(kmin, k); kmax = max(kmax, k); }
                }
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, o, kWave));
            kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o, kWave));
        }
        if (lane == 0) { s_min[wv] = kmin; s_max[wv] = kmax; }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < 4; ++u) { kmin = min(kmin, s_min[u]); kmax = max(kmax, s_max[u]); }

        const uint32_t range = kmax - kmin;
        int remaining = (kmax >= kmin && range) ? 32 - __clz(range) : 0;
        uint32_t prefix = 0, mask = 0, need = (uint32_t)m;
        while (remaining > 0) {
            const int bits = remaining < 8 ? remaining : 8;
            const int shift = remaining - bits;
            const uint32_t dmask = (1u << bits) - 1u;
            hist[tid] = 0;
            __syncthreads();
            for (int r = tid; r < n; r += 256) {
                const uint32_t k = ek[r];
                if (k) {
                    const uint32_t rel = k - kmin;
                    if ((rel & mask) == prefix) atomicAdd(&hist[(rel >> shift) & dmask], 1u);
                }
            }
            __syncthreads();
            if (wv == 0) {   // bin where the count of larger-or-equal digits reaches `need`
                uint32_t tsum = 0;
                for (int b = 0; b < 4; ++b) tsum += hist[4 * lane + b];
                uint32_t incl = tsum;
#pragma unroll
                for (int o = 1; o < 64; o <<= 1) {
                    const uint32_t v = __shfl_down(incl, o, kWave);
                    if (lane + o < 64) incl += v;
                }
                const uint32_t excl = incl - tsum;
                if (excl < need && need <= incl) {
                    uint32_t cum = excl;
                    int b = 3;
                    for (; b > 0; --b) {
                        const uint32_t cb = hist[4 * lane + b];
                        if (cum + cb >= need) break;
                        cum += cb;
                    }
                    s_bin = 4 * lane + b;
                    s_need = need - cum;
                }
            }
            __syncthreads();
            prefix |= s_bin << shift;
            mask |= dmask << shift;
            need = s_need;
            remaining = shift;
        }
        const uint32_t tau = kmin + prefix;
        // Everything that reaches the threshold goes to the list as (entry number, edge bits);
        // its order is fixed by the final ranking.  More entries equal to the threshold than
        // the list has room for beyond m: the head is redone exactly.
        for (int r = tid; r < n; r += 256) {
            const uint32_t k = ek[r];
            if (k >= tau && k) {
                const int at = atomicAdd(&n_win, 1);
                if (at < win_cap) win[at] = ((uint64_t)(uint32_t)r << 32) | ord_key_inv(k);
            }
        }
        __syncthreads();
        const int listed = n_win;
        if (listed > win_cap || listed < m) {   // (fewer than m: the list was short of candidates)
            if (tid == 0) overflow[h] = 1;
            return;
        }
        // the key indices of the listed entries: (key index, edge bits) from here on
        for (int r = tid; r < listed; r += 256) {
            const uint64_t w = win[r];
            const uint32_t j = slices[locate((int)(w >> 32))].y;
            win[r] = ((uint64_t)j << 32) | (uint32_t)w;
        }
        __syncthreads();
        if (listed > m) {
            // Of the entries equal to the threshold only those with the lowest key indices stay:
            // one that `keep` or more tied entries precede is dropped (it then sorts behind all).
            const uint32_t tau_bits = ord_key_inv(tau);
            int n_tied = 0;
            for (int u = 0; u < listed; ++u) n_tied += (uint32_t)win[u] == tau_bits;
            const int keep = m - (listed - n_tied);
            uint32_t drop = 0u;   // bit i: entry tid + 256 i is dropped (written once all have compared)
            for (int r = tid, i = 0; r < listed; r += 256, ++i) {
                const uint64_t mine = win[r];
                if ((uint32_t)mine == tau_bits) {
                    int before = 0;
                    for (int u = 0; u < listed; ++u) {
                        const uint64_t w = win[u];
                        before += (uint32_t)w == tau_bits && w < mine;
                    }
                    if (before >= keep) drop |= 1u << i;
                }
            }
            __syncthreads();
            for (int r = tid, i = 0; r < listed; r += 256, ++i)
                if ((drop >> i) & 1u) win[r] = ~0ull;
            __syncthreads();
        }
        // each winner's rank by key index is its place in the output
        for (int r = tid; r < listed; r += 256) {
            const uint64_t mine = win[r];
            if (mine != ~0ull) {
                int pos = 0;
                for (int u = 0; u < listed; ++u) pos += win[u] < mine;
                nbr[out_row * m + pos] = (int32_t)(mine >> 32);
                nbr_e[out_row * m + pos] = __uint_as_float((uint32_t)mine);
            }
        }
        __syncthreads();   // the lists in LDS are free for the next row
    }
}

// The same select for short lists, one wave per source and no workgroup barrier: a lane
// keeps the keys of up to R candidates in registers, so that a compute unit works on
// several times as many sources at once as with a workgroup per source -- the select is
// a chain of memory and LDS round trips, and only the number of chains in flight hides
// them.  Everything that reaches the m-th largest key goes to a small LDS list per wave
// (m entries and room for 64 more that are tied at the cut); only then are the key
// indices of the listed entries fetched, the tied entries with the lowest key indices are
// kept, and the winners are ranked by key index.  Lists longer than 64 R, with fewer than
// m entries, or with more ties at the cut than the list has room for, raise the head's
// overflow flag (the head is then redone exactly).
template <int R>
__global__ __launch_bounds__(256) void nbr_select_wave_kernel(const uint2 *__restrict__ cand,
                                                              const int32_t *__restrict__ cand_cnt,
                                                              int32_t *__restrict__ overflow,
                                                              const int32_t *__restrict__ src, int S, int pitch,
                                                              int chunks, int slice_cap, int m,
                                                              int32_t *__restrict__ nbr,
                                                              float *__restrict__ nbr_e)
{
    static_assert(R == 16 || R == 32, "register groups of 16");
    extern __shared__ __align__(8) uint32_t dyn[];   // per wave: [64] slice starts, [m + kTieRoom] list (64 bit)
    const int h = blockIdx.y, tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);   // (scalar: so are the row and its addresses)
    const int n_rows = S;        // candidate row x of the head (pitch rows) -> source slot x
    if (overflow[h]) return;
    const int list_cap = m + kTieRoom;
    uint32_t *start_s = dyn + wv * (64 + 2 * list_cap);
    uint64_t *win = reinterpret_cast<uint64_t *>(start_s + 64);
    const uint64_t below = (1ull << lane) - 1ull;

    for (int x = blockIdx.x * 4 + wv; x < n_rows; x += gridDim.x * 4) {
        const long row = (long)h * pitch + x;
        const uint2 *slices = cand + row * chunks * (long)slice_cap;
        // slice sizes -> where each slice starts in the concatenated list
        const int cnt = lane < chunks ? cand_cnt[row * chunks + lane] : 0;
        const uint32_t self = (uint32_t)src[(long)h * S + x];
        const long out_row = (long)h * S + x;
        int incl = cnt;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_up(incl, o, kWave);
            if (lane >= o) incl += v;
        }
        // (values every lane holds alike are moved to scalar registers: the code below then
        // branches as a wave instead of masking lanes)
        const int n = __builtin_amdgcn_readfirstlane(__shfl(incl, 63, kWave));
        if (n > 64 * R || n < m) {   // too long for the lanes (or short of m): the head is redone exactly
            if (lane == 0) overflow[h] = 1;
            return;
        }
        start_s[lane] = (uint32_t)(incl - cnt);
        __builtin_amdgcn_wave_barrier();
        const int n_it = (n + 63) >> 6;

        // Register it of lane L holds entry 64 it + L: first where it sits in the row's slices,
        // then its order-preserving edge key (0 = no entry / dropped).  The slice starts are the
        // same for every lane: a scalar walk over the slices, the last slice that starts at or
        // before the entry wins.  The loads of 16 registers leave together.
        uint32_t E[R];
        // (the lane number as a value the compiler cannot see through: otherwise it keeps
        // "64 it + lane" for every register in a register of its own across the whole loop)
        int ln = lane;
        asm volatile("" : "+v"(ln));
#pragma unroll
        for (int it = 0; it < R; ++it) E[it] = (uint32_t)(ln + it * 64);
        for (int c = 1; c < chunks; ++c) {
            const int s_c = __builtin_amdgcn_readlane(incl - cnt, c);
            const int shift = c * slice_cap - s_c;
#pragma unroll
            for (int it = 0; it < R; ++it)
                if ((it & ~15) < n_it) E[it] = ln >= s_c - it * 64 ? (uint32_t)(ln + (it * 64 + shift)) : E[it];
        }
#pragma unroll
        for (int it = 0; it < R; ++it) E[it] = ln < n - it * 64 ? E[it] : 0u;   // past the end: any valid entry
        uint32_t kmin = 0xffffffffu, kmax = 0u;
        bool dropped = false;   // this lane held the source's own column
#pragma unroll
        for (int g = 0; g < R; g += 16) {
            if (g < n_it) {
                uint2 v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u)
                    v[u] = *reinterpret_cast<const uint2 *>(reinterpret_cast<const char *>(slices) + E[g + u] * 8u);
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    // the source's own column is no neighbour (Eq. 3: j != i): key 0 sorts below every edge
                    const bool present = ln < n - (g + u) * 64, own = present && v[u].y == self;
                    const uint32_t k = (present && !own) ? ord_key_u(v[u].x) : 0u;
                    dropped |= own;
                    E[g + u] = k;
                    if (k) { kmin = min(kmin, k); kmax = max(kmax, k); }
                }
            } else {
#pragma unroll
                for (int u = 0; u < 16; ++u) E[g + u] = 0u;
            }
        }
        const int valid = n - (int)__popcll(__ballot(dropped));
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, o, kWave));
            kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o, kWave));
        }
        kmin = (uint32_t)__builtin_amdgcn_readfirstlane((int)kmin);
        kmax = (uint32_t)__builtin_amdgcn_readfirstlane((int)kmax);
        if (valid < m) {
            if (lane == 0) overflow[h] = 1;
            return;
        }

        uint32_t tau;
        if (n_it <= 4) tau = mth_largest_key<4>(E, kmin, kmax, m);
        else if (n_it <= 8) tau = mth_largest_key<8>(E, kmin, kmax, m);
        else if (n_it <= 12) tau = mth_largest_key<12>(E, kmin, kmax, m);
        else if (n_it <= 16) tau = mth_largest_key<16>(E, kmin, kmax, m);
        else if (n_it <= 24) tau = mth_largest_key<(R > 24 ? 24 : R)>(E, kmin, kmax, m);
        else tau = mth_largest_key<R>(E, kmin, kmax, m);

        // everything that reaches tau -> LDS list as (entry number, key), any order
        int listed = 0;
#pragma unroll
        for (int it = 0; it < R; ++it)
            if ((it & ~3) < n_it) {
                const bool in = E[it] >= tau;
                const uint64_t votes = __ballot(in);
                const int at = listed + (int)__popcll(votes & below);
                if (in && at < list_cap) win[at] = ((uint64_t)(uint32_t)(ln + it * 64) << 32) | E[it];
                listed += (int)__popcll(votes);
            }
        if (listed > list_cap) {   // too many exactly equal edges at the cut
            if (lane == 0) overflow[h] = 1;
            return;
        }
        __builtin_amdgcn_wave_barrier();
        // the key indices of the listed entries: (key index, edge bits) from here on
        for (int r = lane; r < listed; r += 64) {
            const uint64_t w = win[r];
            const int e = (int)(w >> 32);
            int lo = 0, hi = chunks - 1;    // last slice that starts at or before entry e
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if ((int)start_s[mid] <= e) lo = mid; else hi = mid - 1;
            }
            const uint32_t j = slices[lo * slice_cap + (e - (int)start_s[lo])].y;
            win[r] = ((uint64_t)j << 32) | ord_key_inv((uint32_t)w);
        }
        __builtin_amdgcn_wave_barrier();
        if (listed > m) {
            // Of the entries equal to tau only those with the lowest key indices stay: one that
            // `keep` or more tied entries precede is dropped (a dropped entry sorts behind all).
            const uint32_t tau_bits = ord_key_inv(tau);
            int n_tied = 0;
            for (int u = 0; u < listed; ++u) n_tied += (uint32_t)win[u] == tau_bits;
            const int keep = m - (listed - n_tied);
            for (int r0 = 0; r0 < listed; r0 += 64) {
                const int r = r0 + lane;
                const uint64_t mine = r < listed ? win[r] : 0ull;
                int before = 0;
                if (r < listed && (uint32_t)mine == tau_bits)
                    for (int u = 0; u < listed; ++u) {
                        const uint64_t w = win[u];
                        before += (uint32_t)w == tau_bits && w < mine;
                    }
                __builtin_amdgcn_wave_barrier();
                if (before >= keep) win[r] = ~0ull;
            }
            __builtin_amdgcn_wave_barrier();
        }
        // each winner's rank by key index is its place in the output
        for (int r = lane; r < listed; r += 64) {
            const uint64_t mine = win[r];
            if (mine != ~0ull) {
                int pos = 0;
                for (int u = 0; u < listed; ++u) pos += win[u] < mine;
                nbr[out_row * m + pos] = (int32_t)(mine >> 32);
                nbr_e[out_row * m + pos] = __uint_as_float((uint32_t)mine);
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// Where each source of this round (cur [Hkv, S], ascending) gets its neighbour list from:
//   - it was a source in the previous round (prev, ascending): its list (prev_nbr, prev_e
//     [Hkv, S, m]) is copied to its slot of this round (nbr, nbr_e);
//   - it is one of the head's speculative rows (entries S .. S + X of ext [Hkv, S + X],
//     ascending, whose candidate lists the first round's filter pass built in rows
//     spec_row0 .. of the per-row buffers) and
//     those lists are complete (the head raised no overflow flag in the first round): the
//     exact select runs on that row;
//   - otherwise it goes, in order, to new_src[h, 0 .. n_new[h]) for another bound and filter
//     pass, which uses rows 0 .. of the per-row buffers (the candidates of the first round's
//     sources are no longer needed once their lists are selected).
// The selections to run are listed as (candidate row, source slot) in sel_row / sel_pos
// [Hkv, S], n_sel[h] of them.  spec_bad [Hkv] remembers across rounds whether a head's
// speculative lists may be used: the first match of a call sets it from the overflow flags
// of the first round (first != 0), later ones read it.  One workgroup per head.
__global__ __launch_bounds__(256) void match_sources_kernel(
    const int32_t *__restrict__ prev, const int32_t *__restrict__ cur, int S, int m,
    const int32_t *__restrict__ prev_nbr, const float *__restrict__ prev_e, int32_t *__restrict__ nbr,
    float *__restrict__ nbr_e, const int32_t *__restrict__ ext, int X, int spec_row0,
    int32_t *__restrict__ spec_bad, const int32_t *__restrict__ overflow, int first,
    int32_t *__restrict__ new_src, int32_t *__restrict__ n_new, int32_t *__restrict__ sel_row,
    int32_t *__restrict__ sel_pos, int32_t *__restrict__ n_sel)
{
    extern __shared__ int32_t prev_s[];   // [S] previous sources, [S] where this round's lists come from, [X] spec
    int32_t *code_s = prev_s + S, *spec_s = code_s + S;
    __shared__ int32_t wave_new[4], wave_fb[4];
    const int h = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const long row0 = (long)h * S;
    for (int b = tid; b < S; b += 256) prev_s[b] = prev[row0 + b];
    for (int b = tid; b < X; b += 256) spec_s[b] = ext[(long)h * (S + X) + S + b];   // the rows behind the S sources
    bool bad = X == 0;
    if (X > 0) {
        bad = first ? overflow[h] != 0 : spec_bad[h] != 0;
        if (first && tid == 0) spec_bad[h] = bad ? 1 : 0;
    }
    __syncthreads();
    // first slot of a sorted list that holds i or more
    auto lower_bound = [](const int32_t *list, int n, int32_t i) {
        int lo = 0, hi = n;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (list[mid] < i) lo = mid + 1; else hi = mid;
        }
        return lo;
    };
    int base = 0, base_fb = 0;
    for (int a0 = 0; a0 < S; a0 += 256) {
        const int a = a0 + tid;
        int i = 0, found = -1, spec_at = -1;
        if (a < S) {
            i = cur[row0 + a];
            const int lo = lower_bound(prev_s, S, i);
            if (lo < S && prev_s[lo] == i) found = lo;
            if (found < 0 && !bad) {
                const int u = lower_bound(spec_s, X, i);
                if (u < X && spec_s[u] == i) spec_at = u;
            }
        }
        const bool is_new = a < S && found < 0, is_fb = is_new && spec_at < 0;
        const uint64_t mask = __ballot(is_new), mask_fb = __ballot(is_fb);
        if (lane == 0) { wave_new[wv] = (int32_t)__popcll(mask); wave_fb[wv] = (int32_t)__popcll(mask_fb); }
        __syncthreads();
        int before = base, total = 0, before_fb = base_fb, total_fb = 0;
        for (int u = 0; u < 4; ++u) {
            if (u < wv) { before += wave_new[u]; before_fb += wave_fb[u]; }
            total += wave_new[u];
            total_fb += wave_fb[u];
        }
        if (a < S) code_s[a] = found;
        if (is_new) {
            const uint64_t lower = (1ull << lane) - 1ull;
            const int x = before + (int)__popcll(mask & lower);
            int crow = spec_row0 + spec_at;
            if (is_fb) {
                const int r = before_fb + (int)__popcll(mask_fb & lower);
                new_src[row0 + r] = i;
                crow = r;
            }
            sel_row[row0 + x] = crow;
            sel_pos[row0 + x] = a;
        }
        base += total;
        base_fb += total_fb;
        __syncthreads();
    }
    if (tid == 0) {
        n_new[h] = base_fb;
        n_sel[h] = base;
    }
    // the lists that stay: the neighbourhood of a source does not depend on the scores
    for (long u = tid; u < (long)S * m; u += 256) {
        const int a = (int)(u / m), r = (int)(u % m);
        const int from = code_s[a];
        if (from >= 0) {
            nbr[(row0 + a) * m + r] = prev_nbr[(row0 + from) * m + r];
            nbr_e[(row0 + a) * m + r] = prev_e[(row0 + from) * m + r];
        }
    }
}

// Columns per workgroup: about 1024 workgroups in flight over all heads and source
// groups, at least 8 key blocks per wave, and at least `min_chunks` chunks per head.
int chunk_cols_for(int Hkv, int sgroups, int n_cols, int min_chunks = 1)
{
    long ck = ((long)Hkv * sgroups * n_cols + 1023) / 1024;
    if (ck < 1024) ck = 1024;
    const long cap = (n_cols + min_chunks - 1) / min_chunks;
    if (ck > cap) ck = cap;
    ck = ((ck + 127) / 128) * 128;
    return (int)(ck < 128 ? 128 : ck);
}

}  // namespace

// Keys in the strided sample of the bound pass: every 8th key, between 2048 and 8192 keys (one
// workgroup walks the whole sample of a head's sources).  A denser sample costs the bound pass
// more and gives a tighter bound, i.e. fewer candidates for the filter pass to park and list
// (measured at 131008 keys and m = 128: 8192 sampled keys 10.2 ms per 32-layer pass, 16384 keys
// 10.4 ms, 4096 keys 10.3 ms).
int mfma_sample_cols(int P)
{
    int ps = ((P / 8 + 127) / 128) * 128;
    if (ps < 2048) ps = 2048;
    if (ps > 8192) ps = 8192;
    return ps;
}

// Rank of the sampled edge that the bound is taken at.  The bound is useful for a source when at
// least m of its edges lie above it, i.e. when fewer than `rank` of its m - 1 largest edges fell
// into the sample.  With every stride-th key sampled that count is binomial, (m - 1) trials at
// 1 / stride: the rank is its mean plus six standard deviations (and one), at most m, so that
// about one source in 10^7 comes out short -- which the select notices (fewer than m candidates)
// and answers by redoing the head exactly, like an overflow.  About rank * stride keys lie above
// the bound instead of m * stride: fewer rows to park, list and select from.
int mfma_bound_rank(int m, int stride)
{
    if (stride <= 1) return m;
    const double mean = (m - 1.0) / stride, dev = sqrt(mean * (1.0 - 1.0 / stride));
    const int rank = (int)ceil(mean + 6.0 * dev) + 1;
    return rank < m ? rank : m;
}

int mfma_cand_cap(int P, int m)
{
    // four times the rank * stride keys expected above the bound (the bin that the bound is
    // rounded down to adds up to a few hundred more at long prompts)
    const int stride = P / mfma_sample_cols(P);
    long cap = 4L * mfma_bound_rank(m, stride) * stride;
    if (cap < 1024) cap = 1024;
    return (int)cap;
}

bool mfma_filter_applies(int P, int m)
{
    // The sample must hold far more than m keys for its m-th largest edge to be a
    // useful bound, the key index must fit the 24 bits of a staged candidate, and
    // the select kernel's LDS must hold a full list.
    if (P < 8192 || P >= (1 << 24)) return false;
    if (m > mfma_sample_cols(P) / 8) return false;
    return (size_t)mfma_cand_cap(P, m) * 8 + (size_t)m * 8 + 8 <= 140 * 1024;
}

bool source_reuse_applies(int S) { return S <= 4096; }   // the previous list and the match's bookkeeping sit in LDS

// Geometry of the filter route for a call.  X speculative rows (see the head of this file)
// ride along in the first round when the lists are kept from round to round and the extended
// source list still fits the small-k source selection; their workgroups then carry three
// 32-row groups.  Key chunks per head and the capacity of one (row, chunk) slice: four times
// the expected share of a chunk, at least 2 m (and 64) entries.
MfmaFilterPlan mfma_filter_plan(int Hkv, int P, int S, int m, bool keep_lists, bool speculate)
{
    MfmaFilterPlan g{};
    g.S = S;
    // speculative rows: at least one 32-row block; the extended list fills whole 96-row workgroups
    // where that takes at most two blocks
    g.X = 0;
    if (keep_lists && speculate && S + kSpecRows <= kMaxExtSources) {
        int x = (S + kSpecRows + 95) / 96 * 96 - S;
        if (x > 2 * kSpecRows) x = 2 * kSpecRows;
        if (S + x > kMaxExtSources) x = (kMaxExtSources - S) / 8 * 8;
        g.X = x;
    }
    g.sb = g.X > 0 ? 3 : 2;
    g.pitch = S + g.X;
    const int rows_wg = kBlk * g.sb;
    const int sgroups = (S + g.X + rows_wg - 1) / rows_wg;
    g.chunk_cols = chunk_cols_for(Hkv, sgroups, P);
    g.chunks = (P + g.chunk_cols - 1) / g.chunk_cols;
    if (g.chunks > 256) {   // the exact select keeps the slice sizes of a source in LDS
        g.chunk_cols = (((P + 255) / 256 + 127) / 128) * 128;
        g.chunks = (P + g.chunk_cols - 1) / g.chunk_cols;
    }
    // a slice holds four times its expected share of a row's ~rank * stride candidates (rank: the
    // bound pass's rank in the sample), and 2 m on top
    const int stride = P / mfma_sample_cols(P);
    const long share = ((long)mfma_bound_rank(m, stride) * stride + g.chunks - 1) / g.chunks;
    long sc = 4L * share + 2L * m;
    if (sc < 64) sc = 64;
    g.cand_cap = mfma_cand_cap(P, m);
    if (sc > g.cand_cap) sc = g.cand_cap;
    g.slice_cap = (int)sc;
    return g;
}

hipError_t launch_mfma_cosine(const void *Ac, const void *Kc, int Hkv, int N, int P, int S, const int32_t *src,
                              float *E, const int32_t *gate, hipStream_t st)
{
    const int sgroups = (S + kRows - 1) / kRows;
    const int ck = chunk_cols_for(Hkv, sgroups, P);
    const int chunks = (P + ck - 1) / ck;
    FilterArgs fa{};
    if (!allow_big_lds((const void *)cosine_dense_kernel)) return hipGetLastError();
    hipLaunchKernelGGL(cosine_dense_kernel, dim3(chunks, Hkv, sgroups), dim3(kThreads), 2 * kTileBytes,
                       st, (const uint16_t *)Ac, (const uint16_t *)Kc, N, P, 1, S, src, ck, E, fa, gate);
    return hipGetLastError();
}

namespace {

// Chunks of the sample per (head, source group): 1 when the heads alone give 128 workgroups or
// more, else enough for about 256 workgroups, at least two key tiles each.
int bound_chunks(int Hkv, int P, int sgroups)
{
    const int ps = mfma_sample_cols(P);
    if (Hkv * sgroups >= 128) return 1;
    int chunks = 256 / (Hkv * sgroups);
    if (chunks > ps / (2 * kTileKeys)) chunks = ps / (2 * kTileKeys);
    return chunks < 1 ? 1 : chunks;
}

template <int SB, int BINS>
hipError_t launch_bound(const void *Ac, const void *Kc, int Hkv, int N, int P, int rows, int m, const int32_t *src,
                        int src_pitch, const int32_t *n_src, void *hist_part, float *tau, int pitch, int row0,
                        int32_t *overflow, hipStream_t st)
{
    constexpr int ROWS = SB * kBlk;
    const int ps = mfma_sample_cols(P), stride = P / ps;
    const int sgroups = (rows + ROWS - 1) / ROWS;
    const int chunks = bound_chunks(Hkv, P, sgroups);
    const int chunk_cols = (((ps + chunks - 1) / chunks + kTileKeys - 1) / kTileKeys) * kTileKeys;
    const int rank = mfma_bound_rank(m, stride);
    if (!allow_big_lds((const void *)cosine_bound_kernel<SB, BINS>)) return hipGetLastError();
    hipLaunchKernelGGL((cosine_bound_kernel<SB, BINS>), dim3(sgroups, Hkv, chunks), dim3(256 * SB),
                       2 * kTileBytes + ROWS * BINS * 4, st, (const uint16_t *)Ac, (const uint16_t *)Kc, N, ps,
                       stride, rows, src_pitch, src, n_src, rank, chunk_cols, (uint32_t *)hist_part, tau, pitch, row0,
                       overflow);
    if (chunks > 1)
        hipLaunchKernelGGL((bound_merge_kernel<SB, BINS>), dim3((rows + 3) / 4, Hkv), dim3(256), 0, st,
                           (const uint32_t *)hist_part, chunks, sgroups, rows, n_src, rank, tau, pitch, row0);
    return hipGetLastError();
}

template <int SB, int RING>
hipError_t launch_filter(const void *Ac, const void *Kc, int Hkv, int N, int P, int rows, int m, const int32_t *src,
                         int src_pitch, const int32_t *n_src, const MfmaFilterPlan &g, int row0, const float *tau,
                         void *cand, int32_t *cand_cnt, int32_t *overflow, hipStream_t st)
{
    constexpr int ROWS = SB * kBlk;
    const int sgroups = (rows + ROWS - 1) / ROWS;
    const int stride = P / mfma_sample_cols(P);
    // Rows a half-wave parks per tile: 32 lanes x P(a lane's 16 edges hold a hit), with a
    // per-edge hit rate of about rank * stride / P (each source keeps about that many candidates,
    // rank = the bound pass's rank in the sample).  Drains are scheduled for when most of a
    // half-wave's 32 lanes get a row and the ring is not yet full.
    const double rate = (double)mfma_bound_rank(m, stride) * stride / (double)P;
    const double per_tile = 32.0 * (1.0 - pow(1.0 - (rate < 1.0 ? rate : 1.0), 16.0));
    int drain_every = (int)((RING > kBlk ? 30.0 : 24.0) / (per_tile > 0.45 ? per_tile : 0.45));
    if (drain_every < 1) drain_every = 1;
    FilterArgs fa{n_src, tau, (uint2 *)cand, cand_cnt, overflow, g.slice_cap, drain_every, sgroups, src_pitch,
                  g.pitch, row0};
    if (!allow_big_lds((const void *)cosine_filter_kernel<SB, RING>)) return hipGetLastError();
    hipLaunchKernelGGL((cosine_filter_kernel<SB, RING>), dim3(g.chunks * sgroups, Hkv), dim3(256 * SB),
                       2 * kTileBytes + 2 * (4 * SB) * RING * kStagePitch, st, (const uint16_t *)Ac,
                       (const uint16_t *)Kc, N, P, rows, src, g.chunk_cols, fa);
    return hipGetLastError();
}

}  // namespace

size_t mfma_bound_scratch_bytes(int Hkv, int P, const MfmaFilterPlan &g)
{
    // (the first round's launch has the most rows per workgroup and the fewest groups)
    size_t need = 0;
    for (int pass = 0; pass < 2; ++pass) {
        const int sb = pass == 0 ? g.sb : 2, rows = pass == 0 ? g.S + g.X : g.S;
        const int rows_wg = kBlk * sb, sgroups = (rows + rows_wg - 1) / rows_wg;
        const int chunks = bound_chunks(Hkv, P, sgroups);
        const size_t bytes = chunks > 1 ? (size_t)Hkv * sgroups * chunks * rows_wg * 256 * 4 : 0;
        if (bytes > need) need = bytes;
    }
    return need;
}

hipError_t launch_mfma_cosine_bound(const void *Ac, const void *Kc, int Hkv, int N, int P, int m,
                                    const MfmaFilterPlan &g, bool first_round, const int32_t *src,
                                    const int32_t *n_src, void *hist_part, float *tau, int32_t *overflow,
                                    hipStream_t st)
{
    if (first_round && g.sb == 3)
        return launch_bound<3, 224>(Ac, Kc, Hkv, N, P, g.S + g.X, m, src, g.S + g.X, n_src, hist_part, tau, g.pitch,
                                    0, overflow, st);
    if (first_round)
        return launch_bound<2, 256>(Ac, Kc, Hkv, N, P, g.S, m, src, g.S, n_src, hist_part, tau, g.pitch, 0,
                                    overflow, st);
    return launch_bound<2, 256>(Ac, Kc, Hkv, N, P, g.S, m, src, g.S, n_src, hist_part, tau, g.pitch, 0, overflow, st);
}

hipError_t launch_mfma_cosine_filter(const void *Ac, const void *Kc, int Hkv, int N, int P, int m,
                                     const MfmaFilterPlan &g, bool first_round, const int32_t *src,
                                     const int32_t *n_src, const float *tau, void *cand, int32_t *cand_cnt,
                                     int32_t *overflow, hipStream_t st)
{
    if (first_round && g.sb == 3)
        return launch_filter<3, 32>(Ac, Kc, Hkv, N, P, g.S + g.X, m, src, g.S + g.X, n_src, g, 0, tau, cand, cand_cnt,
                                    overflow, st);
    if (first_round)
        return launch_filter<2, 64>(Ac, Kc, Hkv, N, P, g.S, m, src, g.S, n_src, g, 0, tau, cand, cand_cnt, overflow, st);
    return launch_filter<2, 64>(Ac, Kc, Hkv, N, P, g.S, m, src, g.S, n_src, g, 0, tau, cand, cand_cnt, overflow, st);
}

hipError_t launch_match_sources(const int32_t *prev, const int32_t *cur, int Hkv, int m, const MfmaFilterPlan &g,
                                const int32_t *prev_nbr, const float *prev_e, int32_t *nbr, float *nbr_e,
                                const int32_t *ext, int32_t *spec_bad, const int32_t *overflow, bool first_match,
                                int32_t *new_src, int32_t *n_new, int32_t *sel_row, int32_t *sel_pos,
                                int32_t *n_sel, hipStream_t st)
{
    hipLaunchKernelGGL(match_sources_kernel, dim3(Hkv), dim3(256), (size_t)(2 * g.S + g.X) * 4, st, prev, cur, g.S,
                       m, prev_nbr, prev_e, nbr, nbr_e, ext, g.X, g.S, spec_bad, overflow, first_match ? 1 : 0, new_src,
                       n_new, sel_row, sel_pos, n_sel);
    return hipGetLastError();
}

hipError_t launch_nbr_select(const void *cand, const int32_t *cand_cnt, int32_t *overflow, const int32_t *src,
                             int Hkv, int m, const MfmaFilterPlan &g, const SelectRows *rows, int32_t *nbr,
                             float *nbr_e, hipStream_t st)
{
    const int S = g.S, cap = g.cand_cap;
    // Every source has a list (first round, or nothing kept) and the lists are short: a wave
    // per source.  That kernel is long straight-line code, which only pays when there are
    // many lists to go through; the few selections of a later round take the other one.
    if (!rows && cap <= 64 * 32 && g.chunks <= 64) {
        int per_head = 8192 / Hkv < 1 ? 1 : 8192 / Hkv;   // four sources per workgroup
        const int wgs = per_head > (S + 3) / 4 ? (S + 3) / 4 : per_head;
        const size_t lds = (size_t)4 * (64 + 2 * (m + kTieRoom)) * 4;
        auto *kernel = cap <= 64 * 16 ? nbr_select_wave_kernel<16> : nbr_select_wave_kernel<32>;
        hipLaunchKernelGGL(kernel, dim3(wgs, Hkv), dim3(256), lds, st, (const uint2 *)cand, cand_cnt, overflow,
                           src, S, g.pitch, g.chunks, g.slice_cap, m, nbr, nbr_e);
        return hipGetLastError();
    }
    // The workgroups of a head share its selections in turn: few workgroups when only some
    // sources of a round need a select (most would find nothing to do), many otherwise.
    const SelectRows sel = rows ? *rows : SelectRows{};
    int per_head = (rows ? 3072 : 16384) / Hkv;
    per_head = per_head < 1 ? 1 : (per_head > S ? S : per_head);
    const size_t lds = (size_t)(cap + (cap & 1)) * 4 + (size_t)(m + kTieRoom) * 8;
    if (!allow_big_lds((const void *)nbr_select_kernel)) return hipGetLastError();
    hipLaunchKernelGGL(nbr_select_kernel, dim3(per_head, Hkv), dim3(256), lds, st, (const uint2 *)cand,
                       cand_cnt, overflow, src, S, g.pitch, g.chunks, g.slice_cap, cap, m, sel, nbr, nbr_e);
    return hipGetLastError();
}

}  // namespace gkv
