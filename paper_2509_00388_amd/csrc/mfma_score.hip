// Stage I on the matrix cores (bf16 inputs, d = 128, fp32 accumulation).
//
// Per KV head the window queries of its G query heads are stacked into one
// R x 128 operand (R = G*w rows), held in registers for the whole kernel.
// Keys stream from HBM in tiles of 128 rows through LDS (mfma_tile.hpp); each of
// the 4 key streams of a workgroup multiplies 32 of those rows, so one key block
// costs R/32 x 8 v_mfma_f32_32x32x16_bf16 and every key is read from HBM exactly
// once per pass.  256 query rows (long windows) take tiles of 64 keys instead: two key
// streams and four row groups of 64 rows in the same 8 waves, so that those keys are
// streamed once too.
//
// The column sums of a row softmax need the row statistics first, so there are
// two passes over the keys:
//   pass A  per-row running max and sum of exp over the visible keys (online,
//           kept per lane; queries are the MFMA's column dimension so that one
//           lane owns one query and no cross-lane traffic is needed);
//   pass B  logits recomputed; exp2(l*c - (max + log2 sum)) summed down the
//           query rows (queries are the MFMA's row dimension here, so the sum
//           is in-lane) and written as the vote of the key.
// Everything is done in the base-2 domain: c = scale * log2(e).
#include "common.hpp"
#include "kernels.hpp"
#include "mfma_tile.hpp"


namespace gkv {

namespace {

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// (m1, z1) <- softmax-statistics merge with (m2, z2), base 2.
__device__ __forceinline__ void merge_stats(float &m1, float &z1, float m2, float z2)
{
    const float mn = fmaxf(m1, m2);
    if (mn == -INFINITY) { m1 = mn; z1 = 0.f; return; }
    z1 = z1 * fast_exp2(m1 - mn) + z2 * fast_exp2(m2 - mn);
    m1 = mn;
}

template <int NB>
__device__ __forceinline__ void load_queries(const uint16_t *Qb, int l32, int hh, bf16x8 (&q)[NB][kSteps])
{
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int s = 0; s < kSteps; ++s)
            q[b][s] = load8(Qb + (long)(kBlk * b + l32) * kD + 16 * s + 8 * hh);
}

// The R query rows are split over SPLIT waves per key stream: a workgroup has 4
// key streams (wave & 3) and SPLIT row groups (wave >> 2), i.e. 4*SPLIT waves.  The
// waves of one stream load the same key block (the second load hits L1) and each
// handles NB/SPLIT of the 32-row query blocks.  With SPLIT = 2 a wave needs under
// 256 registers, two waves share a SIMD, and one wave's exp2 work overlaps the
// other's MFMAs.

// Which (head, chunk, part) a workgroup takes.  The parts of a key chunk stream the same keys
// and should run at about the same time on the same XCD, so that all but the first find the
// keys in that XCD's L2.  Workgroups go to the 8 XCDs round robin in the order of their linear
// number, so the parts of one (head, chunk) unit sit 8 apart: 8 units x their parts take
// 8 x nparts consecutive numbers.  (Unit counts that are no multiple of 8 keep the plain order,
// parts next to each other.)
__device__ __forceinline__ void unit_of_workgroup(int nparts, int &h, int &chunk, int &part)
{
    const int nchunks = gridDim.x / nparts;
    h = blockIdx.y;
    chunk = blockIdx.x / nparts;
    part = blockIdx.x % nparts;
    if (nparts > 1 && ((long)gridDim.y * nchunks) % 8 == 0) {
        const long lin = (long)blockIdx.y * gridDim.x + blockIdx.x;
        const long grp8 = lin / (8 * nparts);
        const int r = (int)(lin % (8 * nparts));
        const long unit = grp8 * 8 + (r & 7);
        h = (int)(unit / nchunks);
        chunk = (int)(unit % nchunks);
        part = r >> 3;
    }
}

// ---------------------------------------------------------------- pass A ---
template <int NB, int SPLIT, int STREAMS = 4>
__global__ __launch_bounds__(64 * STREAMS * SPLIT) void score_stats_kernel(
    const uint16_t *__restrict__ Kc, const uint16_t *__restrict__ Qw, int N, int P, int w,
    int chunk_keys, float c, float *__restrict__ part, int R_total, int row_base, int nparts)
{
    constexpr int R = NB * kBlk, NBW = NB / SPLIT, NT = 64 * STREAMS * SPLIT, TK = kBlk * STREAMS;
    extern __shared__ __align__(16) unsigned char kt[];   // two key tiles
    __shared__ float sm[STREAMS][R], sz[STREAMS][R];
    // nparts > 1: equal parts of 128 rows share one launch
    int h, chunk, row_part;
    unit_of_workgroup(nparts, h, chunk, row_part);
    const int nchunks = gridDim.x / nparts;
    row_base += 128 * row_part;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, hh = lane >> 5;
    const int stream = wv % STREAMS, row0 = (wv / STREAMS) * NBW * kBlk;   // first query row of this wave

    bf16x8 q[NBW][kSteps];
    load_queries<NBW>(Qw + ((long)h * R_total + row_base + row0) * kD, l32, hh, q);
    int last_vis[NBW];   // last key the lane's query of block b may see (causal window)
    float m[NBW], z[NBW];
#pragma unroll
    for (int b = 0; b < NBW; ++b) {
        last_vis[b] = P + (row_base + row0 + kBlk * b + l32) % w;
        m[b] = -INFINITY;
        z[b] = 0.f;
    }

    const uint16_t *Kh = Kc + (long)h * N * kD;
    const int k0 = chunk * chunk_keys, k1 = min(N, k0 + chunk_keys);
    const int ntile = (k1 - k0 + TK - 1) / TK;

    // Two accumulator sets: the products of tile t are issued between the softmax instructions of
    // tile t - 1, so that the matrix core works while the vector unit does the exponentials.
    f32x16 acc[2][NBW];
    // the kSteps * NBW matrix instructions of one tile; between(j) is placed after the j-th
    auto multiply = [&](const bf16x8 (&kc)[kSteps], int set, auto &&between) {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < kSteps; ++s)
#pragma unroll
            for (int b = 0; b < NBW; ++b) {   // rows = keys, columns = queries
                acc[set][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kc[s], q[b][s], s == 0 ? zero : acc[set][b], 0, 0, 0);
                between(s * NBW + b);
            }
    };
    // running (max, sum) of the lane's queries updated with tile t, whose products are in `set`
    auto finish = [&](int t, int set) {
        const int kb = k0 + TK * t + kBlk * stream;
        if (kb + kBlk <= P) {   // every key of the block is a prefix key: visible to all rows
#pragma unroll
            for (int b = 0; b < NBW; ++b) {
                float tm = acc[set][b][0];
#pragma unroll
                for (int i = 1; i < 16; ++i) tm = fmaxf(tm, acc[set][b][i]);
                const float mn = fmaxf(m[b], tm * c);
                float zz = z[b] * fast_exp2(m[b] - mn);
#pragma unroll
                for (int i = 0; i < 16; ++i) zz += fast_exp2(fmaf(acc[set][b][i], c, -mn));
                m[b] = mn;
                z[b] = zz;
            }
        } else {                // the block touches the window (or the end of the head): mask
#pragma unroll
            for (int b = 0; b < NBW; ++b) {
                float tm = -INFINITY;
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (kb + acc_row(i, hh) <= last_vis[b]) tm = fmaxf(tm, acc[set][b][i]);
                const float mn = fmaxf(m[b], tm * c);
                if (mn != -INFINITY) {
                    float zz = z[b] * fast_exp2(m[b] - mn);
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        if (kb + acc_row(i, hh) <= last_vis[b]) zz += fast_exp2(fmaf(acc[set][b][i], c, -mn));
                    m[b] = mn;
                    z[b] = zz;
                }
            }
        }
    };
    auto head = [&](const unsigned char *buf) {
        bf16x8 kc[kSteps];
        tile_read(buf, stream, l32, hh, kc);
        multiply(kc, 0, [](int) {});
    };
    auto body = [&](const unsigned char *buf, int t, int set) {
        bf16x8 kc[kSteps];
        tile_read(buf, stream, l32, hh, kc);
        const int kb = k0 + TK * (t - 1) + kBlk * stream;   // the block finished here
        if (kb + kBlk <= P) {
            // the same arithmetic as finish(), in the same order, cut into slices: the row maxima
            // while the LDS reads are on their way, then two exponentials after every matrix
            // instruction (the scheduling barriers keep the compiler from regrouping them)
#pragma unroll
            for (int b = 0; b < NBW; ++b) {
                float tm = acc[set ^ 1][b][0];
#pragma unroll
                for (int i = 1; i < 16; ++i) tm = fmaxf(tm, acc[set ^ 1][b][i]);
                const float mn = fmaxf(m[b], tm * c);
                z[b] = z[b] * fast_exp2(m[b] - mn);
                m[b] = mn;
            }
            __builtin_amdgcn_sched_barrier(0);
            multiply(kc, set, [&](int j) {
                constexpr int per = 16 / kSteps;   // NBW * 16 values over NBW * kSteps instructions
#pragma unroll
                for (int e = per * j; e < per * j + per; ++e)
                    z[e / 16] += fast_exp2(fmaf(acc[set ^ 1][e / 16][e % 16], c, -m[e / 16]));
                __builtin_amdgcn_sched_barrier(0);
            });
        } else {
            multiply(kc, set, [](int) {});
            finish(t - 1, set ^ 1);
        }
    };
    if constexpr (NBW <= 2) {
        GKV_TILE_PIPELINE_OVERLAPPED(TK, NT, Kh, k0, k1 - 1, 1, ntile, head, body, finish);
    } else {   // three row blocks per wave: a second accumulator set does not fit the registers
        auto one_tile = [&](const unsigned char *buf, int t) {
            bf16x8 kc[kSteps];
            tile_read(buf, stream, l32, hh, kc);
            multiply(kc, 0, [](int) {});
            finish(t, 0);
        };
        GKV_TILE_PIPELINE_TK(TK, NT, Kh, k0, k1 - 1, 1, ntile, one_tile, (void)0);
    }

    // merge the two half-waves (same query, other key rows), then the key streams
#pragma unroll
    for (int b = 0; b < NBW; ++b) {
        const float m2 = __shfl_xor(m[b], 32, kWave), z2 = __shfl_xor(z[b], 32, kWave);
        merge_stats(m[b], z[b], m2, z2);
        if (hh == 0) { sm[stream][row0 + kBlk * b + l32] = m[b]; sz[stream][row0 + kBlk * b + l32] = z[b]; }
    }
    __syncthreads();
    if (tid < R) {
        float mm = sm[0][tid], zz = sz[0][tid];
#pragma unroll
        for (int u = 1; u < STREAMS; ++u) merge_stats(mm, zz, sm[u][tid], sz[u][tid]);
        float *o = part + (((long)h * nchunks + chunk) * R_total + row_base + tid) * 2;
        o[0] = mm;
        o[1] = zz;
    }
}

// ---------------------------------------------------------------- pass B ---
// votes: PERQ = false: [Hkv * vote_rows, P], row h*vote_rows + vote_row_base + g holds
// the sum over the query rows of row group g; PERQ = true: [Hkv * G, P], one row per
// query head (needs every query head's rows inside one row group).
//
// Heads with more than 128 stacked query rows are handled in parts of at most 128
// rows (row_base .. row_base + R of R_total), one launch per part: the keys are then
// streamed once per part.
//
// pool_half >= 0 (average pooling, all rows of a head in one workgroup): the votes never leave the workgroup.  Each row
// group keeps the votes of the workgroup's keys in LDS, the workgroup also multiplies the
// pool_half keys on either side of its chunk, and at the end it writes the pooled, grouped
// scores of its chunk itself: votes[] is then the score array [Hkv, P].  The sums are
// formed in the order of the separate pooling kernel, so the bits are the same.
template <int NB, int SPLIT, bool PERQ, int STREAMS = 4>
__global__ __launch_bounds__(64 * STREAMS * SPLIT) void score_votes_kernel(
    const uint16_t *__restrict__ Kc, const uint16_t *__restrict__ Qw, int N, int P, int w, int G,
    int chunk_keys, float c, const float *__restrict__ part, int part_chunks,
    float *__restrict__ votes, int R_total, int row_base, int vote_rows, int vote_row_base, int nparts,
    int pool_half)
{
    constexpr int R = NB * kBlk, NBW = NB / SPLIT, NT = 64 * STREAMS * SPLIT, TK = kBlk * STREAMS;
    extern __shared__ __align__(16) unsigned char kt[];   // two key tiles
    __shared__ float bias_s[R];
    int h, chunk, row_part;
    unit_of_workgroup(nparts, h, chunk, row_part);
    row_base += 128 * row_part;
    vote_row_base += SPLIT * row_part;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, hh = lane >> 5;
    const int stream = wv % STREAMS, grp = wv / STREAMS, row0 = grp * NBW * kBlk;

    const int k0 = chunk * chunk_keys, k1 = min(P, k0 + chunk_keys);
    if (k0 >= P) return;
    const bool fused = !PERQ && pool_half >= 0;
    const int first = fused ? max(0, k0 - pool_half) : k0;      // keys this workgroup multiplies
    const int kend = fused ? min(P, k1 + pool_half) : k1;
    const int span = chunk_keys + 2 * pool_half;
    float *vs = reinterpret_cast<float *>(kt + 2 * TK * kPitch);   // [SPLIT][span], slot 0 = key k0 - pool_half
    if (fused)
        for (int u = tid; u < SPLIT * span; u += NT) vs[u] = 0.f;   // zero padding outside the row

    if (tid < R) {   // row statistics of the whole head: merge the chunks of pass A
        float mm = -INFINITY, zz = 0.f;
        for (int ch = 0; ch < part_chunks; ++ch) {
            const float *o = part + (((long)h * part_chunks + ch) * R_total + row_base + tid) * 2;
            merge_stats(mm, zz, o[0], o[1]);
        }
        bias_s[tid] = mm + __log2f(zz);   // zz >= 1: the row maximum itself contributes exp2(0)
    }
    __syncthreads();

    bf16x8 q[NBW][kSteps];
    load_queries<NBW>(Qw + ((long)h * R_total + row_base + row0) * kD, l32, hh, q);
    float bias[NBW][16];
#pragma unroll
    for (int b = 0; b < NBW; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) bias[b][i] = bias_s[row0 + kBlk * b + acc_row(i, hh)];

    const uint16_t *Kh = Kc + (long)h * N * kD;
    const int ntile = (kend - first + TK - 1) / TK;
    const int bpq = PERQ ? w / kBlk : 1;   // MFMA row blocks per query head

    auto multiply_tile = [&](const unsigned char *buf, int t) {
        bf16x8 kc[kSteps];
        tile_read(buf, stream, l32, hh, kc);

        f32x16 acc[NBW];
#pragma unroll
        for (int b = 0; b < NBW; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[b][i] = 0.f;
#pragma unroll
        for (int s = 0; s < kSteps; ++s)
#pragma unroll
            for (int b = 0; b < NBW; ++b)   // rows = queries, columns = keys
                acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q[b][s], kc[s], acc[b], 0, 0, 0);

        float pb[NBW];
#pragma unroll
        for (int b = 0; b < NBW; ++b) {
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) s += fast_exp2(fmaf(acc[b][i], c, -bias[b][i]));
            pb[b] = s;
        }
        const int key = first + TK * t + kBlk * stream + l32;
        if constexpr (!PERQ) {
            float p = pb[0];
#pragma unroll
            for (int b = 1; b < NBW; ++b) p += pb[b];
            p = add_other_half(p);
            if (hh == 0 && key < kend) {
                if (fused) vs[grp * span + key - (k0 - pool_half)] = p;
                else votes[((long)h * vote_rows + vote_row_base + grp) * P + key] = p;
            }
        } else {
            const int g0 = (row_base / kBlk + grp * NBW) / bpq;   // first query head of this row group
#pragma unroll
            for (int g = 0; g < NBW; ++g) {
                float p = 0.f;
#pragma unroll
                for (int b = 0; b < NBW; ++b) p += (b / bpq == g) ? pb[b] : 0.f;
                p = add_other_half(p);
                if (g0 + g < G && g * bpq < NBW && hh == 0 && key < kend)
                    votes[((long)h * G + g0 + g) * P + key] = p;
            }
        }
    };
    GKV_TILE_PIPELINE_TK(TK, NT, Kh, first, kend - 1, 1, ntile, multiply_tile, (void)0);
    if (fused) {
        __syncthreads();
        // votes of a key summed over the row groups (in group order, into group 0's array), then the
        // taps of every output in key order: the additions of the separate pooling kernel
        if (SPLIT > 1) {
            for (int u = tid; u < span; u += NT) {
                float v = 0.f;
#pragma unroll
                for (int g = 0; g < SPLIT; ++g) v += vs[g * span + u];
                vs[u] = v;
            }
            __syncthreads();
        }
        const float taps = (float)(2 * pool_half + 1), div = (float)G;
        for (int o = tid; o < k1 - k0; o += NT) {
            float acc = 0.f;
            if (pool_half == 3) {
#pragma unroll
                for (int t = 0; t < 7; ++t) acc += vs[o + t];
            } else {
                for (int t = 0; t <= 2 * pool_half; ++t) acc += vs[o + t];
            }
            votes[(long)h * P + k0 + o] = acc / taps / div;
        }
    }
}

// Keys per workgroup: about `wgs` workgroups over all heads, but at least 8 key blocks per
// wave so that loading the query operand is amortised.  The statistics pass takes half as many,
// twice as long workgroups as the votes pass (its workgroups hold no votes in LDS, and every
// workgroup pays for its queries and its first tiles: 423 -> 409 us on the 32-layer batch).
constexpr int kStatsWorkgroups = 512;
int chunk_keys_for(int Hkv, int N, int wgs = 1024)
{
    long ck = ((long)Hkv * N + wgs - 1) / wgs;
    if (ck < 1024) ck = 1024;
    ck = ((ck + 127) / 128) * 128;                            // 4 waves x 32 keys
    return (int)ck;
}

}  // namespace

MfmaScorePlan mfma_score_plan(int Hkv, int rows, int N)
{
    MfmaScorePlan pl;
    const int ck = chunk_keys_for(Hkv, N, kStatsWorkgroups);
    pl.chunks = (N + ck - 1) / ck;
    pl.part_bytes = (size_t)Hkv * pl.chunks * rows * 2 * sizeof(float);
    return pl;
}

namespace {

// The stacked query rows of a head are cut into parts of at most 128 rows; a part of
// nb 32-row blocks runs with 2 row groups per key stream when nb is even (and, for
// per-query-head votes, every query head stays inside one group), else with 1.
int part_rows(int R_total, int part) { return R_total - 128 * part < 128 ? R_total - 128 * part : 128; }
int part_split(int rows, int w, int per_qhead_votes)
{
    const int nb = rows / 32;
    if (nb % 2) return 1;
    if (per_qhead_votes && (w / 32) > nb / 2) return 1;
    return 2;
}

}  // namespace

// Rows of the votes array per KV head.
int mfma_score_vote_rows(int G, int w, int per_qhead_votes)
{
    if (per_qhead_votes) return G;
    const int R = G * w;
    int rows = 0;
    for (int part = 0; 128 * part < R; ++part) rows += part_split(part_rows(R, part), w, 0);
    return rows;
}

hipError_t launch_mfma_score_stats(const void *Kc, const void *Qw, int Hkv, int Hq, int N, int w,
                                  float scale, float *part, hipStream_t st)
{
    const int G = Hq / Hkv, R = G * w, P = N - w;
    const MfmaScorePlan plan = mfma_score_plan(Hkv, R, N);
    const int ck = chunk_keys_for(Hkv, N, kStatsWorkgroups);
    const float c = scale * 1.4426950408889634f;
    const uint16_t *K = (const uint16_t *)Kc, *Q = (const uint16_t *)Qw;
    if (R == 256) {   // one workgroup takes all 256 rows: 2 key streams x 4 row groups, tiles of 64 keys
        if (!allow_big_lds((const void *)score_stats_kernel<8, 4, 2>)) return hipGetLastError();
        hipLaunchKernelGGL((score_stats_kernel<8, 4, 2>), dim3(plan.chunks, Hkv), dim3(512), 2 * 64 * kPitch, st, K, Q, N,
                           P, w, ck, c, part, R, 0, 1);
        return hipGetLastError();
    }
    // other row counts beyond 128: parts of at most 128 rows, one launch per part
    const int merged = 1;
    dim3 grid(plan.chunks * merged, Hkv);
#define GKV_STATS(NB, SP)                                                                          \
    do {                                                                                           \
        if (!allow_big_lds((const void *)score_stats_kernel<NB, SP>)) return hipGetLastError();    \
        hipLaunchKernelGGL((score_stats_kernel<NB, SP>), grid, dim3(256 * SP), 2 * kTileBytes, st, \
                           K, Q, N, P, w, ck, c, part, R, row_base, merged);                       \
    } while (0)
    for (int pt = 0; 128 * pt < R; pt += merged) {
        const int row_base = 128 * pt;
        switch (part_rows(R, pt) / 32) {
            case 1: GKV_STATS(1, 1); break;
            case 2: GKV_STATS(2, 2); break;
            case 3: GKV_STATS(3, 1); break;
            case 4: GKV_STATS(4, 2); break;
            default: return hipErrorInvalidValue;
        }
        if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
    }
#undef GKV_STATS
    return hipGetLastError();
}

template <int NB, int SPLIT, int STREAMS = 4>
static void launch_votes_nb(dim3 grid, const uint16_t *K, const uint16_t *Q, int N, int P, int w, int G,
                            int ck, float c, const float *part, int chunks, int per_q, float *votes,
                            int R_total, int row_base, int vote_rows, int vote_row_base, int nparts,
                            int pool_half, hipStream_t st)
{
    const size_t lds = 2 * (kBlk * STREAMS) * kPitch + (pool_half >= 0 ? (size_t)SPLIT * (ck + 2 * pool_half) * 4 : 0);
    if (per_q) {
        if (!allow_big_lds((const void *)score_votes_kernel<NB, SPLIT, true, STREAMS>)) return;
        hipLaunchKernelGGL((score_votes_kernel<NB, SPLIT, true, STREAMS>), grid, dim3(64 * STREAMS * SPLIT),
                           lds, st, K, Q, N, P, w, G, ck, c, part, chunks, votes, R_total,
                           row_base, vote_rows, vote_row_base, nparts, pool_half);
    } else {
        if (!allow_big_lds((const void *)score_votes_kernel<NB, SPLIT, false, STREAMS>)) return;
        hipLaunchKernelGGL((score_votes_kernel<NB, SPLIT, false, STREAMS>), grid, dim3(64 * STREAMS * SPLIT),
                           lds, st, K, Q, N, P, w, G, ck, c, part, chunks, votes, R_total,
                           row_base, vote_rows, vote_row_base, nparts, pool_half);
    }
}

bool mfma_score_fuses_pool(int G, int w, int per_qhead_votes, int pool_kernel)
{
    return !per_qhead_votes && (G * w <= 128 || G * w == 256) && pool_kernel <= 33;
}

hipError_t launch_mfma_score_votes(const void *Kc, const void *Qw, int Hkv, int Hq, int N, int w,
                                  float scale, int per_qhead_votes, int fused_pool_kernel,
                                  const float *part, float *votes, hipStream_t st)
{
    const int G = Hq / Hkv, R = G * w, P = N - w;
    const MfmaScorePlan plan = mfma_score_plan(Hkv, R, N);
    // fused pooling: a workgroup also multiplies pool_half keys on either side of its chunk; the
    // P prefix keys are spread evenly over the chunks
    const int pool_half = fused_pool_kernel > 0 ? (fused_pool_kernel - 1) / 2 : -1;
    const int vchunks = (N + chunk_keys_for(Hkv, N) - 1) / chunk_keys_for(Hkv, N);
    const int ck = pool_half >= 0 ? (P + vchunks - 1) / vchunks : chunk_keys_for(Hkv, N);
    const float c = scale * 1.4426950408889634f;
    const uint16_t *K = (const uint16_t *)Kc, *Q = (const uint16_t *)Qw;
    const int merged = 1;
    dim3 grid(vchunks * merged, Hkv);
    const int vote_rows = mfma_score_vote_rows(G, w, per_qhead_votes);
    int vote_row_base = 0;
    if (R == 256 && !per_qhead_votes) {   // all rows in one workgroup (see the statistics pass): four row groups
        // with fused pooling the votes of four row groups stay in LDS: chunks of 6144 keys
        const int ckv = pool_half >= 0 ? 6144 : ck;
        const dim3 gridv = pool_half >= 0 ? dim3((P + ckv - 1) / ckv, Hkv) : grid;
        launch_votes_nb<8, 4, 2>(gridv, K, Q, N, P, w, G, ckv, c, part, plan.chunks, 0, votes, R, 0, vote_rows, 0, 1,
                                 pool_half, st);
        return hipGetLastError();
    }
#define GKV_VOTES(NB, SP)                                                                             \
    launch_votes_nb<NB, SP>(grid, K, Q, N, P, w, G, ck, c, part, plan.chunks, per_qhead_votes, votes, R, \
                            row_base, vote_rows, vote_row_base, merged, pool_half, st)
    for (int pt = 0; 128 * pt < R; pt += merged) {
        const int row_base = 128 * pt, rows = part_rows(R, pt);
        const int split = part_split(rows, w, per_qhead_votes);
        switch (rows / 32) {
            case 1: GKV_VOTES(1, 1); break;
            case 2: if (split == 2) GKV_VOTES(2, 2); else GKV_VOTES(2, 1); break;
            case 3: GKV_VOTES(3, 1); break;
            case 4: if (split == 2) GKV_VOTES(4, 2); else GKV_VOTES(4, 1); break;
            default: return hipErrorInvalidValue;
        }
        vote_row_base += split;
        if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
    }
#undef GKV_VOTES
    return hipGetLastError();
}

}  // namespace gkv
