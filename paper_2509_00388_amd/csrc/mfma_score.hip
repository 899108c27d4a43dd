// Stage I on the matrix cores (bf16 inputs, d = 128, fp32 accumulation).
//
// Per KV head the window queries of its G query heads are stacked into one
// R x 128 operand (R = G*w <= 128 rows), held in registers by every wave for
// the whole kernel.  Keys stream from HBM in blocks of 32 rows straight into
// MFMA operand registers (each lane loads 16-byte pieces of "its" key row; the
// 8 pieces cover the row's half that belongs to the lane's half-wave), so one
// key block costs R/32 x 8 v_mfma_f32_32x32x16_bf16 and is read exactly once
// per pass.  Each wave walks its own key blocks: no barrier in the main loop.
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

namespace gkv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int kD = 128;      // head dimension
constexpr int kSteps = 8;    // k-steps of 16 per 128
constexpr int kBlk = 32;     // keys per MFMA block

__device__ __forceinline__ bf16x8 load8(const uint16_t *p)
{
    return *reinterpret_cast<const bf16x8 *>(p);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// (m1, z1) <- softmax-statistics merge with (m2, z2), base 2.
__device__ __forceinline__ void merge_stats(float &m1, float &z1, float m2, float z2)
{
    const float mn = fmaxf(m1, m2);
    if (mn == -INFINITY) { m1 = mn; z1 = 0.f; return; }
    z1 = z1 * fast_exp2(m1 - mn) + z2 * fast_exp2(m2 - mn);
    m1 = mn;
}

// Row of the 32x32 MFMA result held in accumulator register i of a lane in
// half-wave hh (the column is lane % 32).
__device__ __forceinline__ int acc_row(int i, int hh) { return 8 * (i >> 2) + 4 * hh + (i & 3); }

template <int NB>
__device__ __forceinline__ void load_queries(const uint16_t *Qb, int l32, int hh, bf16x8 (&q)[NB][kSteps])
{
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int s = 0; s < kSteps; ++s)
            q[b][s] = load8(Qb + (long)(kBlk * b + l32) * kD + 16 * s + 8 * hh);
}

// Key block t of the chunk: lane (l32, hh) takes row k0 + 32 t + l32, clamped
// to the last row of the head (clamped rows are masked by the caller).
__device__ __forceinline__ void load_keys(const uint16_t *Kh, int key, int last_row, int hh,
                                          bf16x8 (&kr)[kSteps])
{
    const uint16_t *p = Kh + (long)min(key, last_row) * kD + 8 * hh;
#pragma unroll
    for (int s = 0; s < kSteps; ++s) kr[s] = load8(p + 16 * s);
}

// ---------------------------------------------------------------- pass A ---
template <int NB>
__global__ __launch_bounds__(256) void score_stats_kernel(
    const uint16_t *__restrict__ Kc, const uint16_t *__restrict__ Qw, int N, int P, int w,
    int chunk_keys, float c, float *__restrict__ part)
{
    constexpr int R = NB * kBlk;
    __shared__ float sm[4][R], sz[4][R];
    const int h = blockIdx.y, chunk = blockIdx.x, nchunks = gridDim.x;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, hh = lane >> 5;

    bf16x8 q[NB][kSteps];
    load_queries<NB>(Qw + (long)h * R * kD, l32, hh, q);
    int last_vis[NB];   // last key the lane's query of block b may see (causal window)
    float m[NB], z[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        last_vis[b] = P + (kBlk * b + l32) % w;
        m[b] = -INFINITY;
        z[b] = 0.f;
    }

    const uint16_t *Kh = Kc + (long)h * N * kD;
    const int k0 = chunk * chunk_keys, k1 = min(N, k0 + chunk_keys);
    const int nblk = (k1 - k0 + kBlk - 1) / kBlk;

    bf16x8 kn[kSteps];
    int t = wv;
    if (t < nblk) load_keys(Kh, k0 + kBlk * t + l32, N - 1, hh, kn);
    for (; t < nblk; t += 4) {
        bf16x8 kc[kSteps];
#pragma unroll
        for (int s = 0; s < kSteps; ++s) kc[s] = kn[s];
        if (t + 4 < nblk) load_keys(Kh, k0 + kBlk * (t + 4) + l32, N - 1, hh, kn);

        f32x16 acc[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[b][i] = 0.f;
#pragma unroll
        for (int s = 0; s < kSteps; ++s)
#pragma unroll
            for (int b = 0; b < NB; ++b)   // rows = keys, columns = queries
                acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kc[s], q[b][s], acc[b], 0, 0, 0);

        const int kb = k0 + kBlk * t;
        if (kb + kBlk <= P) {   // every key of the block is a prefix key: visible to all rows
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                float tm = acc[b][0];
#pragma unroll
                for (int i = 1; i < 16; ++i) tm = fmaxf(tm, acc[b][i]);
                const float mn = fmaxf(m[b], tm * c);
                float zz = z[b] * fast_exp2(m[b] - mn);
#pragma unroll
                for (int i = 0; i < 16; ++i) zz += fast_exp2(fmaf(acc[b][i], c, -mn));
                m[b] = mn;
                z[b] = zz;
            }
        } else {                // the block touches the window (or the end of the head): mask
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                float tm = -INFINITY;
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (kb + acc_row(i, hh) <= last_vis[b]) tm = fmaxf(tm, acc[b][i]);
                const float mn = fmaxf(m[b], tm * c);
                if (mn != -INFINITY) {
                    float zz = z[b] * fast_exp2(m[b] - mn);
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        if (kb + acc_row(i, hh) <= last_vis[b]) zz += fast_exp2(fmaf(acc[b][i], c, -mn));
                    m[b] = mn;
                    z[b] = zz;
                }
            }
        }
    }

    // merge the two half-waves (same query, other key rows), then the 4 waves
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const float m2 = __shfl_xor(m[b], 32, kWave), z2 = __shfl_xor(z[b], 32, kWave);
        merge_stats(m[b], z[b], m2, z2);
        if (hh == 0) { sm[wv][kBlk * b + l32] = m[b]; sz[wv][kBlk * b + l32] = z[b]; }
    }
    __syncthreads();
    if (tid < R) {
        float mm = sm[0][tid], zz = sz[0][tid];
#pragma unroll
        for (int u = 1; u < 4; ++u) merge_stats(mm, zz, sm[u][tid], sz[u][tid]);
        float *o = part + (((long)h * nchunks + chunk) * R + tid) * 2;
        o[0] = mm;
        o[1] = zz;
    }
}

// ---------------------------------------------------------------- pass B ---
template <int NB, bool PERQ>
__global__ __launch_bounds__(256) void score_votes_kernel(
    const uint16_t *__restrict__ Kc, const uint16_t *__restrict__ Qw, int N, int P, int w, int G,
    int chunk_keys, float c, const float *__restrict__ part, int part_chunks,
    float *__restrict__ votes)
{
    constexpr int R = NB * kBlk;
    __shared__ float bias_s[R];
    const int h = blockIdx.y, chunk = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, hh = lane >> 5;

    const int k0 = chunk * chunk_keys, k1 = min(P, k0 + chunk_keys);
    if (k0 >= P) return;

    if (tid < R) {   // row statistics of the whole head: merge the chunks of pass A
        float mm = -INFINITY, zz = 0.f;
        for (int ch = 0; ch < part_chunks; ++ch) {
            const float *o = part + (((long)h * part_chunks + ch) * R + tid) * 2;
            merge_stats(mm, zz, o[0], o[1]);
        }
        bias_s[tid] = mm + __log2f(zz);   // zz >= 1: the row maximum itself contributes exp2(0)
    }
    __syncthreads();

    bf16x8 q[NB][kSteps];
    load_queries<NB>(Qw + (long)h * R * kD, l32, hh, q);
    float bias[NB][16];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) bias[b][i] = bias_s[kBlk * b + acc_row(i, hh)];

    const uint16_t *Kh = Kc + (long)h * N * kD;
    const int nblk = (k1 - k0 + kBlk - 1) / kBlk;
    const int bpq = PERQ ? w / kBlk : 1;   // MFMA row blocks per query head

    bf16x8 kn[kSteps];
    int t = wv;
    if (t < nblk) load_keys(Kh, k0 + kBlk * t + l32, P - 1, hh, kn);
    for (; t < nblk; t += 4) {
        bf16x8 kc[kSteps];
#pragma unroll
        for (int s = 0; s < kSteps; ++s) kc[s] = kn[s];
        if (t + 4 < nblk) load_keys(Kh, k0 + kBlk * (t + 4) + l32, P - 1, hh, kn);

        f32x16 acc[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[b][i] = 0.f;
#pragma unroll
        for (int s = 0; s < kSteps; ++s)
#pragma unroll
            for (int b = 0; b < NB; ++b)   // rows = queries, columns = keys
                acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q[b][s], kc[s], acc[b], 0, 0, 0);

        float pb[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) s += fast_exp2(fmaf(acc[b][i], c, -bias[b][i]));
            pb[b] = s;
        }
        const int key = k0 + kBlk * t + l32;
        if constexpr (!PERQ) {
            float p = pb[0];
#pragma unroll
            for (int b = 1; b < NB; ++b) p += pb[b];
            p += __shfl_xor(p, 32, kWave);
            if (hh == 0 && key < k1) votes[(long)h * P + key] = p;
        } else {
#pragma unroll
            for (int g = 0; g < NB; ++g) {
                float p = 0.f;
#pragma unroll
                for (int b = 0; b < NB; ++b) p += (b / bpq == g) ? pb[b] : 0.f;
                p += __shfl_xor(p, 32, kWave);
                if (g < G && hh == 0 && key < k1) votes[((long)h * G + g) * P + key] = p;
            }
        }
    }
}

// Keys per workgroup: about 1024 workgroups in flight over all heads, but at least
// 8 key blocks per wave so that loading the query operand is amortised.
int chunk_keys_for(int Hkv, int N)
{
    long ck = ((long)Hkv * N + 1023) / 1024;
    if (ck < 1024) ck = 1024;
    ck = ((ck + 127) / 128) * 128;                            // 4 waves x 32 keys
    return (int)ck;
}

}  // namespace

MfmaScorePlan mfma_score_plan(int Hkv, int rows, int N)
{
    MfmaScorePlan pl;
    const int ck = chunk_keys_for(Hkv, N);
    pl.chunks = (N + ck - 1) / ck;
    pl.part_bytes = (size_t)Hkv * pl.chunks * rows * 2 * sizeof(float);
    return pl;
}

hipError_t launch_mfma_score_stats(const void *Kc, const void *Qw, int Hkv, int Hq, int N, int w,
                                  float scale, float *part, hipStream_t st)
{
    const int G = Hq / Hkv, R = G * w, P = N - w;
    const MfmaScorePlan plan = mfma_score_plan(Hkv, R, N);
    const int ck = chunk_keys_for(Hkv, N);
    const float c = scale * 1.4426950408889634f;
    const uint16_t *K = (const uint16_t *)Kc, *Q = (const uint16_t *)Qw;
    dim3 grid(plan.chunks, Hkv), block(256);
    switch (R / 32) {
        case 1: hipLaunchKernelGGL(score_stats_kernel<1>, grid, block, 0, st, K, Q, N, P, w, ck, c, part); break;
        case 2: hipLaunchKernelGGL(score_stats_kernel<2>, grid, block, 0, st, K, Q, N, P, w, ck, c, part); break;
        case 3: hipLaunchKernelGGL(score_stats_kernel<3>, grid, block, 0, st, K, Q, N, P, w, ck, c, part); break;
        case 4: hipLaunchKernelGGL(score_stats_kernel<4>, grid, block, 0, st, K, Q, N, P, w, ck, c, part); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int NB>
static void launch_votes_nb(dim3 grid, const uint16_t *K, const uint16_t *Q, int N, int P, int w, int G,
                            int ck, float c, const float *part, int chunks, int per_q, float *votes,
                            hipStream_t st)
{
    if (per_q)
        hipLaunchKernelGGL((score_votes_kernel<NB, true>), grid, dim3(256), 0, st, K, Q, N, P, w, G, ck,
                           c, part, chunks, votes);
    else
        hipLaunchKernelGGL((score_votes_kernel<NB, false>), grid, dim3(256), 0, st, K, Q, N, P, w, G, ck,
                           c, part, chunks, votes);
}

hipError_t launch_mfma_score_votes(const void *Kc, const void *Qw, int Hkv, int Hq, int N, int w,
                                  float scale, int per_qhead_votes, const float *part, float *votes,
                                  hipStream_t st)
{
    const int G = Hq / Hkv, R = G * w, P = N - w;
    const MfmaScorePlan plan = mfma_score_plan(Hkv, R, N);
    const int ck = chunk_keys_for(Hkv, N);
    const float c = scale * 1.4426950408889634f;
    const uint16_t *K = (const uint16_t *)Kc, *Q = (const uint16_t *)Qw;
    dim3 grid(plan.chunks, Hkv);
    switch (R / 32) {
        case 1: launch_votes_nb<1>(grid, K, Q, N, P, w, G, ck, c, part, plan.chunks, per_qhead_votes, votes, st); break;
        case 2: launch_votes_nb<2>(grid, K, Q, N, P, w, G, ck, c, part, plan.chunks, per_qhead_votes, votes, st); break;
        case 3: launch_votes_nb<3>(grid, K, Q, N, P, w, G, ck, c, part, plan.chunks, per_qhead_votes, votes, st); break;
        case 4: launch_votes_nb<4>(grid, K, Q, N, P, w, G, ck, c, part, plan.chunks, per_qhead_votes, votes, st); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace gkv
