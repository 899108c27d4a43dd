// Eq. 1 and Eq. 3 on the matrix cores: cosine of every source key against every
// prefix key (bf16 inputs, d = 128, fp32 accumulation), and each source's m
// largest edges without ever storing the S x P edge block.
//
// Up to 64 source rows (two 32-row MFMA blocks) are held in registers; keys
// stream from HBM in 32-row blocks straight into MFMA operand registers, as in
// the scoring kernels.  The squared norm of each streamed key is accumulated
// from the very registers that feed the MFMA, so the keys are read once.
//
// Neighbourhoods in one streaming pass:
//   1. the same kernel first runs on an evenly strided sample of the keys and
//      writes that small edge block; the m-th largest sampled edge of a source
//      is a lower bound of its m-th largest edge overall (a subset's m-th
//      largest can only be smaller), and a tight one for a sample of P/16 keys;
//   2. the streaming pass keeps only the edges that reach the bound (a few
//      hundred per source), staged in LDS and appended to per-source lists;
//   3. an exact (value desc, index asc) top-m over each short list.
// A source whose list overflows (masses of equal edges, adversarial order) sets
// a per-head flag and that head is redone through the dense block instead.
#include "common.hpp"
#include "kernels.hpp"

namespace gkv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int kD = 128, kSteps = 8, kBlk = 32;
constexpr int kSB = 2;            // source blocks of 32 per workgroup
constexpr int kRows = kSB * kBlk; // source rows per workgroup
constexpr int kRing = 6144;       // candidates a workgroup can stage in LDS (48 KiB)

__device__ __forceinline__ bf16x8 load8(const uint16_t *p)
{
    return *reinterpret_cast<const bf16x8 *>(p);
}
__device__ __forceinline__ int acc_row(int i, int hh) { return 8 * (i >> 2) + 4 * hh + (i & 3); }

// Sum of squares of the 64 elements a lane holds of its row (8 k-steps x 8).
__device__ __forceinline__ float half_row_sumsq(const bf16x8 (&r)[kSteps])
{
    float a = 0.f;
#pragma unroll
    for (int s = 0; s < kSteps; ++s)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float v = (float)r[s][e];
            a = fmaf(v, v, a);
        }
    return a;
}

enum { kDense = 0, kFilter = 1 };

struct FilterArgs {
    const float *tau;      // [Hkv, S] lower bound of each source's m-th largest edge
    uint2 *cand;           // [Hkv, S, cap] (edge bits, key index)
    int32_t *cand_cnt;     // [Hkv, S]
    int32_t *overflow;     // [Hkv]
    int cap;
};

// Column c of the output is key c * key_stride (key_stride = 1: every key).
// kDense: E[h, slot, c] = cosine, -inf where the key is the source itself.
// kFilter: edges >= tau[h, slot] (self excluded) are appended to cand[h, slot, :].
// zero_cnt (dense only, may be null): the first chunk also clears cand_cnt /
// overflow of its head for the filter pass that follows.
template <int MODE>
__global__ __launch_bounds__(256) void cosine_kernel(const uint16_t *__restrict__ Kc, int N,
                                                     int n_cols, int key_stride, int S,
                                                     const int32_t *__restrict__ src,
                                                     int chunk_cols, float *__restrict__ E,
                                                     FilterArgs fa, const int32_t *__restrict__ gate)
{
    __shared__ float inv_s[kRows];
    __shared__ int32_t idx_s[kRows];
    __shared__ float tau_s[kRows];
    __shared__ uint2 ring[MODE == kFilter ? kRing : 1];
    __shared__ int32_t ring_n, row_cnt[kRows], row_base[kRows], row_pos[kRows];

    const int h = blockIdx.y, chunk = blockIdx.x, s_base = blockIdx.z * kRows;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, hh = lane >> 5;
    if (gate && gate[h] == 0) return;
    const uint16_t *Kh = Kc + (long)h * N * kD;
    const int c0 = chunk * chunk_cols, c1 = min(n_cols, c0 + chunk_cols);
    if (c0 >= n_cols) return;

    if constexpr (MODE == kDense) {
        if (fa.cand_cnt && chunk == 0) {
            if (tid < kRows && s_base + tid < S) fa.cand_cnt[(long)h * S + s_base + tid] = 0;
            if (tid == 0 && blockIdx.z == 0) fa.overflow[h] = 0;
        }
    }

    // source rows -> registers (slots beyond S repeat the last source; never written out)
    bf16x8 q[kSB][kSteps];
#pragma unroll
    for (int b = 0; b < kSB; ++b) {
        const int slot = min(s_base + kBlk * b + l32, S - 1);
        const int32_t i = src[(long)h * S + slot];
        const uint16_t *p = Kh + (long)i * kD + 8 * hh;
#pragma unroll
        for (int s = 0; s < kSteps; ++s) q[b][s] = load8(p + 16 * s);
        float sq = half_row_sumsq(q[b]);
        sq += __shfl_xor(sq, 32, kWave);
        if (wv == 0 && hh == 0) {
            inv_s[kBlk * b + l32] = sq == 0.f ? 0.f : 1.0f / sqrtf(sq);
            idx_s[kBlk * b + l32] = i;
            if constexpr (MODE == kFilter)   // a hair below the bound: never lose an edge to rounding
                tau_s[kBlk * b + l32] = fa.tau[(long)h * S + slot] - 4e-6f;
        }
    }
    if constexpr (MODE == kFilter) {
        if (tid == 0) ring_n = 0;
        if (tid < kRows) { row_cnt[tid] = 0; row_pos[tid] = 0; }
    }
    __syncthreads();
    float inv_src[kSB][16], tau[MODE == kFilter ? kSB : 1][16];
    int32_t idx_src[kSB][16];
#pragma unroll
    for (int b = 0; b < kSB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            inv_src[b][i] = inv_s[kBlk * b + acc_row(i, hh)];
            idx_src[b][i] = idx_s[kBlk * b + acc_row(i, hh)];
            if constexpr (MODE == kFilter) {
                // rows past S never pass the filter
                tau[b][i] = (s_base + kBlk * b + acc_row(i, hh) < S) ? tau_s[kBlk * b + acc_row(i, hh)]
                                                                      : INFINITY;
            }
        }

    const int nblk = (c1 - c0 + kBlk - 1) / kBlk;
    bf16x8 kn[kSteps];
    int t = wv;
    auto load_keys = [&](int col, bf16x8(&kr)[kSteps]) {
        const uint16_t *p = Kh + (long)min(col, n_cols - 1) * key_stride * kD + 8 * hh;
#pragma unroll
        for (int s = 0; s < kSteps; ++s) kr[s] = load8(p + 16 * s);
    };
    if (t < nblk) load_keys(c0 + kBlk * t + l32, kn);
    for (; t < nblk; t += 4) {
        bf16x8 kc[kSteps];
#pragma unroll
        for (int s = 0; s < kSteps; ++s) kc[s] = kn[s];
        if (t + 4 < nblk) load_keys(c0 + kBlk * (t + 4) + l32, kn);

        f32x16 acc[kSB];
#pragma unroll
        for (int b = 0; b < kSB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[b][i] = 0.f;
#pragma unroll
        for (int s = 0; s < kSteps; ++s)
#pragma unroll
            for (int b = 0; b < kSB; ++b)   // rows = sources, columns = keys
                acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q[b][s], kc[s], acc[b], 0, 0, 0);

        float sq = half_row_sumsq(kc);
        sq += __shfl_xor(sq, 32, kWave);
        const float inv_k = sq == 0.f ? 0.f : 1.0f / sqrtf(sq);
        const int col = c0 + kBlk * t + l32;
        const int key = col * key_stride;
        if constexpr (MODE == kDense) {
            if (col < c1) {
#pragma unroll
                for (int b = 0; b < kSB; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int slot = s_base + kBlk * b + acc_row(i, hh);
                        if (slot < S) {
                            float e = acc[b][i] * inv_src[b][i] * inv_k;
                            if (key == idx_src[b][i]) e = -INFINITY;
                            E[((long)h * S + slot) * n_cols + col] = e;
                        }
                    }
            }
        } else {
            uint32_t pass = 0;   // bit (16 b + i): edge of that accumulator reaches its bound
            float ev[kSB][16];
#pragma unroll
            for (int b = 0; b < kSB; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    ev[b][i] = acc[b][i] * inv_src[b][i] * inv_k;
                    if (ev[b][i] >= tau[b][i] && key != idx_src[b][i]) pass |= 1u << (16 * b + i);
                }
            if (col >= c1) pass = 0;
            if (pass) {
                const int cnt = __popc(pass);
                const int at = atomicAdd(&ring_n, cnt);
                int w = 0;
#pragma unroll
                for (int b = 0; b < kSB; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        if (pass & (1u << (16 * b + i))) {
                            if (at + w < kRing)
                                ring[at + w] = make_uint2(__float_as_uint(ev[b][i]),
                                                          ((uint32_t)(kBlk * b + acc_row(i, hh)) << 24) | (uint32_t)key);
                            ++w;
                        }
            }
        }
    }

    if constexpr (MODE == kFilter) {
        // Flush: count per source row, reserve room in the global lists, scatter.
        __syncthreads();
        const int n_stage = ring_n;
        const bool lost = n_stage > kRing;
        const int n_ring = lost ? kRing : n_stage;
        for (int r = tid; r < n_ring; r += 256) atomicAdd(&row_cnt[ring[r].y >> 24], 1);
        __syncthreads();
        if (tid < kRows) {
            const int c = row_cnt[tid];
            int base = 0;
            if (c > 0) base = atomicAdd(&fa.cand_cnt[(long)h * S + s_base + tid], c);
            row_base[tid] = base;
            if (base + c > fa.cap || lost) fa.overflow[h] = 1;
        }
        __syncthreads();
        for (int r = tid; r < n_ring; r += 256) {
            const uint2 v = ring[r];
            const int row = v.y >> 24;
            const int at = row_base[row] + atomicAdd(&row_pos[row], 1);
            if (at < fa.cap)
                fa.cand[((long)h * S + s_base + row) * fa.cap + at] = make_uint2(v.x, v.y & 0xffffffu);
        }
    }
}

__device__ __forceinline__ uint32_t ord_key_u(uint32_t bits)
{
    float f = __uint_as_float(bits) + 0.0f;
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Exact top-m of one source's candidate list by (edge desc, key index asc),
// written in ascending key order.  One workgroup per (source, head); heads whose
// overflow flag is set are left to the dense path.
//
// The list is short (a few hundred entries) and all composite keys
// (edge, -index) are distinct, so the rank of an entry is the number of entries
// that beat it; entries of rank < m are the neighbourhood, and their output
// position is their rank by key index among themselves.
__global__ __launch_bounds__(256) void nbr_select_kernel(const uint2 *__restrict__ cand,
                                                         const int32_t *__restrict__ cand_cnt,
                                                         const int32_t *__restrict__ overflow,
                                                         int S, int cap, int m,
                                                         int32_t *__restrict__ nbr,
                                                         float *__restrict__ nbr_e)
{
    extern __shared__ uint64_t comp[];          // [cap] composite keys, then the winners
    __shared__ int32_t n_win;
    const int a = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
    if (overflow[h]) return;
    const long row = (long)h * S + a;
    const int n = min(cand_cnt[row], cap);
    const uint2 *c = cand + row * cap;
    uint64_t *win = comp + cap;                 // [m] winners as (key index << 32 | edge bits)
    if (tid == 0) n_win = 0;
    for (int r = tid; r < n; r += 256) {
        const uint2 v = c[r];
        comp[r] = ((uint64_t)ord_key_u(v.x) << 32) | (uint32_t)(0xffffffffu - v.y);
    }
    __syncthreads();
    for (int r = tid; r < n; r += 256) {
        const uint64_t mine = comp[r];
        int rank = 0;
        for (int u = 0; u < n; ++u) rank += comp[u] > mine;
        if (rank < m) {
            const int at = atomicAdd(&n_win, 1);
            const uint2 v = c[r];
            win[at] = ((uint64_t)v.y << 32) | v.x;
        }
    }
    __syncthreads();
    const int nw = n_win;                       // == m whenever n >= m
    for (int r = tid; r < nw; r += 256) {
        const uint64_t mine = win[r];
        int pos = 0;
        for (int u = 0; u < nw; ++u) pos += win[u] < mine;
        nbr[row * m + pos] = (int32_t)(mine >> 32);
        nbr_e[row * m + pos] = __uint_as_float((uint32_t)mine);
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

int mfma_sample_cols(int P)
{
    int ps = ((P / 16 + 127) / 128) * 128;
    if (ps < 2048) ps = 2048;
    if (ps > 8192) ps = 8192;
    return ps;
}

int mfma_cand_cap(int P, int m)
{
    const int stride = P / mfma_sample_cols(P);
    long cap = 4L * m * stride;
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
    return (size_t)mfma_cand_cap(P, m) * 8 + (size_t)m * 8 <= 96 * 1024;
}

hipError_t launch_mfma_cosine(const void *Kc, int Hkv, int N, int P, int S, const int32_t *src,
                              float *E, const int32_t *gate, hipStream_t st)
{
    const int sgroups = (S + kRows - 1) / kRows;
    const int ck = chunk_cols_for(Hkv, sgroups, P);
    const int chunks = (P + ck - 1) / ck;
    FilterArgs fa{};
    hipLaunchKernelGGL(cosine_kernel<kDense>, dim3(chunks, Hkv, sgroups), dim3(256), 0, st,
                       (const uint16_t *)Kc, N, P, 1, S, src, ck, E, fa, gate);
    return hipGetLastError();
}

hipError_t launch_mfma_cosine_sample(const void *Kc, int Hkv, int N, int P, int S,
                                     const int32_t *src, float *E_sample, int32_t *cand_cnt,
                                     int32_t *overflow, hipStream_t st)
{
    const int ps = mfma_sample_cols(P), stride = P / ps;
    const int sgroups = (S + kRows - 1) / kRows;
    const int ck = chunk_cols_for(Hkv, sgroups, ps);
    const int chunks = (ps + ck - 1) / ck;
    FilterArgs fa{};
    fa.cand_cnt = cand_cnt;
    fa.overflow = overflow;
    hipLaunchKernelGGL(cosine_kernel<kDense>, dim3(chunks, Hkv, sgroups), dim3(256), 0, st,
                       (const uint16_t *)Kc, N, ps, stride, S, src, ck, E_sample, fa,
                       (const int32_t *)nullptr);
    return hipGetLastError();
}

hipError_t launch_mfma_cosine_filter(const void *Kc, int Hkv, int N, int P, int S, int m,
                                     const int32_t *src, const float *tau, void *cand,
                                     int32_t *cand_cnt, int32_t *overflow, hipStream_t st)
{
    const int sgroups = (S + kRows - 1) / kRows;
    // expected staged candidates per workgroup = rows * m * stride / chunks: keep it under half the ring
    const int stride = P / mfma_sample_cols(P);
    const int min_chunks = (int)(((long)kRows * m * stride + kRing / 2 - 1) / (kRing / 2));
    const int ck = chunk_cols_for(Hkv, sgroups, P, min_chunks);
    const int chunks = (P + ck - 1) / ck;
    FilterArgs fa{tau, (uint2 *)cand, cand_cnt, overflow, mfma_cand_cap(P, m)};
    hipLaunchKernelGGL(cosine_kernel<kFilter>, dim3(chunks, Hkv, sgroups), dim3(256), 0, st,
                       (const uint16_t *)Kc, N, P, 1, S, src, ck, (float *)nullptr, fa,
                       (const int32_t *)nullptr);
    return hipGetLastError();
}

hipError_t launch_nbr_select(const void *cand, const int32_t *cand_cnt, const int32_t *overflow,
                             int Hkv, int P, int S, int m, int32_t *nbr, float *nbr_e,
                             hipStream_t st)
{
    const int cap = mfma_cand_cap(P, m);
    const size_t lds = (size_t)cap * 8 + (size_t)m * 8;
    static bool opt_in = false;   // more than 64 KiB of dynamic LDS needs a one-time opt-in
    if (lds > 65536 && !opt_in) {
        if (hipFuncSetAttribute((const void *)nbr_select_kernel,
                                hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024) != hipSuccess)
            return hipGetLastError();
        opt_in = true;
    }
    hipLaunchKernelGGL(nbr_select_kernel, dim3(S, Hkv), dim3(256), lds, st, (const uint2 *)cand,
                       cand_cnt, overflow, S, cap, m, nbr, nbr_e);
    return hipGetLastError();
}

}  // namespace gkv
