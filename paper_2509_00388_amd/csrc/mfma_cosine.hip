// Eq. 1 on the matrix cores: cosine of every source key against every prefix
// key (bf16 inputs, d = 128, fp32 accumulation).
//
// Up to 64 source rows (two 32-row MFMA blocks) are held in registers; keys
// stream from HBM in 32-row blocks straight into MFMA operand registers, as in
// the scoring kernels.  The squared norm of each streamed key is accumulated
// from the very registers that feed the MFMA, so the keys are read once.  The
// source's own column gets -inf (Eq. 3 excludes j = i).
#include "common.hpp"
#include "kernels.hpp"

namespace gkv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int kD = 128, kSteps = 8, kBlk = 32;
constexpr int kSB = 2;   // source blocks of 32 per workgroup

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

__global__ __launch_bounds__(256) void cosine_kernel(const uint16_t *__restrict__ Kc, int N, int P,
                                                     int S, const int32_t *__restrict__ src,
                                                     int chunk_keys, float *__restrict__ E)
{
    __shared__ float inv_s[kSB * kBlk];
    __shared__ int32_t idx_s[kSB * kBlk];
    const int h = blockIdx.y, chunk = blockIdx.x, s_base = blockIdx.z * (kSB * kBlk);
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, hh = lane >> 5;
    const uint16_t *Kh = Kc + (long)h * N * kD;
    const int k0 = chunk * chunk_keys, k1 = min(P, k0 + chunk_keys);
    if (k0 >= P) return;

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
        }
    }
    __syncthreads();
    float inv_src[kSB][16];
    int32_t idx_src[kSB][16];
#pragma unroll
    for (int b = 0; b < kSB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            inv_src[b][i] = inv_s[kBlk * b + acc_row(i, hh)];
            idx_src[b][i] = idx_s[kBlk * b + acc_row(i, hh)];
        }

    const int nblk = (k1 - k0 + kBlk - 1) / kBlk;
    bf16x8 kn[kSteps];
    int t = wv;
    auto load_keys = [&](int key, bf16x8(&kr)[kSteps]) {
        const uint16_t *p = Kh + (long)min(key, P - 1) * kD + 8 * hh;
#pragma unroll
        for (int s = 0; s < kSteps; ++s) kr[s] = load8(p + 16 * s);
    };
    if (t < nblk) load_keys(k0 + kBlk * t + l32, kn);
    for (; t < nblk; t += 4) {
        bf16x8 kc[kSteps];
#pragma unroll
        for (int s = 0; s < kSteps; ++s) kc[s] = kn[s];
        if (t + 4 < nblk) load_keys(k0 + kBlk * (t + 4) + l32, kn);

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
        const int key = k0 + kBlk * t + l32;
        if (key < k1) {
#pragma unroll
            for (int b = 0; b < kSB; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int slot = s_base + kBlk * b + acc_row(i, hh);
                    if (slot < S) {
                        float e = acc[b][i] * inv_src[b][i] * inv_k;
                        if (key == idx_src[b][i]) e = -INFINITY;
                        E[((long)h * S + slot) * P + key] = e;
                    }
                }
        }
    }
}

}  // namespace

hipError_t launch_mfma_cosine(const void *Kc, int Hkv, int N, int P, int S, const int32_t *src,
                              float *E, hipStream_t st)
{
    const int sgroups = (S + kSB * kBlk - 1) / (kSB * kBlk);
    int target = 256 / (Hkv * sgroups);
    if (target < 1) target = 1;
    int ck = (P + target - 1) / target;
    ck = ((ck + 127) / 128) * 128;
    if (ck < 128) ck = 128;
    const int chunks = (P + ck - 1) / ck;
    hipLaunchKernelGGL(cosine_kernel, dim3(chunks, Hkv, sgroups), dim3(256), 0, st,
                       (const uint16_t *)Kc, N, P, S, src, ck, E);
    return hipGetLastError();
}

}  // namespace gkv
