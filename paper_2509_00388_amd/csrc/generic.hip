// Scalar (non-MFMA) kernels for the two contractions of the pass, for any
// storage type and head dimension.  They serve fp32 inputs and shapes the MFMA
// kernels do not cover, and cross-check the MFMA kernels in the tests.  fp32
// fused multiply-adds, fp32 accumulation.
#include "common.hpp"
#include "kernels.hpp"

namespace gkv {

// dot(a, b) and, optionally, |b|^2 over d elements; d is a multiple of the
// 16-byte vector width.  a comes from LDS (already widened), b from global.
template <typename T>
__device__ __forceinline__ float dot_row(const float *__restrict__ a_f32, const T *__restrict__ b,
                                         int d, float *b_sq)
{
    constexpr int V = Elem<T>::kPerVec;
    const uint4 *bv = reinterpret_cast<const uint4 *>(b);
    float acc = 0.f, sq = 0.f;
    for (int c = 0; c < d / V; ++c) {
        float t[V];
        Elem<T>::unpack(bv[c], t);
#pragma unroll
        for (int u = 0; u < V; ++u) {
            acc = fmaf(a_f32[c * V + u], t[u], acc);
            sq = fmaf(t[u], t[u], sq);
        }
    }
    if (b_sq) *b_sq = sq;
    return acc;
}

// One workgroup per query row (q, r): logits over the visible keys, then the
// row's max and sum of exp.  Stage I, softmax statistics.
template <typename T>
__global__ __launch_bounds__(256) void generic_logits_kernel(
    const T *__restrict__ Kc, const T *__restrict__ Qw, int G, int d, int N, int w, float scale,
    float *__restrict__ logits, float *__restrict__ row_max, float *__restrict__ row_sum)
{
    __shared__ float q_f32[512];
    __shared__ float red[16];
    const int row = blockIdx.x;            // q * w + r
    const int q = row / w, r = row % w, h = q / G;
    const int P = N - w, visible = P + r + 1;
    for (int c = threadIdx.x; c < d; c += 256) {
        float t;
        if constexpr (sizeof(T) == 4) t = Qw[(long)row * d + c];
        else t = bf16_to_f32(Qw[(long)row * d + c]);
        q_f32[c] = t;
    }
    __syncthreads();
    const T *kh = Kc + (long)h * N * d;
    float *lrow = logits + (long)row * N;
    float mx = -INFINITY;
    for (int j = threadIdx.x; j < visible; j += 256) {
        const float l = dot_row<T>(q_f32, kh + (long)j * d, d, nullptr) * scale;
        lrow[j] = l;
        mx = fmaxf(mx, l);
    }
    mx = block_max(mx, red);
    float z = 0.f;
    for (int j = threadIdx.x; j < visible; j += 256) z += expf(lrow[j] - mx);
    z = block_sum(z, red);
    if (threadIdx.x == 0) { row_max[row] = mx; row_sum[row] = z; }
}

// votes[q, j] = sum over window rows r of exp(l_rj - max_r) / sum_r, j < P.
__global__ __launch_bounds__(256) void generic_votes_kernel(
    const float *__restrict__ logits, const float *__restrict__ row_max,
    const float *__restrict__ row_sum, int N, int w, float *__restrict__ votes)
{
    const int q = blockIdx.y, P = N - w;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= P) return;
    float acc = 0.f;
    for (int r = 0; r < w; ++r) {
        const int row = q * w + r;
        acc += expf(logits[(long)row * N + j] - row_max[row]) / row_sum[row];
    }
    votes[(long)q * P + j] = acc;
}

// Eq. 1 for source a of head h against prefix key j.  The source itself gets
// -inf so that it can never be its own neighbour (Eq. 3: j != i).
template <typename T>
__global__ __launch_bounds__(256) void generic_cosine_kernel(
    const T *__restrict__ Ac, const T *__restrict__ Kc, int d, int N, int P, int S,
    const int32_t *__restrict__ src, float *__restrict__ E)
{
    __shared__ float s_f32[512];
    const int a = blockIdx.y, h = blockIdx.z;
    const int i = src[h * S + a];
    const T *kh = Kc + (long)h * N * d, *ah = Ac + (long)h * N * d;   // source rows come from Ac
    float part = 0.f;
    for (int c = threadIdx.x; c < d; c += 256) {
        float t;
        if constexpr (sizeof(T) == 4) t = ah[(long)i * d + c];
        else t = bf16_to_f32(ah[(long)i * d + c]);
        s_f32[c] = t;
    }
    __syncthreads();
    // |k_i|^2 in a fixed order (every thread computes the same sum)
    for (int c = 0; c < d; ++c) part = fmaf(s_f32[c], s_f32[c], part);
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= P) return;
    float sq;
    const float dot = dot_row<T>(s_f32, kh + (long)j * d, d, &sq);
    float e;
    if (j == i) e = -INFINITY;
    else if (part == 0.f || sq == 0.f) e = 0.f;
    else e = dot * (1.0f / sqrtf(part)) * (1.0f / sqrtf(sq));
    E[((long)h * S + a) * P + j] = e;
}

template <typename T>
__global__ __launch_bounds__(256) void knorm_kernel(const T *__restrict__ Kc, int d, int N, int P,
                                                    float *__restrict__ scores)
{
    const int h = blockIdx.y, j = blockIdx.x * 256 + threadIdx.x;
    if (j >= P) return;
    constexpr int V = Elem<T>::kPerVec;
    const uint4 *bv = reinterpret_cast<const uint4 *>(Kc + ((long)h * N + j) * d);
    float sq = 0.f;
    for (int c = 0; c < d / V; ++c) {
        float t[V];
        Elem<T>::unpack(bv[c], t);
#pragma unroll
        for (int u = 0; u < V; ++u) sq = fmaf(t[u], t[u], sq);
    }
    scores[(long)h * P + j] = -sqrtf(sq);
}

hipError_t launch_generic_logits(const void *Kc, const void *Qw, int dtype, int Hkv, int Hq, int d,
                                 int N, int w, float scale, float *logits, float *row_max,
                                 float *row_sum, hipStream_t st)
{
    const int G = Hq / Hkv;
    if (dtype == 0)
        hipLaunchKernelGGL(generic_logits_kernel<float>, dim3(Hq * w), dim3(256), 0, st,
                           (const float *)Kc, (const float *)Qw, G, d, N, w, scale, logits, row_max,
                           row_sum);
    else
        hipLaunchKernelGGL(generic_logits_kernel<uint16_t>, dim3(Hq * w), dim3(256), 0, st,
                           (const uint16_t *)Kc, (const uint16_t *)Qw, G, d, N, w, scale, logits,
                           row_max, row_sum);
    return hipGetLastError();
}

hipError_t launch_generic_votes(const float *logits, const float *row_max, const float *row_sum,
                                int Hq, int N, int w, float *votes, hipStream_t st)
{
    const int P = N - w;
    hipLaunchKernelGGL(generic_votes_kernel, dim3((P + 255) / 256, Hq), dim3(256), 0, st, logits,
                       row_max, row_sum, N, w, votes);
    return hipGetLastError();
}

hipError_t launch_generic_cosine(const void *Ac, const void *Kc, int dtype, int Hkv, int d, int N, int P, int S,
                                 const int32_t *src, float *E, hipStream_t st)
{
    dim3 grid((P + 255) / 256, S, Hkv);
    if (dtype == 0)
        hipLaunchKernelGGL(generic_cosine_kernel<float>, grid, dim3(256), 0, st, (const float *)Ac,
                           (const float *)Kc, d, N, P, S, src, E);
    else
        hipLaunchKernelGGL(generic_cosine_kernel<uint16_t>, grid, dim3(256), 0, st,
                           (const uint16_t *)Ac, (const uint16_t *)Kc, d, N, P, S, src, E);
    return hipGetLastError();
}

hipError_t launch_knorm(const void *Kc, int dtype, int Hkv, int d, int N, int P, float *scores,
                        hipStream_t st)
{
    dim3 grid((P + 255) / 256, Hkv);
    if (dtype == 0)
        hipLaunchKernelGGL(knorm_kernel<float>, grid, dim3(256), 0, st, (const float *)Kc, d, N, P,
                           scores);
    else
        hipLaunchKernelGGL(knorm_kernel<uint16_t>, grid, dim3(256), 0, st, (const uint16_t *)Kc, d,
                           N, P, scores);
    return hipGetLastError();
}

}  // namespace gkv
