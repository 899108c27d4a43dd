// Device-side helpers shared by the GraphKV kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gkv {

constexpr int kWave = 64;

// Per-layer quantities of a batched call, passed to kernels by value.  A batch is
// a run of layers whose tensors are contiguous ([L, H, ...]), so every (layer,
// head) pair is simply head q = l * H + h of a layer with L*H heads; only the
// budget, and with it the place of a layer's rows in the packed outputs, varies.
constexpr int kMaxLayers = 64;
struct LayerPlan {
    int32_t heads_per_layer;          // H
    int32_t budget[kMaxLayers];       // B_l
    int64_t row_off[kMaxLayers];      // H * sum_{l' < l} B_l': first output row of layer l
};

// bfloat16 <-> float: bf16 is the upper half of an IEEE float, widening is exact.
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ float bf16lo_to_f32(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int kPerVec = 4;  // elements in a 16-byte vector
    __device__ static __forceinline__ void unpack(const uint4 &v, float *o) {
        o[0] = __uint_as_float(v.x); o[1] = __uint_as_float(v.y);
        o[2] = __uint_as_float(v.z); o[3] = __uint_as_float(v.w);
    }
};
template <> struct Elem<uint16_t> {
    static constexpr int kPerVec = 8;
    __device__ static __forceinline__ void unpack(const uint4 &v, float *o) {
        o[0] = bf16lo_to_f32(v.x); o[1] = bf16hi_to_f32(v.x);
        o[2] = bf16lo_to_f32(v.y); o[3] = bf16hi_to_f32(v.y);
        o[4] = bf16lo_to_f32(v.z); o[5] = bf16hi_to_f32(v.z);
        o[6] = bf16lo_to_f32(v.w); o[7] = bf16hi_to_f32(v.w);
    }
};

// Order-preserving map float -> uint32 (larger float <=> larger key).  -0.0 is
// folded onto +0.0 first so that the two compare equal, as they do as numbers.
__device__ __forceinline__ uint32_t ord_key(float f) {
    f = f + 0.0f;
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}
// Fixed butterfly order: the same inputs always give the same bits.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// Block-wide reductions for blocks of up to 1024 threads; `red` holds >= 16 floats.
__device__ __forceinline__ float block_max(float v, float *red) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    v = wave_max(v);
    __syncthreads();
    if (lane == 0) red[wv] = v;
    __syncthreads();
    float r = red[0];
    for (int i = 1; i < nw; ++i) r = fmaxf(r, red[i]);
    return r;
}
__device__ __forceinline__ float block_sum(float v, float *red) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    v = wave_sum(v);
    __syncthreads();
    if (lane == 0) red[wv] = v;
    __syncthreads();
    float r = red[0];
    for (int i = 1; i < nw; ++i) r += red[i];
    return r;
}

// The m-th largest of the keys in the first NIT registers of every lane (unused registers
// hold 0, below every key), all between kmin and kmax: built bit by bit from the top; the
// count of the keys that reach a trial value is one wave vote per register.  Straight-line
// code for a given NIT: branches between the votes would cost more than the votes.
template <int NIT, int R>
__device__ __forceinline__ uint32_t mth_largest_key(const uint32_t (&E)[R], uint32_t kmin, uint32_t kmax, int m)
{
    static_assert(NIT <= R, "");
    uint32_t tau = kmin;
    if (kmax > kmin) {
        for (int b = 31 - __clz(kmax - kmin); b >= 0; --b) {
            const uint32_t trial = tau + (1u << b);   // bits below b of tau - kmin are still 0
            int reach = 0;
#pragma unroll
            for (int it = 0; it < NIT; ++it) reach += (int)__popcll(__ballot(E[it] >= trial));
            if (trial > tau && reach >= m) tau = trial;   // (a trial that wrapped around is beyond every key)
        }
    }
    return tau;
}

}  // namespace gkv
