// Exact top-k of each row of a float matrix, ties to the lowest index, output in
// ascending index order.  Used for the source nodes (Eq. 2), the neighbourhoods
// (Eq. 3) and the final budgeted selection.
//
// One workgroup per row.  The k-th largest value is found by a most-significant-
// digit-first radix select over an order-preserving 32-bit key (4 passes of 8
// bits, integer histograms in LDS), which also tells how many entries equal to
// the threshold are still needed.  A last sweep emits, in index order, every
// entry above the threshold and the first `need` entries equal to it: that is
// exactly "first k by (value desc, index asc)".  All counting is integer, so the
// result does not depend on scheduling.
#include "common.hpp"
#include "kernels.hpp"

namespace gkv {

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void topk_rows_kernel(
    const float *__restrict__ x, long ld, int n, int k, int32_t *__restrict__ idx_out, long idx_ld,
    float *__restrict__ val_out, long val_ld, int append_from, int append_count)
{
    constexpr int NW = BLOCK / kWave;
    __shared__ uint32_t hist[256];
    __shared__ uint32_t s_bin, s_need;
    __shared__ uint32_t w_gt[NW], w_eq[NW];

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const float *xr = x + (long)blockIdx.x * ld;
    int32_t *out = idx_out + (long)blockIdx.x * idx_ld;
    float *vout = val_out ? val_out + (long)blockIdx.x * val_ld : nullptr;

    for (int r = tid; r < append_count; r += BLOCK) out[k + r] = append_from + r;
    if (k <= 0) return;

    uint32_t prefix = 0, mask = 0, need = (uint32_t)k;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for (int j0 = 0; j0 < n; j0 += BLOCK) {
            const int j = j0 + tid;
            const bool live = j < n;
            const uint32_t key = live ? ord_key(xr[j]) : 0u;
            const bool in = live && ((key & mask) == prefix);
            const uint32_t dig = (key >> shift) & 255u;
            // Same digit in the whole wave (common in the top pass): one add.
            const uint64_t act = __ballot(in);
            if (act) {
                const int first = __ffsll((long long)act) - 1;
                const uint32_t d0 = __shfl(dig, first, kWave);
                const uint64_t same = __ballot(in && dig == d0);
                if (same == act) {
                    if (lane == first) atomicAdd(&hist[d0], (uint32_t)__popcll(act));
                } else if (in) {
                    atomicAdd(&hist[dig], 1u);
                }
            }
        }
        __syncthreads();
        if (wv == 0) {
            // bins 4*lane .. 4*lane+3; suffix sums over higher lanes
            const uint32_t c0 = hist[4 * lane], c1 = hist[4 * lane + 1], c2 = hist[4 * lane + 2],
                           c3 = hist[4 * lane + 3];
            const uint32_t t = c0 + c1 + c2 + c3;
            uint32_t incl = t;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t v = __shfl_down(incl, o, kWave);
                if (lane + o < 64) incl += v;
            }
            const uint32_t excl = incl - t;            // entries in strictly higher lanes
            if (excl < need && need <= incl) {
                uint32_t cum = excl, bin, c[4] = {c0, c1, c2, c3};
                int b = 3;
                for (; b > 0; --b) {
                    if (cum + c[b] >= need) break;
                    cum += c[b];
                }
                bin = 4 * lane + b;
                s_bin = bin;
                s_need = need - cum;
            }
        }
        __syncthreads();
        prefix |= s_bin << shift;
        mask |= 255u << shift;
        need = s_need;
        __syncthreads();
    }
    const uint32_t tau = prefix;   // key of the k-th largest entry; take `need` entries equal to it

    // Each wave owns a contiguous, 64-aligned segment of the row.
    int seg = (n + NW - 1) / NW;
    seg = (seg + 63) & ~63;
    const int beg = wv * seg;
    const int end = min(n, beg + seg);

    uint32_t cg = 0, ce = 0;
    for (int j0 = beg; j0 < end; j0 += kWave) {
        const int j = j0 + lane;
        const uint32_t key = (j < end) ? ord_key(xr[j]) : 0u;
        cg += __popcll(__ballot(j < end && key > tau));
        ce += __popcll(__ballot(j < end && key == tau));
    }
    if (lane == 0) { w_gt[wv] = cg; w_eq[wv] = ce; }
    __syncthreads();
    uint32_t base_g = 0, base_e = 0;
    for (int i = 0; i < wv; ++i) { base_g += w_gt[i]; base_e += w_eq[i]; }

    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    for (int j0 = beg; j0 < end; j0 += kWave) {
        const int j = j0 + lane;
        const bool live = j < end;
        const float v = live ? xr[j] : 0.0f;
        const uint32_t key = live ? ord_key(v) : 0u;
        const bool g = live && key > tau, e = live && key == tau;
        const uint64_t mg = __ballot(g), me = __ballot(e);
        const uint32_t g_before = base_g + __popcll(mg & lt_mask);
        const uint32_t e_before = base_e + __popcll(me & lt_mask);
        if (g || (e && e_before < need)) {
            const uint32_t pos = g_before + min(e_before, need);
            out[pos] = j;
            if (vout) vout[pos] = v;
        }
        base_g += __popcll(mg);
        base_e += __popcll(me);
    }
}

hipError_t launch_topk_rows(const float *x, long ld, int n, int rows, int k, int32_t *idx_out,
                            long idx_ld, float *val_out, long val_ld, int append_from,
                            int append_count, hipStream_t st)
{
    if (rows <= 0) return hipSuccess;
    if (n >= 4096) {
        hipLaunchKernelGGL(topk_rows_kernel<1024>, dim3(rows), dim3(1024), 0, st, x, ld, n, k,
                           idx_out, idx_ld, val_out, val_ld, append_from, append_count);
    } else {
        hipLaunchKernelGGL(topk_rows_kernel<256>, dim3(rows), dim3(256), 0, st, x, ld, n, k,
                           idx_out, idx_ld, val_out, val_ld, append_from, append_count);
    }
    return hipGetLastError();
}

}  // namespace gkv
