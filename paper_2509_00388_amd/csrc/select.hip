// Exact top-k of each row of a float matrix, ties to the lowest index, output in
// ascending index order.  Used for the source nodes (Eq. 2), the neighbourhoods
// (Eq. 3) and the final budgeted selection.
//
// One workgroup per row.  The k-th largest value is found by a most-significant-
// digit-first radix select over an order-preserving 32-bit key (digits of 11,
// 11 and 10 bits, integer histograms in LDS), which also tells how many entries
// equal to the threshold are still needed.  A last sweep emits, in index order,
// every entry above the threshold and the first `need` entries equal to it:
// that is exactly "first k by (value desc, index asc)".  All counting is
// integer, so the result does not depend on scheduling.
//
// Rows of up to 32768 entries are read once, coalesced, and kept in LDS for all
// sweeps; longer rows are re-read from L2 in every sweep.
#include "common.hpp"
#include "kernels.hpp"

#include <type_traits>

namespace gkv {

namespace {

constexpr int kBins = 2048;   // bins of the streaming variant (11-bit digits)

__device__ __forceinline__ float key_to_float(uint32_t key)   // inverse of ord_key
{
    return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}

// Histogram one digit of the keys that still match the prefix.  `in` says
// whether this lane's key takes part.  A wave whose keys all share the digit
// (usual in the top digit) issues a single add.
__device__ __forceinline__ void hist_add(uint32_t *hist, bool in, uint32_t dig, int lane)
{
    const uint64_t act = __ballot(in);
    if (!act) return;
    const int first = __ffsll((long long)act) - 1;
    const uint32_t d0 = __shfl(dig, first, kWave);
    const uint64_t same = __ballot(in && dig == d0);
    if (same == act) {
        if (lane == first) atomicAdd(&hist[d0], (uint32_t)__popcll(act));
    } else if (in) {
        atomicAdd(&hist[dig], 1u);
    }
}

// Wave 0: find the bin where the count of larger-or-equal digits reaches `need`.
// Lane L owns bins BPL*L .. BPL*L+BPL-1 (64*BPL bins in all).  Writes
// {bin, need - (entries in higher bins)}.
template <int BPL>
__device__ __forceinline__ void find_bin(const uint32_t *hist, uint32_t need, int lane,
                                         uint32_t *s_bin, uint32_t *s_need)
{
    uint32_t t = 0;
#pragma unroll
    for (int b = 0; b < BPL; ++b) t += hist[BPL * lane + b];
    uint32_t incl = t;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t v = __shfl_down(incl, o, kWave);
        if (lane + o < 64) incl += v;
    }
    const uint32_t excl = incl - t;   // entries in strictly higher lanes
    if (excl < need && need <= incl) {
        uint32_t cum = excl;
        int b = BPL - 1;
        for (; b > 0; --b) {
            const uint32_t c = hist[BPL * lane + b];
            if (cum + c >= need) break;
            cum += c;
        }
        *s_bin = BPL * lane + b;
        *s_need = need - cum;
    }
}

}  // namespace

// ---- rows kept in LDS ---------------------------------------------------------
// The row is read once, coalesced, and its keys stay in LDS (up to 32768 entries
// = 128 KiB) for all sweeps.  Thread t handles entries i*BLOCK + t; index order is
// therefore (i, wave, lane), and the emit sweep counts per (i, wave) cell with
// ballots and scans the cells once.
// DIG = bits per radix sweep (11 for long rows, 8 for short ones: fewer bins to clear
// and scan).
template <int BLOCK, bool PLAN, int DIG>
__device__ __forceinline__ void topk_row_lds(
    int row, const float *__restrict__ x, long ld, int n, int k, int32_t *__restrict__ idx_out,
    long idx_ld, float *__restrict__ val_out, long val_ld, float *__restrict__ tau_out,
    int append_from, int append_count,
    const typename std::conditional<PLAN, LayerPlan, int>::type &plan)
{
    constexpr int NW = BLOCK / kWave;
    constexpr int NBINS = 1 << DIG;
    extern __shared__ uint32_t dyn[];
    __shared__ uint32_t hist[NBINS];
    __shared__ uint32_t s_bin, s_need;

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int items = (n + BLOCK - 1) / BLOCK;
    const int ncell = items * NW;
    uint32_t *keys = dyn;                    // [items * BLOCK]
    uint32_t *cg = dyn + items * BLOCK;      // [ncell]
    uint32_t *ce = cg + ncell;               // [ncell]
    const float *xr = x + (long)row * ld;
    int32_t *out = idx_out ? idx_out + (long)row * idx_ld : nullptr;
    float *vout = val_out ? val_out + (long)row * val_ld : nullptr;
    if constexpr (PLAN) {   // per-layer budget: k and the output row come from the plan
        const int g = row / plan.heads_per_layer, hl = row % plan.heads_per_layer;
        k = plan.budget[g] - append_count;
        out = idx_out + (plan.row_off[g] + (long)hl * plan.budget[g]);
    }

    if (out)
        for (int r = tid; r < append_count; r += BLOCK) out[k + r] = append_from + r;
    if (k <= 0) return;

    // Keys to LDS; the row's key range [kmin, kmax] on the way.
    __shared__ uint32_t s_min[NW], s_max[NW];
    uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll 8
    for (int i = 0; i < items; ++i) {
        const int j = i * BLOCK + tid;
        const uint32_t key = ord_key(j < n ? xr[j] : 0.f);
        keys[j] = key;
        if (j < n) { kmin = min(kmin, key); kmax = max(kmax, key); }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, o, kWave));
        kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o, kWave));
    }
    if (lane == 0) { s_min[wv] = kmin; s_max[wv] = kmax; }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < NW; ++u) { kmin = min(kmin, s_min[u]); kmax = max(kmax, s_max[u]); }

    // Radix select on (key - kmin): only the bits in which the row's keys differ
    // are swept, and the top digit is spread over the bins whatever the value range.
    const uint32_t range = kmax - kmin;
    int remaining = range ? 32 - __clz(range) : 0;
    uint32_t prefix = 0, mask = 0, need = (uint32_t)k;
    while (remaining > 0) {
        const int bits = remaining < DIG ? remaining : DIG;
        const int shift = remaining - bits;
        const uint32_t dmask = (1u << bits) - 1u;
        for (int b = tid; b < NBINS; b += BLOCK) hist[b] = 0;
        __syncthreads();
        for (int i = 0; i < items; ++i) {
            const int j = i * BLOCK + tid;
            const uint32_t rel = keys[j] - kmin;
            if (j < n && (rel & mask) == prefix) atomicAdd(&hist[(rel >> shift) & dmask], 1u);
        }
        __syncthreads();
        if (wv == 0) find_bin<NBINS / 64>(hist, need, lane, &s_bin, &s_need);
        __syncthreads();
        prefix |= s_bin << shift;
        mask |= dmask << shift;
        need = s_need;
        remaining = shift;
    }
    const uint32_t tau = kmin + prefix;   // key of the k-th largest entry; take `need` entries equal to it
    if (tau_out && tid == 0) tau_out[row] = key_to_float(tau);
    if (!out) return;


    for (int i = 0; i < items; ++i) {
        const int j = i * BLOCK + tid;
        const uint32_t key = keys[j];
        const uint32_t ng = __popcll(__ballot(j < n && key > tau));
        const uint32_t ne = __popcll(__ballot(j < n && key == tau));
        if (lane == 0) { cg[i * NW + wv] = ng; ce[i * NW + wv] = ne; }
    }
    __syncthreads();
    if (wv == 0) {   // exclusive scan of the cells in index order; lane L owns a contiguous run
        const int per = (ncell + 63) / 64;
        const int c0 = min(lane * per, ncell), c1 = min(c0 + per, ncell);
        uint32_t sg = 0, se = 0;
        for (int c = c0; c < c1; ++c) { sg += cg[c]; se += ce[c]; }
        uint32_t ig = sg, ie = se;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t a = __shfl_up(ig, o, kWave), b = __shfl_up(ie, o, kWave);
            if (lane >= o) { ig += a; ie += b; }
        }
        uint32_t bg = ig - sg, be = ie - se;
        for (int c = c0; c < c1; ++c) {
            const uint32_t tg = cg[c], te = ce[c];
            cg[c] = bg; ce[c] = be;
            bg += tg; be += te;
        }
    }
    __syncthreads();
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));

    for (int i = 0; i < items; ++i) {
        const int j = i * BLOCK + tid;
        const uint32_t key = keys[j];
        const bool g = j < n && key > tau, e = j < n && key == tau;
        const uint64_t mg = __ballot(g), me = __ballot(e);
        if (g || e) {
            const uint32_t g_before = cg[i * NW + wv] + __popcll(mg & lt_mask);
            const uint32_t e_before = ce[i * NW + wv] + __popcll(me & lt_mask);
            if (g || e_before < need) {
                const uint32_t pos = g_before + min(e_before, need);
                out[pos] = j;
                if (vout) vout[pos] = key_to_float(key);
            }
        }
    }
}

// One workgroup per row (WALK = false); with a gate, a smaller grid whose workgroups walk
// the rows and skip those whose gate is 0 (WALK = true: a launch that mostly skips then
// costs next to nothing).
template <int BLOCK, bool PLAN, int DIG, bool WALK>
__global__ __launch_bounds__(BLOCK) void topk_rows_lds_kernel(
    const float *__restrict__ x, long ld, int n, int rows, int k, int32_t *__restrict__ idx_out,
    long idx_ld, float *__restrict__ val_out, long val_ld, float *__restrict__ tau_out,
    int append_from, int append_count, const int32_t *__restrict__ gate, int rows_per_gate,
    typename std::conditional<PLAN, LayerPlan, int>::type plan)
{
    if constexpr (WALK) {
        // one round trip settles the usual case of no gate being set at all
        int any = 0;
        for (int g = threadIdx.x; g < (rows + rows_per_gate - 1) / rows_per_gate; g += BLOCK)
            any |= gate[g];
        if (!__syncthreads_or(any)) return;
        for (int row = blockIdx.x; row < rows; row += gridDim.x) {
            if (gate[row / rows_per_gate] == 0) continue;
            __syncthreads();   // LDS is reused from row to row
            topk_row_lds<BLOCK, PLAN, DIG>(row, x, ld, n, k, idx_out, idx_ld, val_out, val_ld, tau_out,
                                           append_from, append_count, plan);
        }
    } else {
        topk_row_lds<BLOCK, PLAN, DIG>(blockIdx.x, x, ld, n, k, idx_out, idx_ld, val_out, val_ld,
                                       tau_out, append_from, append_count, plan);
    }
}

// ---- small k out of a long row ------------------------------------------------
// For k far below the row length (the source nodes: 64 of 32736) the keys need not
// go through LDS at all.  Every thread keeps its keys (32 with 1024 threads; 512
// threads measured slower) in registers.  A bound comes almost for free: split the threads into G >= k groups; the smallest
// of the G group maxima is reached by G different entries, so the k-th largest key
// is at least that.  Only the few hundred keys that reach the bound take part in
// the radix select (the same sweeps as above, fed from registers: a compare per key
// and an LDS atomic for the few that pass), and the emit sweep is the one above.
constexpr int kSmallK = 256;       // largest k this path takes

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void topk_rows_smallk_kernel(
    const float *__restrict__ x, long ld, int n, int k, int32_t *__restrict__ idx_out, long idx_ld)
{
    constexpr int ITEMS = 32768 / BLOCK, NW = BLOCK / kWave, DIG = 11, NBINS = 1 << DIG;
    __shared__ uint32_t hist[NBINS];
    __shared__ uint32_t s_bin, s_need, s_grp[kSmallK], s_bound, s_wmax[NW], s_max;
    __shared__ uint32_t cg[ITEMS * NW], ce[ITEMS * NW];
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const float *xr = x + (long)row * ld;
    int32_t *out = idx_out + (long)row * idx_ld;

    uint32_t key[ITEMS];
    uint32_t best = 0;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int j = i * BLOCK + tid;
        key[i] = j < n ? ord_key(xr[j]) : 0u;          // 0 is below the key of every number
        best = max(best, key[i]);
    }
    // G groups of consecutive threads (G a power of two, k <= G <= 256, so a group is 4 to 64
    // lanes of one wave): group maxima, their minimum = the bound; the row maximum on the way.
    int G = 16;
    while (G < k) G <<= 1;
    const int gs = BLOCK / G;
    uint32_t gmax = best;
    for (int o = 1; o < gs; o <<= 1) gmax = max(gmax, (uint32_t)__shfl_xor((int)gmax, o, kWave));
    if ((tid & (gs - 1)) == 0) s_grp[tid / gs] = gmax;
    uint32_t wmax = best;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) wmax = max(wmax, (uint32_t)__shfl_xor((int)wmax, o, kWave));
    if (lane == 0) s_wmax[wv] = wmax;
    __syncthreads();
    if (wv == 0) {
        uint32_t mn = 0xffffffffu, mx = 0u;
        for (int g = lane; g < G; g += kWave) mn = min(mn, s_grp[g]);
        if (lane < NW) mx = s_wmax[lane];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            mn = min(mn, (uint32_t)__shfl_xor((int)mn, o, kWave));
            mx = max(mx, (uint32_t)__shfl_xor((int)mx, o, kWave));
        }
        if (lane == 0) { s_bound = mn; s_max = mx; }
    }
    __syncthreads();
    const uint32_t kmin = s_bound, kmax = s_max;

    // radix select on (key - bound) among the keys that reach the bound
    const uint32_t range = kmax - kmin;
    int remaining = range ? 32 - __clz(range) : 0;
    uint32_t prefix = 0, mask = 0, need = (uint32_t)k;
    while (remaining > 0) {
        const int bits = remaining < DIG ? remaining : DIG;
        const int shift = remaining - bits;
        const uint32_t dmask = (1u << bits) - 1u;
        for (int b = tid; b < NBINS; b += BLOCK) hist[b] = 0;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const uint32_t rel = key[i] - kmin;
            if (key[i] >= kmin && (rel & mask) == prefix) atomicAdd(&hist[(rel >> shift) & dmask], 1u);
        }
        __syncthreads();
        if (wv == 0) find_bin<NBINS / 64>(hist, need, lane, &s_bin, &s_need);
        __syncthreads();
        prefix |= s_bin << shift;
        mask |= dmask << shift;
        need = s_need;
        remaining = shift;
    }
    const uint32_t tau = kmin + prefix;   // key of the k-th largest entry; take `need` entries equal to it

    // emit in index order: entries above tau and the first `need` entries equal to it
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const uint32_t ng = __popcll(__ballot(key[i] > tau));
        const uint32_t ne = __popcll(__ballot(key[i] == tau));
        if (lane == 0) { cg[i * NW + wv] = ng; ce[i * NW + wv] = ne; }
    }
    __syncthreads();
    if (wv == 0) {   // exclusive scan of the cells in index order; lane L owns a contiguous run
        constexpr int per = ITEMS * NW / 64;
        const int c0 = lane * per;
        uint32_t sg = 0, se = 0;
#pragma unroll
        for (int c = 0; c < per; ++c) { sg += cg[c0 + c]; se += ce[c0 + c]; }
        uint32_t ig = sg, ie = se;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t a = __shfl_up(ig, o, kWave), b = __shfl_up(ie, o, kWave);
            if (lane >= o) { ig += a; ie += b; }
        }
        uint32_t bg = ig - sg, be = ie - se;
#pragma unroll
        for (int c = 0; c < per; ++c) {
            const uint32_t tg = cg[c0 + c], te = ce[c0 + c];
            cg[c0 + c] = bg; ce[c0 + c] = be;
            bg += tg; be += te;
        }
    }
    __syncthreads();
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const bool g = key[i] > tau, e = key[i] == tau;   // keys of entries past n are 0 < tau
        const uint64_t mg = __ballot(g), me = __ballot(e);
        if (g || e) {
            const uint32_t g_before = cg[i * NW + wv] + __popcll(mg & lt_mask);
            const uint32_t e_before = ce[i * NW + wv] + __popcll(me & lt_mask);
            if (g || e_before < need) out[g_before + min(e_before, need)] = i * BLOCK + tid;
        }
    }
}

// ---- rows of any length: every sweep re-reads the row ------------------------
template <int BLOCK, bool PLAN>
__device__ __forceinline__ void topk_stream_row(
    int row, const float *__restrict__ x, long ld, int n, int k, int32_t *__restrict__ idx_out, long idx_ld,
    float *__restrict__ val_out, long val_ld, float *__restrict__ tau_out, int append_from,
    int append_count, const int32_t *__restrict__ gate, int rows_per_gate,
    typename std::conditional<PLAN, LayerPlan, int>::type plan)
{
    constexpr int NW = BLOCK / kWave;
    constexpr int U = 8;   // loads in flight per thread
    __shared__ uint32_t hist[kBins];
    __shared__ uint32_t s_bin, s_need;
    __shared__ uint32_t w_gt[NW], w_eq[NW];

    if (gate && gate[row / rows_per_gate] == 0) return;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const float *xr = x + (long)row * ld;
    int32_t *out = idx_out ? idx_out + (long)row * idx_ld : nullptr;
    float *vout = val_out ? val_out + (long)row * val_ld : nullptr;
    if constexpr (PLAN) {   // per-layer budget: k and the output row come from the plan
        const int g = row / plan.heads_per_layer, hl = row % plan.heads_per_layer;
        k = plan.budget[g] - append_count;
        out = idx_out + (plan.row_off[g] + (long)hl * plan.budget[g]);
    }

    if (out)
        for (int r = tid; r < append_count; r += BLOCK) out[k + r] = append_from + r;
    if (k <= 0) return;

    uint32_t prefix = 0, mask = 0, need = (uint32_t)k;
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
        const uint32_t dmask = pass == 2 ? 1023u : 2047u;
        for (int b = tid; b < kBins; b += BLOCK) hist[b] = 0;
        __syncthreads();
        for (int j0 = 0; j0 < n; j0 += BLOCK * U) {
            float t[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int j = j0 + u * BLOCK + tid;
                t[u] = j < n ? xr[j] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t key = ord_key(t[u]);
                const bool in = (j0 + u * BLOCK + tid < n) && ((key & mask) == prefix);
                hist_add(hist, in, (key >> shift) & dmask, lane);
            }
        }
        __syncthreads();
        if (wv == 0) find_bin<32>(hist, need, lane, &s_bin, &s_need);
        __syncthreads();
        prefix |= s_bin << shift;
        mask |= dmask << shift;
        need = s_need;
    }
    const uint32_t tau = prefix;
    if (tau_out && tid == 0) tau_out[row] = key_to_float(tau);
    if (!out) return;

    // Each wave owns a contiguous, 64-aligned segment of the row.
    int seg = (n + NW - 1) / NW;
    seg = (seg + 63) & ~63;
    const int beg = wv * seg;
    const int end = min(n, beg + seg);

    uint32_t cgt = 0, ceq = 0;
    for (int j0 = beg; j0 < end; j0 += kWave * U) {
        float t[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + u * kWave + lane;
            t[u] = j < end ? xr[j] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + u * kWave + lane;
            const uint32_t key = ord_key(t[u]);
            cgt += __popcll(__ballot(j < end && key > tau));
            ceq += __popcll(__ballot(j < end && key == tau));
        }
    }
    if (lane == 0) { w_gt[wv] = cgt; w_eq[wv] = ceq; }
    __syncthreads();
    uint32_t base_g = 0, base_e = 0;
    for (int i = 0; i < wv; ++i) { base_g += w_gt[i]; base_e += w_eq[i]; }

    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    for (int j0 = beg; j0 < end; j0 += kWave * U) {
        float t[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + u * kWave + lane;
            t[u] = j < end ? xr[j] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + u * kWave + lane;
            const bool live = j < end;
            const uint32_t key = ord_key(t[u]);
            const bool g = live && key > tau, e = live && key == tau;
            const uint64_t mg = __ballot(g), me = __ballot(e);
            const uint32_t g_before = base_g + __popcll(mg & lt_mask);
            const uint32_t e_before = base_e + __popcll(me & lt_mask);
            if (g || (e && e_before < need)) {
                const uint32_t pos = g_before + min(e_before, need);
                out[pos] = j;
                if (vout) vout[pos] = t[u];
            }
            base_g += __popcll(mg);
            base_e += __popcll(me);
        }
    }
}

template <int BLOCK, bool PLAN>
__global__ __launch_bounds__(BLOCK) void topk_rows_stream_kernel(
    const float *__restrict__ x, long ld, int n, int rows, int k, int32_t *__restrict__ idx_out, long idx_ld,
    float *__restrict__ val_out, long val_ld, float *__restrict__ tau_out, int append_from,
    int append_count, const int32_t *__restrict__ gate, int rows_per_gate,
    typename std::conditional<PLAN, LayerPlan, int>::type plan)
{
    // (a gated launch has few workgroups that walk the rows; usually no gate is open at all)
    if (gate) {
        const int n_gates = (rows + rows_per_gate - 1) / rows_per_gate;
        int open = 0;
        for (int g = threadIdx.x; g < n_gates; g += BLOCK) open |= gate[g] != 0;
        if (!__syncthreads_or(open)) return;
    }
    for (int row = blockIdx.x; row < rows; row += gridDim.x) {
        topk_stream_row<BLOCK, PLAN>(row, x, ld, n, k, idx_out, idx_ld, val_out, val_ld, tau_out, append_from,
                                     append_count, gate, rows_per_gate, plan);
        __syncthreads();
    }
}

// Long rows, few winners (k <= kSmallK <= BLOCK): two reads of the row instead of five.
// Every thread takes the maximum of the elements it owns; the k-th largest of those maxima is
// a lower bound of the row's k-th largest element (k different elements reach it).  The second
// read collects the few elements that reach the bound into an LDS list, and the exact select
// (radix select over the list, ties at the cut to the lowest indices, winners ranked by index)
// runs on that list.  A row with more than kLongCap elements at or above the bound (masses of
// equal values) goes through the five-read algorithm instead.
constexpr int kLongCap = 4096;

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void topk_rows_long_smallk_kernel(
    const float *__restrict__ x, long ld, int n, int k, int32_t *__restrict__ idx_out, long idx_ld)
{
    constexpr int NW = BLOCK / kWave, U = 8;
    __shared__ uint32_t lk[kLongCap], lj[kLongCap];   // keys and indices of the candidates
    __shared__ uint32_t tmax[BLOCK];
    __shared__ uint64_t win[kSmallK];                 // (index << 32) | key of the winners
    __shared__ uint32_t hist8[256];
    __shared__ uint32_t s_cnt, s_bin, s_need, s_wmax[NW], s_wmin[NW];
    __shared__ int32_t n_win, n_eq;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const float *xr = x + (long)blockIdx.x * ld;
    int32_t *out = idx_out + (long)blockIdx.x * idx_ld;

    // first read: the largest key each thread owns (0 is below the key of every number)
    uint32_t mx = 0u;
    for (int j0 = 0; j0 < n; j0 += BLOCK * U) {
        float t[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + u * BLOCK + tid;
            t[u] = j < n ? xr[j] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (j0 + u * BLOCK + tid < n) mx = max(mx, ord_key(t[u]));
    }
    tmax[tid] = mx;
    uint32_t wmax = mx, wmin = mx;   // the largest and the smallest of the maxima
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        wmax = max(wmax, (uint32_t)__shfl_xor((int)wmax, o, kWave));
        wmin = min(wmin, (uint32_t)__shfl_xor((int)wmin, o, kWave));
    }
    if (lane == 0) { s_wmax[wv] = wmax; s_wmin[wv] = wmin; }
    if (tid == 0) { s_cnt = 0; n_win = 0; n_eq = 0; }
    __syncthreads();
    uint32_t kmax = 0u, kmin = 0xffffffffu;
#pragma unroll
    for (int u = 0; u < NW; ++u) { kmax = max(kmax, s_wmax[u]); kmin = min(kmin, s_wmin[u]); }

    // The want-th largest of arr[0 .. count), all keys in [lo, kmax]: radix select over key - lo,
    // 8 bits a sweep from the top bit in which the keys can differ.  Returns the key and leaves
    // in `left` how many entries equal to it are among the want largest.
    auto kth_largest = [&](const uint32_t *arr, int count, uint32_t lo, int want, uint32_t &left) {
        int remaining = kmax > lo ? 32 - __clz(kmax - lo) : 0;
        uint32_t prefix = 0, mask = 0, need = (uint32_t)want;
        while (remaining > 0) {
            const int bits = remaining < 8 ? remaining : 8;
            const int shift = remaining - bits;
            const uint32_t dmask = (1u << bits) - 1u;
            if (tid < 256) hist8[tid] = 0;
            __syncthreads();
            for (int r = tid; r < count; r += BLOCK) {
                const uint32_t rel = arr[r] - lo;
                if ((rel & mask) == prefix) atomicAdd(&hist8[(rel >> shift) & dmask], 1u);
            }
            __syncthreads();
            if (wv == 0) find_bin<4>(hist8, need, lane, &s_bin, &s_need);
            __syncthreads();
            prefix |= s_bin << shift;
            mask |= dmask << shift;
            need = s_need;
            remaining = shift;
        }
        left = need;
        return lo + prefix;
    };
    uint32_t unused;
    const uint32_t bound = kth_largest(tmax, BLOCK, kmin, k, unused);

    // second read: everything that reaches the bound goes to the list
    for (int j0 = 0; j0 < n; j0 += BLOCK * U) {
        float t[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + u * BLOCK + tid;
            t[u] = j < n ? xr[j] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + u * BLOCK + tid;
            const uint32_t key = ord_key(t[u]);
            if (j < n && key >= bound) {
                const uint32_t at = atomicAdd(&s_cnt, 1u);
                if (at < (uint32_t)kLongCap) { lk[at] = key; lj[at] = (uint32_t)j; }
            }
        }
    }
    __syncthreads();
    const int cnt = (int)s_cnt;
    if (cnt > kLongCap) {   // (the same for every thread)
        topk_stream_row<BLOCK, false>(blockIdx.x, x, ld, n, k, idx_out, idx_ld, nullptr, 0, nullptr, 0, 0, nullptr,
                                      1, 0);
        return;
    }

    uint32_t need;
    const uint32_t tau = kth_largest(lk, cnt, bound, k, need);
    // winners above tau; of the entries equal to tau the `need` lowest indices
    for (int r = tid; r < cnt; r += BLOCK) {
        const uint32_t key = lk[r];
        if (key > tau) win[atomicAdd(&n_win, 1)] = ((uint64_t)lj[r] << 32) | key;
        else if (key == tau) atomicAdd(&n_eq, 1);
    }
    __syncthreads();
    const int ne = n_eq, base = n_win;
    __syncthreads();
    for (int r = tid; r < cnt; r += BLOCK) {
        if (lk[r] == tau) {
            const uint32_t mine = lj[r];
            if (ne == (int)need) {
                win[atomicAdd(&n_win, 1)] = ((uint64_t)mine << 32) | tau;
            } else {
                uint32_t rank = 0;
                for (int u = 0; u < cnt; ++u) rank += (lk[u] == tau) & (lj[u] < mine);
                if (rank < need) win[base + rank] = ((uint64_t)mine << 32) | tau;
            }
        }
    }
    __syncthreads();
    for (int r = tid; r < k; r += BLOCK) {   // ascending index order
        const uint64_t mine = win[r];
        int pos = 0;
        for (int u = 0; u < k; ++u) pos += win[u] < mine;
        out[pos] = (int32_t)(mine >> 32);
    }
}

// ---- neighbourhoods of heads whose candidate lists overflowed ------------------------
// The filter route (mfma_cosine.hip) gives up on a head when a candidate list cannot hold what
// reaches the bound (masses of equal edges, an adversarial key order) and raises the head's
// flag.  Such heads are rare, so they are not worth an [heads, S, P] edge block in memory: a
// fixed number of workgroups walk the (head, source) rows of the flagged heads, and each row's
// edges (Eq. 1, scalar fused multiply-adds over the bf16 rows, d = 128) go to the workgroup's
// own scratch row of P floats, out of which the exact top-m (Eq. 3) is taken by the row
// kernels above.  A launch that finds no flag set returns after one round trip.
constexpr int kRedoBlock = 1024;
constexpr int kRedoDim = 128;

__global__ __launch_bounds__(kRedoBlock) void redo_rows_kernel(
    const uint16_t *__restrict__ Ac, const uint16_t *__restrict__ Kc, int N, int P, int S, int m, int heads,
    const int32_t *__restrict__ src, const int32_t *__restrict__ overflow, float *__restrict__ rows,
    int32_t *__restrict__ nbr, float *__restrict__ nbr_e)
{
    __shared__ float s_f32[kRedoDim];
    const int tid = threadIdx.x;
    int open = 0;
    for (int g = tid; g < heads; g += kRedoBlock) open |= overflow[g] != 0;
    if (!__syncthreads_or(open)) return;
    float *erow = rows + (long)blockIdx.x * P;
    for (long item = blockIdx.x; item < (long)heads * S; item += gridDim.x) {
        const int h = (int)(item / S);
        if (overflow[h] == 0) continue;           // (the same for every thread)
        const int32_t i = src[item];
        const uint16_t *ah = Ac + (long)h * N * kRedoDim, *kh = Kc + (long)h * N * kRedoDim;
        __syncthreads();                          // the previous row's LDS and scratch row are free
        if (tid < kRedoDim) s_f32[tid] = bf16_to_f32(ah[(long)i * kRedoDim + tid]);
        __syncthreads();
        float sq_i = 0.f;                         // |x_i|^2 in a fixed order, the same in every thread
        for (int c = 0; c < kRedoDim; ++c) sq_i = fmaf(s_f32[c], s_f32[c], sq_i);
        const float inv_i = sq_i == 0.f ? 0.f : __builtin_amdgcn_rsqf(sq_i);
        for (int j = tid; j < P; j += kRedoBlock) {
            const uint4 *kv = reinterpret_cast<const uint4 *>(kh + (long)j * kRedoDim);
            float dot = 0.f, sq = 0.f;
#pragma unroll 4
            for (int c = 0; c < kRedoDim / 8; ++c) {
                float t[8];
                Elem<uint16_t>::unpack(kv[c], t);
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    dot = fmaf(s_f32[c * 8 + u], t[u], dot);
                    sq = fmaf(t[u], t[u], sq);
                }
            }
            const float inv_k = sq == 0.f ? 0.f : __builtin_amdgcn_rsqf(sq);
            erow[j] = j == i ? -INFINITY : (dot * inv_k) * inv_i;   // (Eq. 3: j != i; a zero row has e = 0)
        }
        __syncthreads();                          // the row is complete and visible to the workgroup
        int32_t *out = nbr + item * m;
        float *vout = nbr_e + item * m;
        if (P <= 32768)
            topk_row_lds<kRedoBlock, false, 11>(0, erow, P, P, m, out, 0, vout, 0, nullptr, 0, 0, 0);
        else
            topk_stream_row<kRedoBlock, false>(0, erow, P, P, m, out, 0, vout, 0, nullptr, 0, 0, nullptr, 1, 0);
    }
}

template <int BLOCK, bool PLAN, int DIG, typename PlanArg>
static hipError_t launch_lds(const float *x, long ld, int n, int rows, int k, int32_t *idx_out,
                             long idx_ld, float *val_out, long val_ld, float *tau_out,
                             int append_from, int append_count, const int32_t *gate,
                             int rows_per_gate, PlanArg plan, hipStream_t st)
{
    const int items = (n + BLOCK - 1) / BLOCK;
    const size_t lds = ((size_t)items * BLOCK + 2 * (size_t)items * (BLOCK / kWave)) * 4;
    if (lds > 65536 &&    // more than 64 KiB of dynamic LDS needs a one-time opt-in
        (!allow_big_lds((const void *)topk_rows_lds_kernel<BLOCK, PLAN, DIG, false>, 140 * 1024) ||
         !allow_big_lds((const void *)topk_rows_lds_kernel<BLOCK, PLAN, DIG, true>, 140 * 1024)))
        return hipGetLastError();
    if (gate)
        hipLaunchKernelGGL((topk_rows_lds_kernel<BLOCK, PLAN, DIG, true>), dim3(rows > 1024 ? 1024 : rows),
                           dim3(BLOCK), lds, st, x, ld, n, rows, k, idx_out, idx_ld, val_out, val_ld,
                           tau_out, append_from, append_count, gate, rows_per_gate, plan);
    else
        hipLaunchKernelGGL((topk_rows_lds_kernel<BLOCK, PLAN, DIG, false>), dim3(rows), dim3(BLOCK), lds,
                           st, x, ld, n, rows, k, idx_out, idx_ld, val_out, val_ld, tau_out, append_from,
                           append_count, gate, rows_per_gate, plan);
    return hipGetLastError();
}

template <bool PLAN, typename PlanArg>
static hipError_t launch_any(const float *x, long ld, int n, int rows, int k, int32_t *idx_out,
                             long idx_ld, float *val_out, long val_ld, float *tau_out,
                             int append_from, int append_count, const int32_t *gate,
                             int rows_per_gate, PlanArg plan, hipStream_t st)
{
    if (rows <= 0) return hipSuccess;
    if (n <= 4096)
        return launch_lds<256, PLAN, 8>(x, ld, n, rows, k, idx_out, idx_ld, val_out, val_ld, tau_out,
                                        append_from, append_count, gate, rows_per_gate, plan, st);
    if constexpr (!PLAN) {
        if (n > 4096 && n <= 32768 && k <= kSmallK && idx_out && !val_out && !tau_out && append_count == 0 &&
            !gate) {
            hipLaunchKernelGGL(topk_rows_smallk_kernel<1024>, dim3(rows), dim3(1024), 0, st, x, ld, n, k,
                               idx_out, idx_ld);
            return hipGetLastError();
        }
    }
    if (n <= 32768)
        return launch_lds<1024, PLAN, 11>(x, ld, n, rows, k, idx_out, idx_ld, val_out, val_ld, tau_out,
                                          append_from, append_count, gate, rows_per_gate, plan, st);
    if constexpr (!PLAN) {
        if (k <= kSmallK && idx_out && !val_out && !tau_out && append_count == 0 && !gate) {
            hipLaunchKernelGGL(topk_rows_long_smallk_kernel<1024>, dim3(rows), dim3(1024), 0, st, x, ld, n, k,
                               idx_out, idx_ld);
            return hipGetLastError();
        }
    }
    hipLaunchKernelGGL((topk_rows_stream_kernel<1024, PLAN>), dim3(gate && rows > 1024 ? 1024 : rows), dim3(1024),
                       0, st, x, ld, n, rows, k, idx_out, idx_ld, val_out, val_ld, tau_out, append_from,
                       append_count, gate, rows_per_gate, plan);
    return hipGetLastError();
}

hipError_t launch_topk_rows(const float *x, long ld, int n, int rows, int k, int32_t *idx_out,
                            long idx_ld, float *val_out, long val_ld, float *tau_out,
                            int append_from, int append_count, const int32_t *gate,
                            int rows_per_gate, hipStream_t st)
{
    return launch_any<false, int>(x, ld, n, rows, k, idx_out, idx_ld, val_out, val_ld, tau_out,
                                  append_from, append_count, gate, rows_per_gate, 0, st);
}

int redo_rows_workgroups(int heads, int S)
{
    const long items = (long)heads * S;
    return (int)(items < 256 ? items : 256);
}

size_t redo_rows_scratch_bytes(int heads, int S, int P)
{
    return (size_t)redo_rows_workgroups(heads, S) * P * sizeof(float);
}

hipError_t launch_redo_rows(const void *Ac, const void *Kc, int heads, int N, int P, int S, int m,
                            const int32_t *src, const int32_t *overflow, float *rows, int32_t *nbr,
                            float *nbr_e, hipStream_t st)
{
    const int items = P <= 32768 ? (P + kRedoBlock - 1) / kRedoBlock : 0;   // keys of a row in LDS
    const size_t lds = ((size_t)items * kRedoBlock + 2 * (size_t)items * (kRedoBlock / kWave)) * 4;
    if (lds > 65536 && !allow_big_lds((const void *)redo_rows_kernel, 140 * 1024)) return hipGetLastError();
    hipLaunchKernelGGL(redo_rows_kernel, dim3(redo_rows_workgroups(heads, S)), dim3(kRedoBlock), lds, st,
                       (const uint16_t *)Ac, (const uint16_t *)Kc, N, P, S, m, heads, src, overflow, rows, nbr,
                       nbr_e);
    return hipGetLastError();
}

hipError_t launch_topk_final(const float *scores, int P, int rows, const LayerPlan &plan, int w,
                             int32_t *idx, hipStream_t st)
{
    return launch_any<true, LayerPlan>(scores, P, P, rows, 0, idx, 0, nullptr, 0, nullptr, P, w,
                                       nullptr, 1, plan, st);
}

}  // namespace gkv
