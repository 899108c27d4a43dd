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
#include "mfma_tile.hpp"

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
        const float v = xr[min(j, n - 1)];   // (unconditional: the loads of a batch leave together)
        const uint32_t key = ord_key(j < n ? v : 0.f);
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
// Winners of a row, (index << 32) | key each, in any order -> the row's outputs.  With
// ext_out the k winners are the S best and the X = k - S next best: a winner that fewer
// than S others beat by (key descending, index ascending) is one of the S; src_out gets
// those in ascending index order, ext_out the same S followed by the others in ascending
// index order.  Without ext_out (S = k) this is the plain ascending list.  `cls` holds k
// bytes of LDS; every thread of the workgroup calls this (k <= kSmallK <= blockDim.x).
constexpr int kSmallK = 256;       // largest k the small-k paths take

__device__ __forceinline__ void emit_sources(const uint64_t *win, int k, int S, int32_t *src_out,
                                             int32_t *ext_out, uint8_t *cls, int tid)
{
    uint64_t mine = 0;
    bool first_s = true;
    if (tid < k) {
        mine = win[tid];
        const uint32_t key = (uint32_t)mine, idx = (uint32_t)(mine >> 32);
        int beat = 0;
        for (int u = 0; u < k; ++u) {
            const uint64_t w = win[u];
            const uint32_t ku = (uint32_t)w, iu = (uint32_t)(w >> 32);
            beat += (ku > key) || (ku == key && iu < idx);
        }
        first_s = beat < S;
        cls[tid] = first_s ? 1 : 0;
    }
    __syncthreads();
    if (tid < k) {
        int before = 0;   // winners of the same class with a lower index
        for (int u = 0; u < k; ++u) before += (win[u] >> 32) < (mine >> 32) && (cls[u] != 0) == first_s;
        const int32_t idx = (int32_t)(mine >> 32);
        if (first_s) {
            src_out[before] = idx;
            if (ext_out) ext_out[before] = idx;
        } else {
            ext_out[S + before] = idx;
        }
    }
}

// The same by one wave on its own (no workgroup barrier, no LDS in the loops): lane L keeps
// winners L, L + 64, ... in R registers (k <= 64 R) and every winner in turn is broadcast to
// the wave from its lane.
template <int R>
__device__ __forceinline__ void emit_sources_wave_r(const uint64_t *win, int k, int S, int32_t *src_out,
                                                    int32_t *ext_out, int lane)
{
    uint32_t key[R], idx[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint64_t w = r * kWave + lane < k ? win[r * kWave + lane] : 0ull;
        key[r] = (uint32_t)w;
        idx[r] = (uint32_t)(w >> 32);
    }
    // One of the S best: above the S-th largest key of the winners, or equal to it and among the
    // lowest indices of those (only if the tie straddles the cut are the tied entries ranked).
    bool first_s[R];
#pragma unroll
    for (int r = 0; r < R; ++r) first_s[r] = true;
    if (ext_out && S < k) {
        uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (r * kWave + lane < k) { kmin = min(kmin, key[r]); kmax = max(kmax, key[r]); }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, o, kWave));
            kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o, kWave));
        }
        const uint32_t tau_s = mth_largest_key<R>(key, kmin, kmax, S);
        int above = 0, equal = 0;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            above += (int)__popcll(__ballot(r * kWave + lane < k && key[r] > tau_s));
            equal += (int)__popcll(__ballot(r * kWave + lane < k && key[r] == tau_s));
        }
        const int need = S - above;   // tied entries that still belong to the S
        int tied_before[R];
#pragma unroll
        for (int r = 0; r < R; ++r) tied_before[r] = 0;
        if (equal != need) {
#pragma unroll
            for (int ru = 0; ru < R; ++ru)
                for (int l = 0; l < kWave && ru * kWave + l < k; ++l) {
                    const uint32_t ku = (uint32_t)__builtin_amdgcn_readlane((int)key[ru], l);
                    const uint32_t iu = (uint32_t)__builtin_amdgcn_readlane((int)idx[ru], l);
#pragma unroll
                    for (int r = 0; r < R; ++r) tied_before[r] += ku == tau_s && iu < idx[r];
                }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) first_s[r] = key[r] > tau_s || (key[r] == tau_s && tied_before[r] < need);
    }
    // place = winners of the same class with a lower index
    int before[R];
#pragma unroll
    for (int r = 0; r < R; ++r) before[r] = 0;
#pragma unroll
    for (int ru = 0; ru < R; ++ru)
        for (int l = 0; l < kWave && ru * kWave + l < k; ++l) {
            const uint32_t iu = (uint32_t)__builtin_amdgcn_readlane((int)idx[ru], l);
            const bool su = __builtin_amdgcn_readlane(first_s[ru] ? 1 : 0, l) != 0;
#pragma unroll
            for (int r = 0; r < R; ++r) before[r] += iu < idx[r] && su == first_s[r];
        }
#pragma unroll
    for (int r = 0; r < R; ++r)
        if (r * kWave + lane < k) {
            if (first_s[r]) {
                src_out[before[r]] = (int32_t)idx[r];
                if (ext_out) ext_out[before[r]] = (int32_t)idx[r];
            } else {
                ext_out[S + before[r]] = (int32_t)idx[r];
            }
        }
}

__device__ __forceinline__ void emit_sources_wave(const uint64_t *win, int k, int S, int32_t *src_out,
                                                  int32_t *ext_out, int lane)
{
    if (k <= kWave) emit_sources_wave_r<1>(win, k, S, src_out, ext_out, lane);
    else if (k <= 2 * kWave) emit_sources_wave_r<2>(win, k, S, src_out, ext_out, lane);
    else emit_sources_wave_r<kSmallK / kWave>(win, k, S, src_out, ext_out, lane);
}

// For k far below the row length (the source nodes: 64 of 32736, with the speculative
// rows 96) the row is read once into registers (32 keys per thread).  A bound comes almost
// for free: split the threads into G >= k groups; the smallest of the G group maxima is
// reached by G different entries, so the k-th largest key is at least that (if too many
// entries reach it, one radix sweep raises it).  The few hundred
// keys that reach the bound are compacted into an LDS list (positions from wave votes, one
// atomic per wave and register), and from there on the registers are free: one wave finds the
// k-th largest key of the list bit by bit (its keys in registers, a wave vote per register and
// bit, no barrier), every entry above it and the lowest-index entries equal to it are the
// winners, and emit_sources() orders them.  A row with more than kPickCap entries at or above
// the bound (masses of equal values) takes the algorithm that re-reads the row instead.
constexpr int kPickCap = 2048;     // list entries: 32 registers of a wave

template <int BLOCK, bool PLAN> __device__ __forceinline__ void topk_stream_row(
    int row, const float *__restrict__ x, long ld, int n, int k, int32_t *__restrict__ idx_out, long idx_ld,
    float *__restrict__ val_out, long val_ld, float *__restrict__ tau_out, int append_from,
    int append_count, const int32_t *__restrict__ gate, int rows_per_gate,
    typename std::conditional<PLAN, LayerPlan, int>::type plan);

template <int NIT>
__device__ __forceinline__ uint32_t pick_tau(const uint32_t *lk, int cnt, int lane, int k, uint32_t kmin,
                                             uint32_t kmax)
{
    uint32_t E[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) E[it] = it * 64 + lane < cnt ? lk[it * 64 + lane] : 0u;
    return mth_largest_key<NIT>(E, kmin, kmax, k);
}

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void pick_sources_kernel(
    const float *__restrict__ x, long ld, int n, int k, int S, int32_t *__restrict__ src_out, long src_ld,
    int32_t *__restrict__ ext_out, long ext_ld)
{
    constexpr int ITEMS = 32768 / BLOCK, NW = BLOCK / kWave, DIG = 11, NBINS = 1 << DIG;
    __shared__ uint32_t lk[kPickCap], lj[kPickCap];   // keys and indices of the entries that reach the bound
    __shared__ uint32_t hist[NBINS];
    __shared__ uint64_t win[kSmallK];
    __shared__ uint8_t cls[kSmallK];
    __shared__ uint32_t s_grp[kSmallK], s_bound, s_wmax[NW], s_max, s_cnt, s_need, s_bin;
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const float *xr = x + (long)row * ld;
    int32_t *src_row = src_out + (long)row * src_ld;
    int32_t *ext_row = ext_out ? ext_out + (long)row * ext_ld : nullptr;

    // All loads of the row leave together: clamped, unconditional, and their values pinned in
    // registers before the first use (otherwise the compiler moves every load behind the
    // test of its index and waits for each in turn).
    float val[ITEMS];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) val[i] = xr[min(i * BLOCK + tid, n - 1)];
#pragma unroll
    for (int i = 0; i < ITEMS; i += 8)
        asm volatile("" : "+v"(val[i]), "+v"(val[i + 1]), "+v"(val[i + 2]), "+v"(val[i + 3]), "+v"(val[i + 4]),
                          "+v"(val[i + 5]), "+v"(val[i + 6]), "+v"(val[i + 7]));
    uint32_t key[ITEMS];
    uint32_t best = 0;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        key[i] = i * BLOCK + tid < n ? ord_key(val[i]) : 0u;   // 0 is below the key of every number
        best = max(best, key[i]);
    }
    // G groups (G a power of two, k <= G <= 256): thread t belongs to group t mod G, so a group
    // owns the entries whose index is t mod G -- scores are smooth along the row (pooling), and
    // this way the few peaks that hold the winners spread over many groups.  Group maxima (an
    // LDS atomic per thread), their minimum = the bound; the row maximum on the way.
    int G = 16;
    while (G < k) G <<= 1;
    if (tid < G) s_grp[tid] = 0u;
    if (tid == 0) s_cnt = 0;
    for (int b = tid; b < NBINS; b += BLOCK) hist[b] = 0;
    __syncthreads();
    atomicMax(&s_grp[tid & (G - 1)], best);
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
    uint32_t bound = s_bound;
    const uint32_t kmax = s_max;

    // One radix sweep over the entries that reach the bound -- 11 bits of key - bound from the
    // top bit in which they can differ -- raises the bound to the lower edge of the bin in which
    // the count from the top reaches k: a handful of entries beyond the k winners remain.
    if (kmax > bound) {   // (the same for every thread)
        const int remaining = 32 - __clz(kmax - bound);
        const int bits = remaining < DIG ? remaining : DIG, shift = remaining - bits;
#pragma unroll
        for (int i = 0; i < ITEMS; ++i)
            if (key[i] >= bound && key[i] != 0u) atomicAdd(&hist[(key[i] - bound) >> shift], 1u);
        __syncthreads();
        if (wv == 0) find_bin<NBINS / 64>(hist, (uint32_t)k, lane, &s_bin, &s_need);
        __syncthreads();
        bound += s_bin << shift;
    }

    // everything that reaches the bound -> the list (any order): a wave counts its entries with
    // wave votes, takes its stretch of the list with one atomic, and places them
    const uint64_t below = (1ull << lane) - 1ull;
    uint32_t mine = 0;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) mine += (uint32_t)__popcll(__ballot(key[i] >= bound && key[i] != 0u));
    uint32_t at0 = 0;
    if (lane == 0 && mine) at0 = atomicAdd(&s_cnt, mine);
    at0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)at0);
    if (mine) {   // (the same for every lane of the wave)
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const bool in = key[i] >= bound && key[i] != 0u;
            const uint64_t votes = __ballot(in);
            const uint32_t at = at0 + (uint32_t)__popcll(votes & below);
            if (in && at < (uint32_t)kPickCap) { lk[at] = key[i]; lj[at] = (uint32_t)(i * BLOCK + tid); }
            at0 += (uint32_t)__popcll(votes);
        }
    }
    __syncthreads();
    const int cnt = (int)s_cnt;
    if (cnt > kPickCap) {   // (the same for every thread) masses of equal values: re-read the row
        int32_t *tmp = ext_row ? ext_row : src_row;
        topk_stream_row<BLOCK, false>(row, x, ld, n, k, tmp, 0, nullptr, 0, nullptr, 0, 0, nullptr, 1, 0);
        if (!ext_row) return;
        __syncthreads();
        if (tid < k) {
            const uint32_t j = (uint32_t)ext_row[tid];
            win[tid] = ((uint64_t)j << 32) | ord_key(xr[j]);
        }
        __syncthreads();
        emit_sources(win, k, S, src_row, ext_row, cls, tid);
        return;
    }
    if (wv != 0) return;

    // One wave finishes the row on its own: the k-th largest key of the list, ...
    const int n_it = (cnt + 63) >> 6;
    uint32_t tau;
    if (n_it <= 4) tau = pick_tau<4>(lk, cnt, lane, k, bound, kmax);
    else if (n_it <= 8) tau = pick_tau<8>(lk, cnt, lane, k, bound, kmax);
    else if (n_it <= 16) tau = pick_tau<16>(lk, cnt, lane, k, bound, kmax);
    else tau = pick_tau<32>(lk, cnt, lane, k, bound, kmax);
    int above = 0, equal = 0;
    for (int r = lane; r < cnt; r += kWave) { above += lk[r] > tau; equal += lk[r] == tau; }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { above += __shfl_xor(above, o, kWave); equal += __shfl_xor(equal, o, kWave); }
    // ... the winners: every entry above it and, of the entries equal to it, the `need` lowest
    // indices (usually all of them) ...
    const int need = k - above;
    int listed = 0;
    for (int r0 = 0; r0 < cnt; r0 += kWave) {
        const int r = r0 + lane;
        const uint32_t kr = r < cnt ? lk[r] : 0u, jr = r < cnt ? lj[r] : 0u;
        bool in = r < cnt && kr >= tau;
        if (in && kr == tau && equal != need) {
            int rank = 0;
            for (int u = 0; u < cnt; ++u) rank += (lk[u] == tau) & (lj[u] < jr);
            in = rank < need;
        }
        const uint64_t votes = __ballot(in);
        if (in) win[listed + (int)__popcll(votes & below)] = ((uint64_t)jr << 32) | kr;
        listed += (int)__popcll(votes);
    }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
    // ... and their order.
    emit_sources_wave(win, k, S, src_row, ext_row, lane);
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
                t[u] = xr[min(j, n - 1)];
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
            t[u] = xr[min(j, n - 1)];
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
            t[u] = xr[min(j, n - 1)];
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
    const float *__restrict__ x, long ld, int n, int k, int S, int32_t *__restrict__ idx_out, long idx_ld,
    int32_t *__restrict__ ext_out, long ext_ld)
{
    constexpr int NW = BLOCK / kWave, U = 8;
    __shared__ uint32_t lk[kLongCap], lj[kLongCap];   // keys and indices of the candidates
    __shared__ uint32_t tmax[BLOCK];
    __shared__ uint64_t win[kSmallK];                 // (index << 32) | key of the winners
    __shared__ uint32_t hist8[256];
    __shared__ uint32_t s_cnt, s_bin, s_need, s_wmax[NW], s_wmin[NW];
    __shared__ int32_t n_win, n_eq;
    __shared__ uint8_t cls[kSmallK];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const float *xr = x + (long)blockIdx.x * ld;
    int32_t *out = idx_out + (long)blockIdx.x * idx_ld;
    int32_t *ext_row = ext_out ? ext_out + (long)blockIdx.x * ext_ld : nullptr;

    // first read: the largest key each thread owns (0 is below the key of every number)
    uint32_t mx = 0u;
    for (int j0 = 0; j0 < n; j0 += BLOCK * U) {
        float t[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + u * BLOCK + tid;
            t[u] = xr[min(j, n - 1)];
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
            t[u] = xr[min(j, n - 1)];
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
        int32_t *tmp = ext_row ? ext_row : out;
        topk_stream_row<BLOCK, false>(0, x + (long)blockIdx.x * ld, ld, n, k, tmp, 0, nullptr, 0, nullptr, 0, 0,
                                      nullptr, 1, 0);
        if (!ext_row) return;
        __syncthreads();
        if (tid < k) {
            const uint32_t j = (uint32_t)ext_row[tid];
            win[tid] = ((uint64_t)j << 32) | ord_key(xr[j]);
        }
        __syncthreads();
        emit_sources(win, k, S, out, ext_row, cls, tid);
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
    emit_sources(win, k, S, out, ext_row, cls, tid);   // ascending index order
}

// ---- neighbourhoods of heads whose candidate lists overflowed ------------------------
// The filter route (mfma_cosine.hip) gives up on a head when a candidate list cannot hold what
// reaches the bound (masses of equal edges, an adversarial key order) and raises the head's
// flag.  Such heads are rare, so they are not worth an [heads, S, P] edge block in memory: a
// fixed number of workgroups walk the (head, source) rows of the flagged heads, and each row's
// edges (Eq. 1) go to the workgroup's own scratch row of P floats, out of which the exact top-m
// (Eq. 3) is taken by the row kernels above.  The edges are formed exactly as in the streaming
// kernels -- the same matrix-core instruction sequence with the source in every operand row, the
// same norms -- so that a head gets the same bits whichever route it takes.  A launch that
// finds no flag set returns after one round trip.
constexpr int kRedoBlock = 1024;

__global__ __launch_bounds__(kRedoBlock) void redo_rows_kernel(
    const uint16_t *__restrict__ Ac, const uint16_t *__restrict__ Kc, int N, int P, int S, int m, int heads,
    const int32_t *__restrict__ src, const int32_t *__restrict__ overflow, float *__restrict__ rows,
    int32_t *__restrict__ nbr, float *__restrict__ nbr_e)
{
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, hh = lane >> 5;
    int open = 0;
    for (int g = tid; g < heads; g += kRedoBlock) open |= overflow[g] != 0;
    if (!__syncthreads_or(open)) return;
    float *erow = rows + (long)blockIdx.x * P;
    for (long item = blockIdx.x; item < (long)heads * S; item += gridDim.x) {
        const int h = (int)(item / S);
        if (overflow[h] == 0) continue;           // (the same for every thread)
        const int32_t i = src[item];
        const uint16_t *ah = Ac + (long)h * N * kD, *kh = Kc + (long)h * N * kD;
        __syncthreads();                          // the previous row's LDS and scratch row are free
        // the source's row in every row of the operand (a lane holds elements 16 s + 8 hh ..)
        bf16x8 q[kSteps];
#pragma unroll
        for (int s = 0; s < kSteps; ++s) q[s] = load8(ah + (long)i * kD + 16 * s + 8 * hh);
        float sq_i = half_row_sumsq(q);
        sq_i = add_other_half(sq_i);
        const float inv_i = inv_norm(sq_i);
        // blocks of 32 keys, one per wave at a time: key l32 of the block is the operand's column
        for (int j0 = wv * kBlk; j0 < P; j0 += (kRedoBlock / kWave) * kBlk) {
            const int j = min(j0 + l32, P - 1);
            bf16x8 kc[kSteps];
#pragma unroll
            for (int s = 0; s < kSteps; ++s) kc[s] = load8(kh + (long)j * kD + 16 * s + 8 * hh);
            f32x16 acc;
#pragma unroll
            for (int u = 0; u < 16; ++u) acc[u] = 0.f;
#pragma unroll
            for (int s = 0; s < kSteps; ++s)   // rows = the source (32 times), columns = keys
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q[s], kc[s], acc, 0, 0, 0);
            float sq = half_row_sumsq(kc);
            sq = add_other_half(sq);
            const float e = (acc[0] * inv_norm(sq)) * inv_i;
            if (hh == 0 && j0 + l32 < P) erow[j] = j == i ? -INFINITY : e;   // (Eq. 3: j != i)
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
            hipLaunchKernelGGL(pick_sources_kernel<1024>, dim3(rows), dim3(1024), 0, st, x, ld, n, k, k, idx_out,
                               idx_ld, (int32_t *)nullptr, 0L);
            return hipGetLastError();
        }
    }
    if (n <= 32768)
        return launch_lds<1024, PLAN, 11>(x, ld, n, rows, k, idx_out, idx_ld, val_out, val_ld, tau_out,
                                          append_from, append_count, gate, rows_per_gate, plan, st);
    if constexpr (!PLAN) {
        if (k <= kSmallK && idx_out && !val_out && !tau_out && append_count == 0 && !gate) {
            hipLaunchKernelGGL(topk_rows_long_smallk_kernel<1024>, dim3(rows), dim3(1024), 0, st, x, ld, n, k, k,
                               idx_out, idx_ld, (int32_t *)nullptr, 0L);
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

// Workgroups that walk the rows of flagged heads: one per compute unit, fewer for long rows
// (their scratch rows stay within 64 MiB), at least 16.
int redo_rows_workgroups(int heads, int S, int P)
{
    const long items = (long)heads * S;
    long wgs = ((long)64 << 20) / ((long)P * 4);
    wgs = wgs < 16 ? 16 : (wgs > 256 ? 256 : wgs);
    return (int)(items < wgs ? items : wgs);
}

size_t redo_rows_scratch_bytes(int heads, int S, int P)
{
    return (size_t)redo_rows_workgroups(heads, S, P) * P * sizeof(float);
}

hipError_t launch_redo_rows(const void *Ac, const void *Kc, int heads, int N, int P, int S, int m,
                            const int32_t *src, const int32_t *overflow, float *rows, int32_t *nbr,
                            float *nbr_e, hipStream_t st)
{
    const int items = P <= 32768 ? (P + kRedoBlock - 1) / kRedoBlock : 0;   // keys of a row in LDS
    const size_t lds = ((size_t)items * kRedoBlock + 2 * (size_t)items * (kRedoBlock / kWave)) * 4;
    if (lds > 65536 && !allow_big_lds((const void *)redo_rows_kernel, 140 * 1024)) return hipGetLastError();
    hipLaunchKernelGGL(redo_rows_kernel, dim3(redo_rows_workgroups(heads, S, P)), dim3(kRedoBlock), lds, st,
                       (const uint16_t *)Ac, (const uint16_t *)Kc, N, P, S, m, heads, src, overflow, rows, nbr,
                       nbr_e);
    return hipGetLastError();
}

hipError_t launch_pick_sources(const float *x, long ld, int n, int rows, int S, int X, int32_t *src,
                               int32_t *ext, hipStream_t st)
{
    if (rows <= 0) return hipSuccess;
    if (n <= 4096 || S + X > kSmallK) return hipErrorInvalidValue;
    if (n <= 32768)
        hipLaunchKernelGGL(pick_sources_kernel<1024>, dim3(rows), dim3(1024), 0, st, x, ld, n, S + X, S, src,
                           (long)S, ext, (long)(S + X));
    else
        hipLaunchKernelGGL(topk_rows_long_smallk_kernel<1024>, dim3(rows), dim3(1024), 0, st, x, ld, n, S + X, S,
                           src, (long)S, ext, (long)(S + X));
    return hipGetLastError();
}

hipError_t launch_topk_final(const float *scores, int P, int rows, const LayerPlan &plan, int w,
                             int32_t *idx, hipStream_t st)
{
    return launch_any<true, LayerPlan>(scores, P, P, rows, 0, idx, 0, nullptr, 0, nullptr, P, w,
                                       nullptr, 1, plan, st);
}

}  // namespace gkv
