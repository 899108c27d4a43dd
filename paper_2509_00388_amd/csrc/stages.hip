// Pooling of the window votes, the signal-propagation update (Eq. 4 / Eq. 5)
// and the K/V gather of the retained rows.
#include "common.hpp"
#include "kernels.hpp"

#include <mutex>
#include <set>
#include <utility>

namespace gkv {

bool allow_big_lds(const void *kernel, int bytes)
{
    static std::mutex mu;
    static std::set<std::pair<int, const void *>> done;   // (device, kernel) pairs that are opted in
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    std::lock_guard<std::mutex> lock(mu);
    if (done.count({dev, kernel})) return true;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess)
        return false;
    done.insert({dev, kernel});
    return true;
}

// scores[h, j] = (1/div) * sum_g pool(votes[h*Gv + g, j-half .. j+half]).
// Average pooling pads with zeros and divides by the kernel size; max pooling
// ignores positions outside the row.
__global__ __launch_bounds__(256) void pool_group_kernel(const float *__restrict__ votes, int Gv,
                                                         int P, int pool_kernel, int pool_mode,
                                                         float div, float *__restrict__ scores)
{
    const int h = blockIdx.y, j = blockIdx.x * 256 + threadIdx.x;
    if (j >= P) return;
    const int half = (pool_kernel - 1) / 2;
    const int lo = max(0, j - half), hi = min(P - 1, j + half);
    float total = 0.f;
    for (int g = 0; g < Gv; ++g) {
        const float *v = votes + ((long)h * Gv + g) * P;
        float acc;
        if (pool_mode == 0) {
            acc = 0.f;
            for (int t = lo; t <= hi; ++t) acc += v[t];
            acc = acc / (float)pool_kernel;
        } else {
            acc = -INFINITY;
            for (int t = lo; t <= hi; ++t) acc = fmaxf(acc, v[t]);
        }
        total += acc;
    }
    scores[(long)h * P + j] = total / div;
}

// Average pooling is linear, so the Gv vote rows of a head are added first (one
// coalesced load per row and thread) and the sum is pooled once out of an LDS tile
// with a halo.  Same value as pooling each row and adding, up to fp32 rounding order.
constexpr int kPoolHalo = 16;
// kPoolTile outputs per workgroup: 2048 (8 per thread, enough loads in flight per CU) when
// there are many heads, 256 when the grid would otherwise not fill the chip.
template <int kPoolTile>
__global__ __launch_bounds__(256) void pool_avg_kernel(const float *__restrict__ votes, int Gv, int P,
                                                       int pool_kernel, float div,
                                                       float *__restrict__ scores)
{
    __shared__ float tile[kPoolTile + 2 * kPoolHalo];
    const int h = blockIdx.y, j0 = blockIdx.x * kPoolTile, tid = threadIdx.x;
    const int half = (pool_kernel - 1) / 2;
    for (int u = tid; u < kPoolTile + 2 * kPoolHalo; u += 256) {
        const int j = j0 - kPoolHalo + u;
        float v = 0.f;                               // zero padding outside the row
        if (j >= 0 && j < P && u >= kPoolHalo - half && u < kPoolTile + kPoolHalo + half)
            for (int g = 0; g < Gv; ++g) v += votes[((long)h * Gv + g) * P + j];
        tile[u] = v;
    }
    __syncthreads();
    for (int o = tid; o < kPoolTile; o += 256) {
        const int j = j0 + o;
        if (j >= P) break;
        float acc = 0.f;
        for (int t = -half; t <= half; ++t) acc += tile[kPoolHalo + o + t];
        scores[(long)h * P + j] = acc / (float)pool_kernel / div;
    }
}

// Factor of one edge (Eq. 4 / Eq. 5).  The signal acts on the magnitude of the score the
// round started with: the decay takes alpha * e * |s| away, the enhanced signal adds it, so
// for a negative score (an indicator such as minus the key norm) the signs swap and the
// decay still lowers the score.  For s >= 0 this is (1 - alpha e) as printed.
__device__ __forceinline__ float signal_factor(float e, float alpha, int signal, bool negative)
{
    return ((signal == 1) != negative) ? fmaf(alpha, e, 1.0f) : fmaf(-alpha, e, 1.0f);
}

// Bitonic sort of npad 64-bit keys in LDS by one workgroup of NW waves.  Wave w
// owns pairs [w*Q, (w+1)*Q), Q = npad / (2 NW).  For compare distances j <= Q those
// pairs touch only elements [2wQ, 2(w+1)Q), so such stages need no workgroup barrier:
// LDS operations of one wave complete in order.  Only the stages with j > Q
// synchronise the workgroup.
template <int NW>
__device__ __forceinline__ void bitonic_sort_lds(uint64_t *keys, int npad, int lane, int wv)
{
    const int Q = npad / (2 * NW);
    for (int k = 2; k <= npad; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            const bool wide = j > Q;
            if (wide) __syncthreads();
            for (int e = wv * Q + lane; e < (wv + 1) * Q; e += kWave) {
                const int t = ((e & ~(j - 1)) << 1) | (e & (j - 1)), u = t + j;
                const uint64_t a = keys[t], b = keys[u];
                const bool up = (t & k) == 0;
                if ((a > b) == up) { keys[t] = b; keys[u] = a; }
            }
            if (wide) __syncthreads();
            else __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        }
    }
    __syncthreads();
}

// Eq. 5 for one round, S*m <= 4096.  One workgroup per head, no sort and no float
// atomics.  Every (source slot, node, edge) triple t finds its node's cell in an
// LDS hash table (open addressing; integer compare-and-swap claims a cell).  Then
// the triples of a node are peeled off in ascending t, one per pass: all pending
// triples post their t with an integer min, the one that reads its own t back
// multiplies its factor into the cell's product -- it is the cell's only writer in
// that pass -- and retires.  Sources are stored in ascending index order, so the
// product is Eq. 5's with a fixed floating-point order whatever the thread timing.
// Most nodes have a single triple; the number of passes is the largest number of
// sources that share one neighbour.  Two sets of min cells alternate so that a
// winner can reset its cell without a third barrier per pass.
constexpr int kDecayThreads = 512;
constexpr int kDecayPer = 4096 / kDecayThreads;
constexpr uint32_t kNoNode = 0xffffffffu;

__global__ __launch_bounds__(kDecayThreads) void decay_hash_kernel(
    float *__restrict__ scores, int P, int count, int table_log2, const int32_t *__restrict__ nbr,
    const float *__restrict__ nbr_e, float alpha, int signal)
{
    extern __shared__ uint32_t table[];
    const int Tn = 1 << table_log2;
    uint32_t *cell_node = table;                               // [Tn] node of a cell
    uint32_t *low0 = table + Tn, *low1 = table + 2 * Tn;       // [Tn] lowest pending triple, two sets
    float *prod = reinterpret_cast<float *>(table + 3 * Tn);   // [Tn] product of the retired factors
    const int h = blockIdx.x, tid = threadIdx.x;
    const int32_t *nb = nbr + (long)h * count;
    const float *ne = nbr_e + (long)h * count;
    float *s = scores + (long)h * P;

    uint32_t node[kDecayPer], cell[kDecayPer];
    float fac[kDecayPer];
#pragma unroll
    for (int q = 0; q < kDecayPer; ++q) {
        const int t = q * kDecayThreads + tid;
        const int tc = min(t, count - 1);   // (unconditional loads leave together)
        const uint32_t nd = (uint32_t)nb[tc];
        const float ed = ne[tc];
        node[q] = t < count ? nd : kNoNode;
        fac[q] = t < count ? ed : 0.f;
    }
    // the sign of each node's score decides the direction of its factors; these loads are in
    // flight while the table is set up
    static_assert(kDecayPer == 8, "the loads below are pinned eight at a time");
    float sj[kDecayPer];
#pragma unroll
    for (int q = 0; q < kDecayPer; ++q) sj[q] = s[node[q] != kNoNode ? node[q] : 0u];   // (unconditional)
    asm volatile("" : "+v"(sj[0]), "+v"(sj[1]), "+v"(sj[2]), "+v"(sj[3]), "+v"(sj[4]), "+v"(sj[5]), "+v"(sj[6]),
                      "+v"(sj[7]));
#pragma unroll
    for (int q = 0; q < kDecayPer; ++q)
        fac[q] = node[q] != kNoNode ? signal_factor(fac[q], alpha, signal, sj[q] < 0.f) : 1.0f;
    for (int i = tid; i < Tn; i += kDecayThreads) {
        cell_node[i] = kNoNode;
        low0[i] = kNoNode;
        low1[i] = kNoNode;
        prod[i] = 1.0f;
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < kDecayPer; ++q) {
        cell[q] = 0;
        if (node[q] != kNoNode) {
            uint32_t c = (node[q] * 2654435761u) >> (32 - table_log2);
            while (true) {   // the table has at least twice as many cells as triples
                const uint32_t prev = atomicCAS(&cell_node[c], kNoNode, node[q]);
                if (prev == kNoNode || prev == node[q]) break;
                c = (c + 1) & (Tn - 1);
            }
            cell[q] = c;
        }
    }
    __syncthreads();
    for (int pass = 0;; ++pass) {
        uint32_t *low = (pass & 1) ? low1 : low0;
#pragma unroll
        for (int q = 0; q < kDecayPer; ++q)
            if (node[q] != kNoNode) atomicMin(&low[cell[q]], (uint32_t)(q * kDecayThreads + tid));
        __syncthreads();
        int left = 0;
#pragma unroll
        for (int q = 0; q < kDecayPer; ++q) {
            if (node[q] == kNoNode) continue;
            if (low[cell[q]] == (uint32_t)(q * kDecayThreads + tid)) {
                prod[cell[q]] *= fac[q];
                node[q] = kNoNode;
            } else {
                left = 1;
            }
        }
        // every compare above is done before a winner resets its cell below; the set
        // is next used two passes on, behind the barriers of the pass in between
        const int more = __syncthreads_or(left);
#pragma unroll
        for (int q = 0; q < kDecayPer; ++q)
            if (node[q] == kNoNode && low[cell[q]] == (uint32_t)(q * kDecayThreads + tid))
                low[cell[q]] = kNoNode;
        if (!more) break;
    }
    __syncthreads();
    for (int base = 0; base < Tn; base += kDecayThreads * 4) {
        uint32_t nd[4];
        float sv[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int i = base + q * kDecayThreads + tid;
            nd[q] = i < Tn ? cell_node[i] : kNoNode;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) sv[q] = nd[q] != kNoNode ? s[nd[q]] : 0.f;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (nd[q] != kNoNode)
                s[nd[q]] = signal == 2 ? -INFINITY : sv[q] * prod[base + q * kDecayThreads + tid];
    }
}

// 4096 < S*m <= 16384: the triples are sorted by (node, slot) in LDS (128 KiB of
// keys); the first triple of every node multiplies that node's factors in ascending
// slot order and writes the node's score once.  Edge weights come from global memory.
template <int NT>
__global__ __launch_bounds__(NT) void decay_sorted_kernel(
    float *__restrict__ scores, int P, int count, int npad, const int32_t *__restrict__ nbr,
    const float *__restrict__ nbr_e, float alpha, int signal)
{
    extern __shared__ uint64_t keys[];     // (node << 32) | triple id
    const int h = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int32_t *nb = nbr + (long)h * count;
    const float *ne = nbr_e + (long)h * count;
    float *s = scores + (long)h * P;
    for (int t = tid; t < npad; t += NT)
        keys[t] = t < count ? (((uint64_t)(uint32_t)nb[min(t, count - 1)] << 32) | (uint32_t)t) : ~0ull;
    __syncthreads();
    bitonic_sort_lds<NT / kWave>(keys, npad, lane, wv);
    for (int t = tid; t < count; t += NT) {
        const uint64_t key = keys[t];
        const uint32_t node = (uint32_t)(key >> 32);
        if (t > 0 && (uint32_t)(keys[t - 1] >> 32) == node) continue;   // not the first of its node
        if (signal == 2) { s[node] = -INFINITY; continue; }
        const float sj = s[node];
        float f = 1.0f;
        for (int u = t; u < count; ++u) {
            const uint64_t ku = keys[u];
            if ((uint32_t)(ku >> 32) != node) break;
            f *= signal_factor(ne[(uint32_t)ku], alpha, signal, sj < 0.f);
        }
        s[node] = sj * f;
    }
}

// The same update by a radix sort, for up to BLOCK * ITEMS triples whose (node, triple)
// pair fits 32 bits (node < 2^(32 - kTripleBits)).  Key = node << kTripleBits | triple id.
// The triple ids ascend in the input, and a least-significant-digit radix sort is stable, so
// sorting by the node bits alone (6 bits a pass) leaves the triples of a node in ascending
// id, i.e. ascending source order -- Eq. 5's fixed order.  Per pass every wave ranks the keys of
// its own contiguous block: the lanes that hold the same digit find each other with six wave
// votes, the lowest of them adds their number to the wave's counter of that digit, and a
// block-wide scan of the (digit, wave) counters gives every key its place; three barriers a
// pass.  Then the first triple of every node multiplies that node's factors and writes its
// score once.  Two key buffers in LDS (8 bytes per triple in all).
constexpr int kTripleBits = 14;   // triple ids below 16384

template <int BLOCK, int ITEMS>
__global__ __launch_bounds__(BLOCK) void decay_radix_kernel(
    float *__restrict__ scores, int P, int count, int node_bits, const int32_t *__restrict__ nbr,
    const float *__restrict__ nbr_e, float alpha, int signal)
{
    constexpr int NW = BLOCK / kWave, NPAD = BLOCK * ITEMS;
    static_assert(NPAD <= (1 << kTripleBits), "triple ids must fit kTripleBits");
    extern __shared__ uint32_t radix_lds[];
    uint32_t *buf_a = radix_lds, *buf_b = radix_lds + NPAD;   // [NPAD] each
    __shared__ uint32_t cnt_s[NW][64];                        // keys of each digit in each wave's block
    __shared__ uint32_t wave_sum[NW];
    const int h = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int32_t *nb = nbr + (long)h * count;
    const float *ne = nbr_e + (long)h * count;
    float *s = scores + (long)h * P;
    const uint64_t below = (1ull << lane) - 1ull;

    // keys of this wave's block, entry it * 64 + lane of it: registers hold them through a pass
    uint32_t key[ITEMS];
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const int t = (wv * ITEMS + it) * kWave + lane;
        const uint32_t node = (uint32_t)nb[min(t, count - 1)];
        key[it] = t < count ? (node << kTripleBits) | (uint32_t)t : 0xffffffffu;   // padding sorts last
    }
    uint32_t *src_buf = buf_a, *dst_buf = buf_b;
    for (int shift = kTripleBits; shift < kTripleBits + node_bits; shift += 6) {
        for (int i = lane; i < 64; i += kWave) cnt_s[wv][i] = 0;
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        uint32_t place[ITEMS];   // digit << 16 | rank among the wave's keys of that digit
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) {
            const uint32_t d = (key[it] >> shift) & 63u;
            uint64_t peers = ~0ull;   // lanes whose key has the same digit
#pragma unroll
            for (int b = 0; b < 6; ++b) {
                const uint64_t v = __ballot((d >> b) & 1u);
                peers &= ((d >> b) & 1u) ? v : ~v;
            }
            const int leader = __ffsll((long long)peers) - 1;
            uint32_t base = 0;
            if (lane == leader) base = atomicAdd(&cnt_s[wv][d], (uint32_t)__popcll(peers));
            base = __shfl(base, leader, kWave);
            place[it] = (d << 16) | (base + (uint32_t)__popcll(peers & below));
        }
        __syncthreads();
        // exclusive scan of the counters in (digit, wave) order: thread t <-> digit t / NW, wave t % NW
        uint32_t run = 0;
        {
            uint32_t v = 0;
            if (tid < 64 * NW) v = cnt_s[tid % NW][tid / NW];
            uint32_t incl = v;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t u = __shfl_up(incl, o, kWave);
                if (lane >= o) incl += u;
            }
            if (lane == 63) wave_sum[wv] = incl;
            __syncthreads();
            uint32_t before = 0;
            for (int u = 0; u < wv; ++u) before += wave_sum[u];
            run = before + incl - v;
            __syncthreads();      // every counter is read before it is overwritten with its offset
            if (tid < 64 * NW) cnt_s[tid % NW][tid / NW] = run;
        }
        __syncthreads();
#pragma unroll
        for (int it = 0; it < ITEMS; ++it)
            dst_buf[cnt_s[wv][place[it] >> 16] + (place[it] & 0xffffu)] = key[it];
        __syncthreads();
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) key[it] = dst_buf[(wv * ITEMS + it) * kWave + lane];
        uint32_t *tmp = src_buf; src_buf = dst_buf; dst_buf = tmp;
    }
    // the sorted keys sit in registers (position (wv * ITEMS + it) * 64 + lane) and in src_buf
    if (src_buf == buf_a) {   // (no pass at all: node_bits = 0 cannot happen, P >= 2; keep the buffer valid)
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) buf_a[(wv * ITEMS + it) * kWave + lane] = key[it];
        __syncthreads();
    }
    const uint32_t *sorted = src_buf;
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const int pos = (wv * ITEMS + it) * kWave + lane;
        const uint32_t k = key[it];
        if (pos >= count) continue;
        const uint32_t node = k >> kTripleBits;
        if (pos > 0 && (sorted[pos - 1] >> kTripleBits) == node) continue;   // not the first of its node
        if (signal == 2) { s[node] = -INFINITY; continue; }
        const float sj = s[node];
        float f = 1.0f;
        for (int u = pos; u < count; ++u) {
            const uint32_t ku = sorted[u];
            if ((ku >> kTripleBits) != node) break;
            f *= signal_factor(ne[ku & ((1u << kTripleBits) - 1u)], alpha, signal, sj < 0.f);
        }
        s[node] = sj * f;
    }
}

// Same update without the sort, for S*m beyond the LDS capacity: sources are
// applied one after the other; inside one source the m neighbours are distinct
// nodes, so they can be updated in parallel.  Multiplying s_j by the factors one
// at a time differs from multiplying by their product only in rounding order, so
// here too the product is formed first, per node, by the lowest slot that holds it.
__global__ __launch_bounds__(1024) void decay_sequential_kernel(
    float *__restrict__ scores, int P, int S, int m, const int32_t *__restrict__ nbr,
    const float *__restrict__ nbr_e, float alpha, int signal)
{
    const int h = blockIdx.x;
    const int32_t *nb = nbr + (long)h * S * m;
    const float *ne = nbr_e + (long)h * S * m;
    float *s = scores + (long)h * P;
    // Thread (a, u) owns node j = nb[a][u] if no earlier slot a' < a lists j.
    // Neighbour lists are ascending, so membership is a binary search.
    for (long t = threadIdx.x; t < (long)S * m; t += 1024) {
        const int a = (int)(t / m);
        const int32_t j = nb[t];
        bool first = true;
        for (int b = 0; b < a && first; ++b) {
            int lo = 0, hi = m - 1;
            while (lo <= hi) {
                const int mid = (lo + hi) >> 1;
                const int32_t v = nb[(long)b * m + mid];
                if (v == j) { first = false; break; }
                if (v < j) lo = mid + 1; else hi = mid - 1;
            }
        }
        if (!first) continue;
        if (signal == 2) { s[j] = -INFINITY; continue; }
        const float sj = s[j];
        const bool neg = sj < 0.f;
        float f = signal_factor(ne[t], alpha, signal, neg);
        for (int b = a + 1; b < S; ++b) {
            int lo = 0, hi = m - 1;
            while (lo <= hi) {
                const int mid = (lo + hi) >> 1;
                const int32_t v = nb[(long)b * m + mid];
                if (v == j) { f *= signal_factor(ne[(long)b * m + mid], alpha, signal, neg); break; }
                if (v < j) lo = mid + 1; else hi = mid - 1;
            }
        }
        s[j] = sj * f;
    }
}

// Kout[q, t, :] = Kc[q, idx[q, t], :] for head q = l * H + h of a batch, same for V;
// 16 bytes per thread, rows of 16 * vec_per_row bytes.  Outputs and idx are packed
// layer after layer (layer l holds H * B_l rows).
__global__ __launch_bounds__(256) void gather_kernel(const uint4 *__restrict__ Kc,
                                                     const uint4 *__restrict__ Vc,
                                                     const int32_t *__restrict__ idx, int N,
                                                     int vec_per_row, uint4 *__restrict__ Kout,
                                                     uint4 *__restrict__ Vout, LayerPlan plan)
{
    const int q = blockIdx.y;
    const int l = q / plan.heads_per_layer, hl = q % plan.heads_per_layer;
    const int B = plan.budget[l];
    const long g = (long)blockIdx.x * 256 + threadIdx.x;
    if (g >= (long)B * vec_per_row) return;
    const int t = (int)(g / vec_per_row), c = (int)(g % vec_per_row);
    const long out_row = plan.row_off[l] + (long)hl * B + t;
    const int32_t j = idx[out_row];
    const long src = ((long)q * N + j) * vec_per_row + c;
    const long dst = out_row * vec_per_row + c;
    const uint4 *in = blockIdx.z == 0 ? Kc : Vc;
    uint4 *out = blockIdx.z == 0 ? Kout : Vout;
    out[dst] = in[src];
}

template <typename T>
__global__ __launch_bounds__(256) void copy_kernel(const T *__restrict__ src, T *__restrict__ dst,
                                                   long n)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

hipError_t launch_pool_group(const float *votes, int Hkv, int Gv, int P, int pool_kernel,
                             int pool_mode, float div, float *scores, hipStream_t st)
{
    if (pool_mode == 0 && pool_kernel <= 2 * kPoolHalo + 1) {
        if ((long)((P + 2047) / 2048) * Hkv >= 1024)
            hipLaunchKernelGGL(pool_avg_kernel<2048>, dim3((P + 2047) / 2048, Hkv), dim3(256), 0, st, votes,
                               Gv, P, pool_kernel, div, scores);
        else
            hipLaunchKernelGGL(pool_avg_kernel<256>, dim3((P + 255) / 256, Hkv), dim3(256), 0, st, votes,
                               Gv, P, pool_kernel, div, scores);
    } else {
        hipLaunchKernelGGL(pool_group_kernel, dim3((P + 255) / 256, Hkv), dim3(256), 0, st, votes, Gv,
                           P, pool_kernel, pool_mode, div, scores);
    }
    return hipGetLastError();
}

hipError_t launch_decay(float *scores, int Hkv, int P, int S, int m, const int32_t *nbr,
                        const float *nbr_e, float alpha, int signal, hipStream_t st)
{
    const long count = (long)S * m;
    long npad = 512;
    while (npad < count) npad <<= 1;
    if (count <= 2048 && P <= (1 << (32 - kTripleBits))) {
        // few edges: the two-items-per-thread sort beats the hash table by a few microseconds
        int node_bits = 1;
        while ((1L << node_bits) < P) ++node_bits;
        hipLaunchKernelGGL((decay_radix_kernel<1024, 2>), dim3(Hkv), dim3(1024), (size_t)2048 * 8, st, scores, P,
                           (int)count, node_bits, nbr, nbr_e, alpha, signal);
    } else if (count <= 4096) {
        int table_log2 = 10;
        while ((1L << table_log2) < 2 * count) ++table_log2;
        const size_t lds = ((size_t)16) << table_log2;
        if (lds > 65536 && !allow_big_lds((const void *)decay_hash_kernel, 8192 * 16)) return hipGetLastError();
        hipLaunchKernelGGL(decay_hash_kernel, dim3(Hkv), dim3(kDecayThreads), lds, st, scores, P,
                           (int)count, table_log2, nbr, nbr_e, alpha, signal);
    } else if (count <= 16384 && P <= (1 << (32 - kTripleBits))) {
        int node_bits = 1;
        while ((1L << node_bits) < P) ++node_bits;
        if (!allow_big_lds((const void *)decay_radix_kernel<1024, 16>, 16384 * 8) ||
            !allow_big_lds((const void *)decay_radix_kernel<1024, 8>, 16384 * 8))
            return hipGetLastError();
        if (count <= 8192)
            hipLaunchKernelGGL((decay_radix_kernel<1024, 8>), dim3(Hkv), dim3(1024), (size_t)8192 * 8, st, scores, P,
                               (int)count, node_bits, nbr, nbr_e, alpha, signal);
        else
            hipLaunchKernelGGL((decay_radix_kernel<1024, 16>), dim3(Hkv), dim3(1024), (size_t)16384 * 8, st, scores, P,
                               (int)count, node_bits, nbr, nbr_e, alpha, signal);
    } else if (npad <= 16384) {
        // 128 KiB of dynamic LDS
        if (npad * 8 > 65536 && !allow_big_lds((const void *)decay_sorted_kernel<1024>, 16384 * 8))
            return hipGetLastError();
        // 16 waves sort 16384 keys four times as fast as 4; 8192 keys are 64 pairs a wave
        if (npad >= 8192)
            hipLaunchKernelGGL(decay_sorted_kernel<1024>, dim3(Hkv), dim3(1024), (size_t)npad * 8, st, scores,
                               P, (int)count, (int)npad, nbr, nbr_e, alpha, signal);
        else
            hipLaunchKernelGGL(decay_sorted_kernel<256>, dim3(Hkv), dim3(256), (size_t)npad * 8, st, scores,
                               P, (int)count, (int)npad, nbr, nbr_e, alpha, signal);
    } else {
        hipLaunchKernelGGL(decay_sequential_kernel, dim3(Hkv), dim3(1024), 0, st, scores, P, S, m,
                           nbr, nbr_e, alpha, signal);
    }
    return hipGetLastError();
}

hipError_t launch_gather(const void *Kc, const void *Vc, const int32_t *idx, int heads, int N,
                         const LayerPlan &plan, int max_budget, int row_bytes, void *Kout, void *Vout,
                         hipStream_t st)
{
    const int vpr = row_bytes / 16;
    const long per_head = (long)max_budget * vpr;
    hipLaunchKernelGGL(gather_kernel, dim3((unsigned)((per_head + 255) / 256), heads, 2), dim3(256), 0,
                       st, (const uint4 *)Kc, (const uint4 *)Vc, idx, N, vpr, (uint4 *)Kout,
                       (uint4 *)Vout, plan);
    return hipGetLastError();
}

hipError_t launch_copy_i32(const int32_t *src, int32_t *dst, long n, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(copy_kernel<int32_t>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                       src, dst, n);
    return hipGetLastError();
}

hipError_t launch_copy_f32(const float *src, float *dst, long n, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(copy_kernel<float>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, src,
                       dst, n);
    return hipGetLastError();
}

}  // namespace gkv
