// C ABI of the library (include/graphkv.h): argument checks, workspace carving
// and the order in which the kernels of one layer call are enqueued.
#include "../../include/graphkv.h"
#include "kernels.hpp"

#include <math.h>
#include <atomic>
#include <mutex>
#include <vector>

namespace {

using namespace gkv;

// Scratch memory of graphkv_compress_static: device memory that belongs to the library's code
// object, so that callers which cannot allocate (HIP graph capture, serving loops) need no
// workspace.  Each GPU the library runs on holds its own copy at its own address until the
// process ends; `scratch` itself is only a host-side stand-in for those addresses.
constexpr size_t kStaticScratchBytes = GRAPHKV_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each device, once resolved

// The address of the current device's copy of `scratch` (resolved on the first call on that
// device); nullptr if it cannot be had.
void *static_scratch()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) & ~(kAlign - 1); }

// H and Hq count the heads of the whole batch (layers x heads per layer).
struct Dims {
    int L, H, Hq, G, d, N, w, P, B, S, m, T;
    bool mfma_score, mfma_cosine, filter;
    bool speculate;      // speculative rows allowed (dropped when their scratch would not fit)
    bool keep;           // neighbour lists are kept from one round to the next
    MfmaFilterPlan fp;   // geometry of the filter route (if `filter`)
    float scale;
    size_t esize;
};

// Workspace: a bump allocation of every scratch array any entry point may need.
struct Workspace {
    size_t logits, row_max, row_sum, votes, E, src, nbr, nbr_e, scores, part;
    size_t bound_hist, tau, cand, cand_cnt, overflow;
    // lists kept from one round to the next, speculative rows
    size_t src_b, nbr_b, nbr_e_b, ext, new_src, n_new, sel_row, sel_pos, n_sel, spec_bad;
    size_t total;
};

// The MFMA kernels cover bf16 keys with d = 128.  Scoring additionally needs the
// stacked query rows G*w to fill whole 32-row MFMA blocks (at most 256 rows: 256 rows
// in one workgroup, other counts beyond 128 in parts of 128); per-query-head votes (max pooling) need w itself to be a multiple
// of 32.
bool mfma_cosine_ok(const graphkv_params *p)
{
    // (fewer than 2^24 rows: the tile loads address a head's rows with 32-bit byte offsets)
    return p->impl == GRAPHKV_IMPL_AUTO && p->dtype == GRAPHKV_BF16 && p->head_dim == 128 &&
           p->n_tokens < (1 << 24);
}

bool mfma_score_ok(const graphkv_params *p)
{
    if (!mfma_cosine_ok(p) || p->n_kv_heads < 1 || p->n_q_heads < p->n_kv_heads) return false;
    const int rows = (p->n_q_heads / p->n_kv_heads) * p->window;
    if (rows % 32 != 0 || rows > 256) return false;
    // per-query-head votes: a query head's rows must not straddle a 128-row part
    if (p->pool_mode == GRAPHKV_POOL_MAX && (p->window % 32 != 0 || (rows > 128 && 128 % p->window != 0)))
        return false;
    return true;
}

// Constraints common to all entry points (see graphkv_params in the header).
bool base_ok(const graphkv_params *p)
{
    if (!p) return false;
    if (p->n_kv_heads < 1 || p->n_kv_heads > 65535) return false;
    if (p->head_dim < 8 || p->head_dim % 8 || p->head_dim > 512) return false;
    if (p->window < 1 || p->n_tokens <= p->window) return false;
    if (p->dtype != GRAPHKV_FP32 && p->dtype != GRAPHKV_BF16) return false;
    if (p->impl != GRAPHKV_IMPL_AUTO && p->impl != GRAPHKV_IMPL_GENERIC) return false;
    if (p->rounds < 0) return false;
    if (p->signal < 0 || p->signal > 2) return false;
    if (p->edges < GRAPHKV_EDGES_KK || p->edges > GRAPHKV_EDGES_VV) return false;
    if (p->scorer != GRAPHKV_SCORER_ATTENTION && p->scorer != GRAPHKV_SCORER_KNORM) return false;
    if (!(p->decay >= 0.f && p->decay <= 1.f)) return false;
    if (p->reselect != 0 && p->reselect != 1) return false;
    if (p->rounds > 0) {
        const long P = (long)p->n_tokens - p->window;
        if (p->n_sources < 1 || p->n_sources > P || p->n_sources > 65535) return false;
        if (p->n_neighbors < 1 || p->n_neighbors > P - 1) return false;
    }
    return true;
}

bool score_ok(const graphkv_params *p)
{
    if (p->n_q_heads < p->n_kv_heads || p->n_q_heads % p->n_kv_heads) return false;
    if ((long)p->n_q_heads * p->window > 65535 * 16L) return false;
    if (p->pool_kernel < 1 || p->pool_kernel % 2 == 0) return false;
    if (p->pool_mode != GRAPHKV_POOL_AVG && p->pool_mode != GRAPHKV_POOL_MAX) return false;
    if (!(p->softmax_scale >= 0.f) || isinf(p->softmax_scale)) return false;
    return true;
}

bool budget_ok(const graphkv_params *p)
{
    return p->budget > p->window && p->budget <= p->n_tokens;
}

Dims dims_of(const graphkv_params *p, int n_layers = 1, bool speculate = true)
{
    Dims D;
    D.L = n_layers;
    D.H = p->n_kv_heads * n_layers;
    D.Hq = (p->n_q_heads > 0 ? p->n_q_heads : p->n_kv_heads) * n_layers;
    D.G = D.Hq / D.H > 0 ? D.Hq / D.H : 1;
    D.d = p->head_dim;
    D.N = p->n_tokens;
    D.w = p->window;
    D.P = D.N - D.w;
    D.B = p->budget;
    D.S = p->rounds > 0 ? p->n_sources : 0;
    D.m = p->rounds > 0 ? p->n_neighbors : 0;
    D.T = p->rounds;
    D.mfma_score = mfma_score_ok(p);
    D.mfma_cosine = mfma_cosine_ok(p);
    D.filter = D.mfma_cosine && D.T > 0 && mfma_filter_applies(D.P, D.m);
    // The neighbourhood of a source depends on the keys alone (Eq. 1, Eq. 3), not on the
    // scores: with re-picked sources the lists of returning sources are kept.
    D.speculate = speculate;
    D.keep = D.filter && D.T > 1 && p->reselect && source_reuse_applies(D.S);
    D.fp = D.filter ? mfma_filter_plan(D.H, D.P, D.S, D.m, D.keep, speculate) : MfmaFilterPlan{};
    D.scale = p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / sqrtf((float)D.d);
    D.esize = p->dtype == GRAPHKV_FP32 ? 4 : 2;
    return D;
}

Workspace carve(const graphkv_params *p, const Dims &D)
{
    Workspace W;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes > 0 ? bytes : 1); return o; };
    const size_t rows = (size_t)D.Hq * D.w;
    const bool scoring = p->scorer == GRAPHKV_SCORER_ATTENTION && p->n_q_heads >= p->n_kv_heads &&
                         p->pool_kernel >= 1;
    W.logits = take(!D.mfma_score && scoring ? rows * D.N * 4 : 0);
    W.row_max = take(rows * 4);
    W.row_sum = take(rows * 4);
    // votes per query head (or row group); not needed when pass B pools and groups them itself
    const bool votes_stay_in_lds = D.mfma_score && scoring &&
        mfma_score_fuses_pool(D.G, D.w, p->pool_mode == GRAPHKV_POOL_MAX, p->pool_kernel);
    W.votes = take(scoring && !votes_stay_in_lds ? (size_t)D.Hq * D.P * 4 : 0);
    // the dense edge block [heads, S, P] of the routes that materialise it; on the filter route
    // only the scratch rows of the workgroups that redo overflowed heads
    W.E = take(D.filter ? redo_rows_scratch_bytes(D.H, D.S, D.P) : (size_t)D.H * D.S * D.P * 4);
    W.src = take((size_t)D.H * D.S * 4);
    W.nbr = take((size_t)D.H * D.S * D.m * 4);
    W.nbr_e = take((size_t)D.H * D.S * D.m * 4);
    W.scores = take((size_t)D.H * D.P * 4);
    W.part = take(D.mfma_score ? mfma_score_plan(D.H, D.G * D.w, D.N).part_bytes : 0);
    const MfmaFilterPlan &g = D.fp;
    const size_t frows = D.filter ? (size_t)D.H * g.pitch : 0;   // rows of the per-row buffers
    W.tau = take(frows * 4);
    W.bound_hist = take(D.filter ? mfma_bound_scratch_bytes(D.H, D.P, g) : 0);
    W.cand = take(frows * g.chunks * g.slice_cap * 8);
    W.cand_cnt = take(frows * g.chunks * 4);
    W.overflow = take((size_t)D.H * 4);
    const bool keep = D.keep;
    W.src_b = take(keep ? (size_t)D.H * D.S * 4 : 0);
    W.nbr_b = take(keep ? (size_t)D.H * D.S * D.m * 4 : 0);
    W.nbr_e_b = take(keep ? (size_t)D.H * D.S * D.m * 4 : 0);
    W.ext = take(keep ? (size_t)D.H * (g.S + g.X) * 4 : 0);
    W.new_src = take(keep ? (size_t)D.H * D.S * 4 : 0);
    W.n_new = take(keep ? (size_t)D.H * 4 : 0);
    W.sel_row = take(keep ? (size_t)D.H * D.S * 4 : 0);
    W.sel_pos = take(keep ? (size_t)D.H * D.S * 4 : 0);
    W.n_sel = take(keep ? (size_t)D.H * 4 : 0);
    W.spec_bad = take(keep ? (size_t)D.H * 4 : 0);
    W.total = off;
    return W;
}

inline bool aligned16(const void *ptr) { return ptr && ((uintptr_t)ptr & 15u) == 0; }
inline bool aligned4(const void *ptr) { return ptr && ((uintptr_t)ptr & 3u) == 0; }

int32_t check_ws(const Workspace &W, const void *ws, size_t ws_bytes)
{
    if (!ws || ((uintptr_t)ws & (kAlign - 1)) || ws_bytes < W.total) return GRAPHKV_EWORKSPACE;
    return GRAPHKV_OK;
}

// ---- optional per-kernel timing (graphkv_profile_begin / _end) ----------------
// While profiling is on, every kernel launch is bracketed by two HIP events on
// the caller's stream.  Process-wide (one recording at a time, whichever host thread
// launches); the records are guarded by a mutex.
struct ProfRec { int id; hipEvent_t e0, e1; };
struct Profiler {
    std::atomic<bool> on{false};
    std::mutex mu;
    std::vector<hipEvent_t> pool;
    size_t used = 0;
    std::vector<ProfRec> recs;
    hipEvent_t next()
    {
        if (used == pool.size()) {
            hipEvent_t e = nullptr;
            if (hipEventCreate(&e) != hipSuccess) return nullptr;
            pool.push_back(e);
        }
        return pool[used++];
    }
};
Profiler g_prof;

const char *const kKernelNames[GRAPHKV_N_KERNELS] = {
    "score_stats", "score_votes", "pool_group", "topk_sources", "cosine", "topk_neighbors",
    "decay", "topk_final", "gather", "generic_logits", "generic_votes", "generic_cosine",
    "knorm", "copy", "cosine_bound", "cosine_filter", "nbr_select",
    "redo_rows", "match_sources", "topk_sources_later", "cosine_bound_new", "cosine_filter_new",
    "nbr_select_later"};

#define GKV_LAUNCH(id, expr)                                              \
    do {                                                                  \
        hipEvent_t e0_ = nullptr, e1_ = nullptr;                          \
        const bool prof_ = g_prof.on.load(std::memory_order_relaxed);     \
        if (prof_) {                                                      \
            std::lock_guard<std::mutex> lock_(g_prof.mu);                 \
            e0_ = g_prof.next();                                          \
            e1_ = g_prof.next();                                          \
            if (e0_ && e1_) (void)hipEventRecord(e0_, st);                \
        }                                                                 \
        const hipError_t err_ = (expr);                                   \
        if (prof_ && e0_ && e1_) {                                        \
            std::lock_guard<std::mutex> lock_(g_prof.mu);                 \
            (void)hipEventRecord(e1_, st);                                \
            g_prof.recs.push_back({(id), e0_, e1_});                      \
        }                                                                 \
        if (err_ != hipSuccess) return GRAPHKV_EHIP;                      \
    } while (0)

template <typename T> T *at(void *ws, size_t off) { return reinterpret_cast<T *>((char *)ws + off); }

int32_t run_score(const graphkv_params *p, const Dims &D, const Workspace &W, const void *Kc,
                  const void *Qw, float *scores, void *ws, hipStream_t st)
{
    float *votes = at<float>(ws, W.votes);
    if (D.mfma_score) {
        const int per_q = p->pool_mode == GRAPHKV_POOL_MAX;
        GKV_LAUNCH(GRAPHKV_K_SCORE_STATS, launch_mfma_score_stats(Kc, Qw, D.H, D.Hq, D.N, D.w, D.scale,
                                                                  at<float>(ws, W.part), st));
        if (mfma_score_fuses_pool(D.G, D.w, per_q, p->pool_kernel)) {
            // average pooling and the mean over the group happen inside pass B
            GKV_LAUNCH(GRAPHKV_K_SCORE_VOTES,
                       launch_mfma_score_votes(Kc, Qw, D.H, D.Hq, D.N, D.w, D.scale, per_q, p->pool_kernel,
                                               at<float>(ws, W.part), scores, st));
            return GRAPHKV_OK;
        }
        GKV_LAUNCH(GRAPHKV_K_SCORE_VOTES,
                   launch_mfma_score_votes(Kc, Qw, D.H, D.Hq, D.N, D.w, D.scale, per_q, 0,
                                           at<float>(ws, W.part), votes, st));
        GKV_LAUNCH(GRAPHKV_K_POOL,
                   launch_pool_group(votes, D.H, mfma_score_vote_rows(D.G, D.w, per_q), D.P, p->pool_kernel,
                                     p->pool_mode, (float)D.G, scores, st));
        return GRAPHKV_OK;
    }
    GKV_LAUNCH(GRAPHKV_K_GENERIC_LOGITS, launch_generic_logits(Kc, Qw, p->dtype, D.H, D.Hq, D.d, D.N, D.w, D.scale,
                                  at<float>(ws, W.logits), at<float>(ws, W.row_max),
                                  at<float>(ws, W.row_sum), st));
    GKV_LAUNCH(GRAPHKV_K_GENERIC_VOTES, launch_generic_votes(at<float>(ws, W.logits), at<float>(ws, W.row_max),
                                 at<float>(ws, W.row_sum), D.Hq, D.N, D.w, votes, st));
    GKV_LAUNCH(GRAPHKV_K_POOL, launch_pool_group(votes, D.H, D.G, D.P, p->pool_kernel, p->pool_mode, (float)D.G,
                              scores, st));
    return GRAPHKV_OK;
}

bool propagation_is_noop(const graphkv_params *p)
{
    return p->rounds == 0 || (p->decay == 0.f && p->signal != GRAPHKV_SIGNAL_EVICTED);
}

// Ac: tensor of the sources' rows, Kc: tensor of the other nodes' rows (Eq. 1: both the keys).
int32_t run_propagate(const graphkv_params *p, const Dims &D, const Workspace &W, const void *Ac,
                      const void *Kc, float *scores, int32_t *dbg_src, int32_t *dbg_nbr, float *dbg_e, void *ws,
                      hipStream_t st)
{
    if (propagation_is_noop(p)) return GRAPHKV_OK;
    const size_t n_src = (size_t)D.H * D.S, n_nbr = n_src * D.m;
    float *E = at<float>(ws, W.E);
    int32_t *src0 = dbg_src ? dbg_src : at<int32_t>(ws, W.src);
    int32_t *nbr0 = dbg_nbr ? dbg_nbr : at<int32_t>(ws, W.nbr);
    float *e0 = dbg_e ? dbg_e : at<float>(ws, W.nbr_e);
    // A source that comes back in the next round keeps its list; of the others, those that
    // were speculative rows of the first round's pass have their candidates waiting, and only
    // the rest take the bound and filter passes again.  The lists of two consecutive rounds
    // live in two buffers that take turns.
    const bool keep = D.keep;
    const MfmaFilterPlan &g = D.fp;
    const int32_t *prev_src = nullptr, *prev_nbr = nullptr;
    const float *prev_e = nullptr;
    for (int t = 0; t < D.T; ++t) {
        int32_t *src = src0, *nbr = nbr0;
        float *ev = e0;
        if (t == 0 || p->reselect) {
            if (keep && (t & 1)) {
                src = at<int32_t>(ws, W.src_b);
                nbr = at<int32_t>(ws, W.nbr_b);
                ev = at<float>(ws, W.nbr_e_b);
            }
            if (dbg_src) src = dbg_src + t * n_src;
            if (dbg_nbr) nbr = dbg_nbr + t * n_nbr;
            if (dbg_e) ev = dbg_e + t * n_nbr;
            if (D.filter) {
                // Eq. 1 + Eq. 3 in one streaming pass over the keys: a bound per source from a
                // strided sample that at least m of its edges reach, then only edges above it are kept.
                float *tau = at<float>(ws, W.tau);
                int32_t *cnt = at<int32_t>(ws, W.cand_cnt), *ovf = at<int32_t>(ws, W.overflow);
                void *cand = at<char>(ws, W.cand);
                int32_t *ext = at<int32_t>(ws, W.ext);
                if (!(keep && prev_src)) {
                    // Eq. 2: source nodes; with speculative rows also the nodes ranked right behind
                    const int32_t *lst = src;
                    if (g.X > 0) {
                        GKV_LAUNCH(GRAPHKV_K_TOPK_SOURCES,
                                   launch_pick_sources(scores, D.P, D.P, D.H, D.S, g.X, src, ext, st));
                        lst = ext;
                    } else {
                        GKV_LAUNCH(GRAPHKV_K_TOPK_SOURCES,
                                   launch_topk_rows(scores, D.P, D.P, D.H, D.S, src, D.S, nullptr, 0, nullptr, 0, 0,
                                                    nullptr, 1, st));
                    }
                    GKV_LAUNCH(GRAPHKV_K_COSINE_BOUND,
                               launch_mfma_cosine_bound(Ac, Kc, D.H, D.N, D.P, D.m, g, true, lst, nullptr,
                                                        at<char>(ws, W.bound_hist), tau, ovf, st));
                    GKV_LAUNCH(GRAPHKV_K_COSINE_FILTER,
                               launch_mfma_cosine_filter(Ac, Kc, D.H, D.N, D.P, D.m, g, true, lst, nullptr, tau, cand,
                                                         cnt, ovf, st));
                    GKV_LAUNCH(GRAPHKV_K_NBR_SELECT,
                               launch_nbr_select(cand, cnt, ovf, src, D.H, D.m, g, nullptr, nbr, ev, st));
                    // heads whose lists overflowed are redone row by row, exactly
                    GKV_LAUNCH(GRAPHKV_K_REDO_ROWS,
                               launch_redo_rows(Ac, Kc, D.H, D.N, D.P, D.S, D.m, src, ovf, E, nbr, ev, st));
                } else {
                    GKV_LAUNCH(GRAPHKV_K_TOPK_SOURCES_LATER,
                               launch_topk_rows(scores, D.P, D.P, D.H, D.S, src, D.S, nullptr, 0, nullptr, 0, 0,
                                                nullptr, 1, st));
                    int32_t *new_src = at<int32_t>(ws, W.new_src), *n_new = at<int32_t>(ws, W.n_new);
                    const SelectRows sel{at<int32_t>(ws, W.n_sel), at<int32_t>(ws, W.sel_row),
                                         at<int32_t>(ws, W.sel_pos)};
                    GKV_LAUNCH(GRAPHKV_K_MATCH_SOURCES,
                               launch_match_sources(prev_src, src, D.H, D.m, g, prev_nbr, prev_e, nbr, ev, ext,
                                                    at<int32_t>(ws, W.spec_bad), ovf, t == 1, new_src, n_new,
                                                    at<int32_t>(ws, W.sel_row), at<int32_t>(ws, W.sel_pos),
                                                    at<int32_t>(ws, W.n_sel), st));
                    // new sources without a kept list (usually none): bound and filter passes
                    // that return at once for heads that have none
                    GKV_LAUNCH(GRAPHKV_K_COSINE_BOUND_NEW,
                               launch_mfma_cosine_bound(Ac, Kc, D.H, D.N, D.P, D.m, g, false, new_src, n_new,
                                                        at<char>(ws, W.bound_hist), tau, ovf, st));
                    GKV_LAUNCH(GRAPHKV_K_COSINE_FILTER_NEW,
                               launch_mfma_cosine_filter(Ac, Kc, D.H, D.N, D.P, D.m, g, false, new_src, n_new, tau,
                                                         cand, cnt, ovf, st));
                    GKV_LAUNCH(GRAPHKV_K_NBR_SELECT_LATER,
                               launch_nbr_select(cand, cnt, ovf, src, D.H, D.m, g, &sel, nbr, ev, st));
                    GKV_LAUNCH(GRAPHKV_K_REDO_ROWS,
                               launch_redo_rows(Ac, Kc, D.H, D.N, D.P, D.S, D.m, src, ovf, E, nbr, ev, st));
                }
            } else {
                // Eq. 2: source nodes
                GKV_LAUNCH(GRAPHKV_K_TOPK_SOURCES,
                           launch_topk_rows(scores, D.P, D.P, D.H, D.S, src, D.S, nullptr, 0, nullptr, 0, 0,
                                            nullptr, 1, st));
                // Eq. 1: edges from every source to every node
                if (D.mfma_cosine)
                    GKV_LAUNCH(GRAPHKV_K_COSINE, launch_mfma_cosine(Ac, Kc, D.H, D.N, D.P, D.S, src, E, nullptr, st));
                else
                    GKV_LAUNCH(GRAPHKV_K_GENERIC_COSINE,
                               launch_generic_cosine(Ac, Kc, p->dtype, D.H, D.d, D.N, D.P, D.S, src, E, st));
                // Eq. 3: neighbourhoods
                GKV_LAUNCH(GRAPHKV_K_TOPK_NEIGHBORS,
                           launch_topk_rows(E, D.P, D.P, D.H * D.S, D.m, nbr, D.m, ev, D.m, nullptr, 0, 0,
                                            nullptr, 1, st));
            }
        } else {
            if (dbg_src) GKV_LAUNCH(GRAPHKV_K_COPY, launch_copy_i32(src0, dbg_src + t * n_src, (long)n_src, st));
            if (dbg_nbr) GKV_LAUNCH(GRAPHKV_K_COPY, launch_copy_i32(nbr0, dbg_nbr + t * n_nbr, (long)n_nbr, st));
            if (dbg_e) GKV_LAUNCH(GRAPHKV_K_COPY, launch_copy_f32(e0, dbg_e + t * n_nbr, (long)n_nbr, st));
        }
        // Eq. 5: one round of the signal
        GKV_LAUNCH(GRAPHKV_K_DECAY, launch_decay(scores, D.H, D.P, D.S, D.m, nbr, ev, p->decay, p->signal, st));
        prev_src = src;
        prev_nbr = nbr;
        prev_e = ev;
    }
    return GRAPHKV_OK;
}

// Budgets of the layers of a batch and where each layer's rows start in the packed outputs.
LayerPlan make_plan(const graphkv_params *p, int n_layers, const int32_t *budgets, int *max_budget)
{
    LayerPlan plan{};
    plan.heads_per_layer = p->n_kv_heads;
    int64_t rows = 0;
    int mx = 0;
    for (int l = 0; l < n_layers; ++l) {
        const int B = budgets ? budgets[l] : p->budget;
        plan.budget[l] = B;
        plan.row_off[l] = rows;
        rows += (int64_t)p->n_kv_heads * B;
        if (B > mx) mx = B;
    }
    if (max_budget) *max_budget = mx;
    return plan;
}

int32_t run_select(const Dims &D, const LayerPlan &plan, const float *scores, int32_t *idx,
                   hipStream_t st)
{
    GKV_LAUNCH(GRAPHKV_K_TOPK_FINAL, launch_topk_final(scores, D.P, D.H, plan, D.w, idx, st));
    return GRAPHKV_OK;
}

// The whole pass for a batch of n_layers contiguous layers (n_layers <= kMaxLayers).
int32_t run_compress(const graphkv_params *p, int n_layers, bool speculate, const int32_t *budgets, const void *Kc,
                     const void *Vc, const void *Qw, void *Kout, void *Vout, int32_t *idx,
                     float *scores_out, void *ws, hipStream_t st)
{
    const Dims D = dims_of(p, n_layers, speculate);
    const Workspace W = carve(p, D);
    int max_budget = 0;
    const LayerPlan plan = make_plan(p, n_layers, budgets, &max_budget);
    float *scores = scores_out ? scores_out : at<float>(ws, W.scores);
    if (p->scorer == GRAPHKV_SCORER_KNORM)
        GKV_LAUNCH(GRAPHKV_K_KNORM, launch_knorm(Kc, p->dtype, D.H, D.d, D.N, D.P, scores, st));
    else if (int32_t rc = run_score(p, D, W, Kc, Qw, scores, ws, st))
        return rc;
    const void *edge_src = p->edges == GRAPHKV_EDGES_VV ? Vc : Kc;
    const void *edge_nbr = p->edges == GRAPHKV_EDGES_KK ? Kc : Vc;
    if (int32_t rc = run_propagate(p, D, W, edge_src, edge_nbr, scores, nullptr, nullptr, nullptr, ws, st))
        return rc;
    if (int32_t rc = run_select(D, plan, scores, idx, st)) return rc;
    GKV_LAUNCH(GRAPHKV_K_GATHER, launch_gather(Kc, Vc, idx, D.H, D.N, plan, max_budget,
                                               (int)(D.d * D.esize), Kout, Vout, st));
    return GRAPHKV_OK;
}

// Layers that go through the kernels together: at most kMaxLayers and 65535 heads, and fewer
// while the scratch memory of a group would exceed 2000 MiB (long prompts: the candidate lists
// and vote rows grow with the number of heads in flight).
constexpr size_t kGroupScratchCap = (size_t)2000 << 20;
// The speculative rows of the filter route cost scratch too.  A smaller group that keeps them
// beats a larger one without (later rounds then stream no keys again), as long as the group
// still has 64 heads or more to fill the chip with; below that they are dropped before a
// group is made smaller still.
Dims group_dims(const graphkv_params *p, int n_layers)
{
    const int g0 = n_layers < kMaxLayers ? n_layers : kMaxLayers;
    for (int speculate = 1; speculate >= 0; --speculate) {
        for (int g = g0;; g = (g + 1) / 2) {
            const bool fits_heads = (long)p->n_kv_heads * g <= 65535;
            if (speculate && g < g0 && (long)p->n_kv_heads * g < 64) break;
            if (fits_heads) {
                const Dims D = dims_of(p, g, speculate != 0);
                if (carve(p, D).total <= kGroupScratchCap) return D;
            }
            if (g == 1) break;
        }
    }
    return dims_of(p, 1, false);
}

bool budgets_ok(const graphkv_params *p, int n_layers, const int32_t *budgets)
{
    for (int l = 0; l < n_layers; ++l) {
        const int B = budgets ? budgets[l] : p->budget;
        if (B <= p->window || B > p->n_tokens) return false;
    }
    return true;
}

}  // namespace

extern "C" {

size_t graphkv_workspace_bytes(const graphkv_params *p)
{
    return graphkv_workspace_bytes_batched(p, 1);
}

int32_t graphkv_uses_mfma(const graphkv_params *p)
{
    if (!base_ok(p) || !score_ok(p)) return 0;
    return mfma_score_ok(p) ? 1 : 0;
}

int32_t graphkv_score(const graphkv_params *p, const void *Kc, const void *Qw, float *scores,
                      void *ws, size_t ws_bytes, void *stream)
{
    if (!base_ok(p) || !score_ok(p)) return GRAPHKV_EINVAL;
    if (!aligned16(Kc) || !aligned16(Qw) || !aligned4(scores)) return GRAPHKV_EINVAL;
    // this call is the attention scorer whatever `scorer` says: its scratch is carved (and the
    // caller's workspace checked) for that
    graphkv_params q = *p;
    q.scorer = GRAPHKV_SCORER_ATTENTION;
    const Dims D = group_dims(&q, 1);
    const Workspace W = carve(&q, D);
    if (int32_t rc = check_ws(W, ws, ws_bytes)) return rc;
    return run_score(&q, D, W, Kc, Qw, scores, ws, (hipStream_t)stream);
}

int32_t graphkv_score_knorm(const graphkv_params *p, const void *Kc, float *scores, void *ws,
                            size_t ws_bytes, void *stream)
{
    (void)ws; (void)ws_bytes;
    if (!base_ok(p)) return GRAPHKV_EINVAL;
    if (!aligned16(Kc) || !aligned4(scores)) return GRAPHKV_EINVAL;
    const Dims D = dims_of(p);
    hipStream_t st = (hipStream_t)stream;
    GKV_LAUNCH(GRAPHKV_K_KNORM, launch_knorm(Kc, p->dtype, D.H, D.d, D.N, D.P, scores, st));
    return GRAPHKV_OK;
}

int32_t graphkv_propagate_edges(const graphkv_params *p, const void *Ac, const void *Bc, float *scores,
                                int32_t *dbg_src, int32_t *dbg_nbr, float *dbg_e, void *ws,
                                size_t ws_bytes, void *stream)
{
    if (!base_ok(p)) return GRAPHKV_EINVAL;
    if (!aligned16(Ac) || !aligned16(Bc) || !aligned4(scores)) return GRAPHKV_EINVAL;
    if ((dbg_src && !aligned4(dbg_src)) || (dbg_nbr && !aligned4(dbg_nbr)) ||
        (dbg_e && !aligned4(dbg_e)))
        return GRAPHKV_EINVAL;
    const Dims D = group_dims(p, 1);
    const Workspace W = carve(p, D);
    if (int32_t rc = check_ws(W, ws, ws_bytes)) return rc;
    return run_propagate(p, D, W, Ac, Bc, scores, dbg_src, dbg_nbr, dbg_e, ws,
                         (hipStream_t)stream);
}

int32_t graphkv_propagate(const graphkv_params *p, const void *Kc, float *scores, int32_t *dbg_src,
                          int32_t *dbg_nbr, float *dbg_e, void *ws, size_t ws_bytes, void *stream)
{
    return graphkv_propagate_edges(p, Kc, Kc, scores, dbg_src, dbg_nbr, dbg_e, ws, ws_bytes, stream);
}

int32_t graphkv_select(const graphkv_params *p, const float *scores, int32_t *idx, void *ws,
                       size_t ws_bytes, void *stream)
{
    (void)ws; (void)ws_bytes;
    if (!base_ok(p) || !budget_ok(p)) return GRAPHKV_EINVAL;
    if (!aligned4(scores) || !aligned4(idx)) return GRAPHKV_EINVAL;
    const Dims D = dims_of(p);
    return run_select(D, make_plan(p, 1, nullptr, nullptr), scores, idx, (hipStream_t)stream);
}

int32_t graphkv_compress(const graphkv_params *p, const void *Kc, const void *Vc, const void *Qw,
                         void *Kout, void *Vout, int32_t *idx, float *scores_out, void *ws,
                         size_t ws_bytes, void *stream)
{
    return graphkv_compress_batched(p, 1, nullptr, Kc, Vc, Qw, Kout, Vout, idx, scores_out, ws,
                                    ws_bytes, stream);
}

int32_t graphkv_compress_static(const graphkv_params *p, const void *Kc, const void *Vc, const void *Qw,
                                void *Kout, void *Vout, int32_t *idx, float *scores_out, void *stream)
{
    const size_t need = graphkv_workspace_bytes(p);   // 0: invalid params
    if (need == 0) return GRAPHKV_EINVAL;
    if (need > kStaticScratchBytes) return GRAPHKV_ESCRATCH;
    // (the pointer checks of the call below come before the address is resolved)
    if (!aligned16(Kc) || !aligned16(Vc) || !aligned16(Kout) || !aligned16(Vout) || !aligned4(idx))
        return GRAPHKV_EINVAL;
    void *ws = static_scratch();
    if (!ws) return GRAPHKV_EHIP;
    return graphkv_compress_batched(p, 1, nullptr, Kc, Vc, Qw, Kout, Vout, idx, scores_out, ws,
                                    kStaticScratchBytes, stream);
}

size_t graphkv_workspace_bytes_batched(const graphkv_params *p, int32_t n_layers)
{
    if (!base_ok(p) || n_layers < 1) return 0;
    return carve(p, group_dims(p, n_layers)).total;
}

int32_t graphkv_compress_batched(const graphkv_params *p, int32_t n_layers, const int32_t *budgets,
                                 const void *Kc, const void *Vc, const void *Qw, void *Kout,
                                 void *Vout, int32_t *idx, float *scores_out, void *ws,
                                 size_t ws_bytes, void *stream)
{
    if (!base_ok(p) || n_layers < 1) return GRAPHKV_EINVAL;
    const bool knorm = p->scorer == GRAPHKV_SCORER_KNORM;   // reads no queries: Qw may be NULL
    if (!knorm && !score_ok(p)) return GRAPHKV_EINVAL;
    if (!budgets_ok(p, n_layers, budgets)) return GRAPHKV_EINVAL;
    if (!aligned16(Kc) || !aligned16(Vc) || (!knorm && !aligned16(Qw)) || !aligned16(Kout) ||
        !aligned16(Vout) || !aligned4(idx))
        return GRAPHKV_EINVAL;
    if (scores_out && !aligned4(scores_out)) return GRAPHKV_EINVAL;
    const Dims DG = group_dims(p, n_layers);   // layers per group, and whether its filter passes speculate
    const int group = DG.L;
    const Workspace W = carve(p, DG);
    if (int32_t rc = check_ws(W, ws, ws_bytes)) return rc;
    hipStream_t st = (hipStream_t)stream;
    const size_t esize = p->dtype == GRAPHKV_FP32 ? 4 : 2;
    const size_t kv_layer = (size_t)p->n_kv_heads * p->n_tokens * p->head_dim * esize;
    const size_t q_layer = (size_t)p->n_q_heads * p->window * p->head_dim * esize;
    const size_t s_layer = (size_t)p->n_kv_heads * (p->n_tokens - p->window);
    size_t out_rows = 0;   // rows of Kout / Vout / idx written so far
    for (int l0 = 0; l0 < n_layers; l0 += group) {
        const int nl = n_layers - l0 < group ? n_layers - l0 : group;
        const int32_t *bl = budgets ? budgets + l0 : nullptr;
        const int32_t rc = run_compress(
            p, nl, DG.speculate, bl, (const char *)Kc + l0 * kv_layer, (const char *)Vc + l0 * kv_layer,
            Qw ? (const char *)Qw + l0 * q_layer : nullptr, (char *)Kout + out_rows * p->head_dim * esize,
            (char *)Vout + out_rows * p->head_dim * esize, idx + out_rows,
            scores_out ? scores_out + l0 * s_layer : nullptr, ws, st);
        if (rc) return rc;
        for (int l = 0; l < nl; ++l) out_rows += (size_t)p->n_kv_heads * (bl ? bl[l] : p->budget);
    }
    return GRAPHKV_OK;
}

int32_t graphkv_profile_begin(void)
{
    std::lock_guard<std::mutex> lock(g_prof.mu);
    g_prof.used = 0;
    g_prof.recs.clear();
    g_prof.on = true;
    return GRAPHKV_OK;
}

int32_t graphkv_profile_end(double *ms, int64_t *launches)
{
    g_prof.on = false;
    std::lock_guard<std::mutex> lock(g_prof.mu);
    for (int i = 0; i < GRAPHKV_N_KERNELS; ++i) {
        if (ms) ms[i] = 0.0;
        if (launches) launches[i] = 0;
    }
    int32_t rc = GRAPHKV_OK;
    for (const ProfRec &r : g_prof.recs) {
        float t = 0.f;
        if (hipEventSynchronize(r.e1) != hipSuccess || hipEventElapsedTime(&t, r.e0, r.e1) != hipSuccess) {
            rc = GRAPHKV_EHIP;
            continue;
        }
        if (ms) ms[r.id] += t;
        if (launches) launches[r.id] += 1;
    }
    g_prof.recs.clear();
    g_prof.used = 0;
    return rc;
}

const char *graphkv_kernel_name(int32_t id)
{
    return (id >= 0 && id < GRAPHKV_N_KERNELS) ? kKernelNames[id] : "unknown";
}

const char *graphkv_strerror(int32_t code)
{
    switch (code) {
        case GRAPHKV_OK: return "ok";
        case GRAPHKV_EINVAL: return "invalid argument (a graphkv_params constraint is violated or a pointer is NULL/misaligned)";
        case GRAPHKV_EWORKSPACE: return "workspace is NULL, misaligned or smaller than graphkv_workspace_bytes()";
        case GRAPHKV_EHIP: return "a HIP kernel launch failed";
        case GRAPHKV_ESCRATCH: return "the problem needs more scratch memory than graphkv_compress_static's built-in buffer holds (use graphkv_compress with a workspace)";
        default: return "unknown graphkv error code";
    }
}

}  // extern "C"
