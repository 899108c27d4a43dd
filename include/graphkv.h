/*
 * graphkv.h -- C ABI of the MI355X (gfx950) GraphKV eviction library.
 *
 * One call handles one transformer layer: the paper states the problem per
 * layer, with key/value matrices K^l, V^l of n x d and a layer budget k_l
 * (Methodology, "Problem Formulation").  The KV heads of the layer are
 * independent instances of that problem and are processed together.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers, contiguous, row-major with the
 *     head dimension innermost, 16-byte aligned.  The params struct and the
 *     returned strings live on the HOST.
 *   - The caller owns every buffer.  The library allocates nothing, never
 *     synchronises and never copies to the host.  It keeps no state between calls
 *     except which kernels have had their one-time opt-in to large shared memory
 *     (process-wide, guarded by a mutex: first calls may come from several host
 *     threads) and the measurement aid at the end of this header.
 *     All work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream).  Inputs are read-only unless stated otherwise.
 *   - `ws` is scratch memory of at least graphkv_workspace_bytes(params) bytes,
 *     256-byte aligned; its contents are undefined before and after a call.
 *     Two calls that overlap in time need two workspaces.
 *   - Return value: GRAPHKV_OK (0) or a negative code.  Arguments are checked
 *     on the host before anything is enqueued: on GRAPHKV_EINVAL or
 *     GRAPHKV_EWORKSPACE nothing has run.  GRAPHKV_EHIP reports a failed
 *     launch (earlier launches of the same call may already be queued).
 *   - Results are deterministic: the same inputs give byte-identical outputs.
 *   - NaN inputs are not supported (selection order is then unspecified).
 *
 * Symbols: N tokens in the layer's cache, of which the last w are the
 * observation window; P = N - w prefix tokens are the graph nodes; H_kv / H_q
 * key-value / query heads, G = H_q / H_kv; d head dimension; B retained tokens
 * per head (window included); S source nodes (k in Eq. 2); m neighbours per
 * source (Eq. 3); T propagation rounds (Eq. 5); alpha decay strength.
 */
#ifndef GRAPHKV_H
#define GRAPHKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    GRAPHKV_OK = 0,
    GRAPHKV_EINVAL = -1,      /* a constraint listed below is violated, or a required pointer is NULL/misaligned */
    GRAPHKV_EWORKSPACE = -2,  /* ws is NULL, misaligned or smaller than graphkv_workspace_bytes() */
    GRAPHKV_EHIP = -3,        /* a kernel launch failed */
    GRAPHKV_ESCRATCH = -4     /* graphkv_compress_static: the params need more scratch than its built-in buffer holds */
};

enum { GRAPHKV_FP32 = 0, GRAPHKV_BF16 = 1 };
enum { GRAPHKV_POOL_AVG = 0, GRAPHKV_POOL_MAX = 1 };
/* Signal sent to the neighbours of a source (Discussion, "Diversity of Graph
 * Signal"): decay multiplies by (1 - alpha e), enhanced by (1 + alpha e),
 * evicted sets the score to -infinity. */
enum { GRAPHKV_SIGNAL_DECAY = 0, GRAPHKV_SIGNAL_ENHANCED = 1, GRAPHKV_SIGNAL_EVICTED = 2 };
/* Kernel family: AUTO picks the bf16 MFMA kernels when the shape allows them
 * (bf16 and d = 128; for scoring also G*w a multiple of 32 and at most 256, and
 * w a multiple of 32 with max pooling) and the scalar kernels otherwise; GENERIC
 * forces the scalar kernels (same results up to fp32 rounding order). */
enum { GRAPHKV_IMPL_AUTO = 0, GRAPHKV_IMPL_GENERIC = 1 };
/* Which tensors the edges of the whole-pass calls are cosines of (Discussion,
 * "Exploration of similarity for Graph Edge"): e_ij = cos(x_i, y_j) with x the
 * source's row and y the other node's row.  KK is Eq. 1 (keys, keys); KV takes the
 * source's key and the other node's value; VV values on both sides.  Pairings
 * with queries need the prefix tokens' queries, which these calls do not
 * receive: graphkv_propagate_edges takes any two tensors. */
enum { GRAPHKV_EDGES_KK = 0, GRAPHKV_EDGES_KV = 1, GRAPHKV_EDGES_VV = 2 };
/* Indicator that initialises the node scores in the whole-pass calls ("Sparse Graph
 * Building", first paragraph: attention-based scores or KNorm): ATTENTION is
 * graphkv_score, KNORM is graphkv_score_knorm (the queries are not read). */
enum { GRAPHKV_SCORER_ATTENTION = 0, GRAPHKV_SCORER_KNORM = 1 };

typedef struct graphkv_params {
    int32_t n_kv_heads;    /* H_kv >= 1                                              */
    int32_t n_q_heads;     /* H_q, a multiple of H_kv (ignored by propagate/select)  */
    int32_t head_dim;      /* d, a multiple of 8, <= 512                             */
    int32_t n_tokens;      /* N, rows of Kc/Vc per head, window included             */
    int32_t window;        /* w >= 1, P = N - w >= 1                                 */
    int32_t pool_kernel;   /* odd, >= 1 (1 = no pooling)                             */
    int32_t pool_mode;     /* GRAPHKV_POOL_*                                         */
    int32_t budget;        /* B, w < B <= N (select/compress only)                   */
    int32_t n_sources;     /* S, 1 <= S <= min(P, 65535) when rounds > 0             */
    int32_t n_neighbors;   /* m, 1 <= m <= P - 1 when rounds > 0                     */
    int32_t rounds;        /* T >= 0                                                 */
    float   decay;         /* alpha in [0, 1]                                        */
    int32_t reselect;      /* 0: sources and neighbourhoods fixed from round 1
                              (Eq. 2 / Eq. 5 as printed); 1: re-picked from the
                              refined scores every round (Fig. 1's caption lets the
                              pick-and-propagate step run more than once)            */
    int32_t dtype;         /* GRAPHKV_FP32 / GRAPHKV_BF16: type of Kc, Vc, Qw        */
    float   softmax_scale; /* 0 selects 1/sqrt(d)                                    */
    int32_t signal;        /* GRAPHKV_SIGNAL_*                                       */
    int32_t impl;          /* GRAPHKV_IMPL_*                                         */
    int32_t edges;         /* GRAPHKV_EDGES_* (compress calls only)                  */
    int32_t scorer;        /* GRAPHKV_SCORER_* (compress calls only)                 */
} graphkv_params;

/* Bytes of scratch any of the calls below needs for these params (0 if the
 * params are invalid). */
size_t graphkv_workspace_bytes(const graphkv_params *p);

/*
 * Stage I, the initial importance score s^(0) of every prefix token.  The
 * paper leaves the indicator to a host method ("Sparse Graph Building", first
 * paragraph); this is the observation-window attention score of SnapKV:
 * logits <q_r, k_j> * scale for the w window queries of each query head, row r
 * (token P + r) seeing columns 0..P+r, softmax over the visible columns, summed
 * over the window rows for j < P, 1-D pooled per query head (stride 1,
 * length-preserving; average pads with zeros and divides by pool_kernel), then
 * averaged over the G query heads of each KV head.
 *   Kc     [H_kv, N, d]  in   keys
 *   Qw     [H_q, w, d]   in   window queries
 *   scores [H_kv, P]     out  fp32
 * The `scorer` field is ignored here (this call is the attention scorer); the
 * workspace must have the size graphkv_workspace_bytes() returns for the params
 * with scorer = GRAPHKV_SCORER_ATTENTION, else GRAPHKV_EWORKSPACE.
 */
int32_t graphkv_score(const graphkv_params *p, const void *Kc, const void *Qw,
                      float *scores, void *ws, size_t ws_bytes, void *stream);

/*
 * KNorm-style initial score, another indicator the paper plugs GraphKV into
 * (Baseline Methods, the key-norm method): scores[h, j] = -||k_j||, so that the
 * low-norm keys that method keeps rank highest.  The scores are negative: see
 * graphkv_propagate for what the signal does to them.
 */
int32_t graphkv_score_knorm(const graphkv_params *p, const void *Kc, float *scores,
                            void *ws, size_t ws_bytes, void *stream);

/*
 * Stages II and III, T rounds on any score array (plug-and-play: Introduction,
 * last paragraph before the contributions).  Per round and head: source nodes =
 * the S largest scores (Eq. 2, Alg. 1); edges e_ij = cosine of keys i and j
 * for every source i and prefix node j != i (Eq. 1); neighbourhood of i = its
 * m largest edges (Eq. 3); every score s_j is multiplied by the product of
 * (1 - alpha e_ij) over the sources whose neighbourhood holds j, factors taken
 * in ascending source index (Eq. 4, Eq. 5, Alg. 2).  Ties in either top-k go
 * to the lowest index; a zero-norm key has e = 0.  rounds = 0, or decay = 0
 * with a multiplicative signal, leaves scores untouched.
 * Scores of either sign: Eq. 4 / Eq. 5 are written for a non-negative indicator.
 * The signal acts on the magnitude of the score a round starts with, s_j' = s_j -
 * alpha e_ij |s_j| (Eq. 4), so that the decay lowers a negative score too, as
 * "Decay Signal Propagation" says it should (it reduces the scores of redundant
 * tokens); the factor of Eq. 5 is then (1 + alpha e_ij) for s_j < 0.  The enhanced
 * signal mirrors this.
 *   Kc      [H_kv, N, d]       in
 *   scores  [H_kv, P]          in/out  fp32
 *   dbg_src [T, H_kv, S]       out, optional (NULL): sources, ascending
 *   dbg_nbr [T, H_kv, S, m]    out, optional: neighbours of each source, ascending
 *   dbg_e   [T, H_kv, S, m]    out, optional: their edge weights, fp32
 * With reselect = 0 the rows of rounds 2..T repeat round 1.
 */
int32_t graphkv_propagate(const graphkv_params *p, const void *Kc, float *scores,
                          int32_t *dbg_src, int32_t *dbg_nbr, float *dbg_e,
                          void *ws, size_t ws_bytes, void *stream);

/*
 * The same rounds with edges e_ij = cosine of row i of Ac and row j of Bc: the
 * source's feature comes from the first tensor, the other node's from the second
 * (Discussion, "Exploration of similarity for Graph Edge": query-to-key,
 * query-to-query, key-to-value, value-to-value similarities as decay signals; the
 * paper gives no formula, this is the reading taken).  Ac = Bc = keys is
 * graphkv_propagate.
 *   Ac, Bc  [H_kv, N, d]  in  of type p->dtype; everything else as above
 */
int32_t graphkv_propagate_edges(const graphkv_params *p, const void *Ac, const void *Bc,
                                float *scores, int32_t *dbg_src, int32_t *dbg_nbr, float *dbg_e,
                                void *ws, size_t ws_bytes, void *stream);

/*
 * Stage IV, selection ("Decay Signal Propagation", closing paragraph: the k_l
 * tokens with the highest refined score are kept).  idx[h, 0..B-w) = the B - w
 * best prefix tokens in ascending order (ties to the lowest index), followed by
 * the window tokens P..N-1.
 *   scores [H_kv, P]  in   fp32
 *   idx    [H_kv, B]  out  int32
 */
int32_t graphkv_select(const graphkv_params *p, const float *scores, int32_t *idx,
                       void *ws, size_t ws_bytes, void *stream);

/*
 * The whole pass for one layer: score -> propagate -> select -> gather of the
 * compressed sub-matrices K_s, V_s of k_l x d ("Problem Formulation").
 *   Kc, Vc     [H_kv, N, d]  in
 *   Qw         [H_q, w, d]   in
 *   Kout, Vout [H_kv, B, d]  out  rows idx[h, t] of Kc / Vc, byte copies
 *   idx        [H_kv, B]     out  int32
 *   scores_out [H_kv, P]     out, optional (NULL): refined scores s^(T), fp32
 * B = N gives the identity copy.  p->edges picks the tensors behind the edges,
 * p->scorer the indicator of stage I (with GRAPHKV_SCORER_KNORM Qw is not read and
 * may be NULL, and n_q_heads, pool_* and softmax_scale are ignored).
 */
int32_t graphkv_compress(const graphkv_params *p, const void *Kc, const void *Vc,
                         const void *Qw, void *Kout, void *Vout, int32_t *idx,
                         float *scores_out, void *ws, size_t ws_bytes, void *stream);

/*
 * The same pass for n_layers layers in one go.  The per-layer call keeps only H_kv
 * workgroups busy in its selection and update kernels and pays every launch per
 * layer; since all (layer, head) pairs are independent instances of the paper's
 * per-layer problem, a whole model can be pushed through each kernel at once
 * when its cache is one slab.
 *   Kc, Vc     [n_layers, H_kv, N, d]   in   contiguous
 *   Qw         [n_layers, H_q, w, d]    in
 *   budgets    HOST array [n_layers] of per-layer budgets B_l (w < B_l <= N), or
 *              NULL for p->budget everywhere (p->budget is ignored otherwise)
 *   Kout, Vout packed: layer l occupies rows [H_kv * sum_{l'<l} B_l', +H_kv * B_l),
 *              each layer laid out [H_kv, B_l, d]
 *   idx        packed the same way, [H_kv, B_l] per layer
 *   scores_out [n_layers, H_kv, P] or NULL
 *   ws         graphkv_workspace_bytes_batched(p, n_layers) bytes
 * Layers are processed in groups: at most 64 layers, fewer while the scratch
 * memory of a group would exceed 2000 MiB (long prompts).  Results are identical
 * to n_layers per-layer calls.
 */
size_t graphkv_workspace_bytes_batched(const graphkv_params *p, int32_t n_layers);
int32_t graphkv_compress_batched(const graphkv_params *p, int32_t n_layers, const int32_t *budgets,
                                 const void *Kc, const void *Vc, const void *Qw, void *Kout,
                                 void *Vout, int32_t *idx, float *scores_out, void *ws,
                                 size_t ws_bytes, void *stream);

/*
 * graphkv_compress for callers that cannot allocate device memory or size a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid allocation.  Same arguments and results as graphkv_compress, without
 * `ws`: the scratch memory is a buffer of GRAPHKV_STATIC_SCRATCH_BYTES that
 * belongs to the library's code object (every GPU the library runs on holds its
 * own copy until the process ends).  The call allocates and frees nothing.
 *   - params whose graphkv_workspace_bytes() exceeds GRAPHKV_STATIC_SCRATCH_BYTES
 *     are rejected with GRAPHKV_ESCRATCH before anything is enqueued;
 *   - every call on a GPU uses that GPU's one buffer: calls that overlap in time on
 *     one GPU (two streams, two host threads) race -- serialise them, or use
 *     graphkv_compress with a workspace each;
 *   - the first call on a device resolves the buffer's address and opts kernels in
 *     to large shared memory: make it outside a graph capture.
 */
#define GRAPHKV_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
int32_t graphkv_compress_static(const graphkv_params *p, const void *Kc, const void *Vc,
                                const void *Qw, void *Kout, void *Vout, int32_t *idx,
                                float *scores_out, void *stream);

/* Host string for a return code (static storage). */
const char *graphkv_strerror(int32_t code);

/*
 * Measurement aid (not part of the method): per-kernel timing with HIP events.
 * Between graphkv_profile_begin() and graphkv_profile_end() every kernel the
 * library launches is bracketed by two events on the caller's stream (the event
 * pool is created on first use and kept; process-wide: one recording at a time,
 * begin and end from one host thread).  graphkv_profile_end() waits for the
 * recorded events and adds up, per kernel id, the elapsed milliseconds into
 * ms[GRAPHKV_N_KERNELS] and the number of launches into launches[...] (HOST
 * arrays, either may be NULL).
 */
enum {
    GRAPHKV_K_SCORE_STATS = 0, GRAPHKV_K_SCORE_VOTES, GRAPHKV_K_POOL, GRAPHKV_K_TOPK_SOURCES,
    GRAPHKV_K_COSINE, GRAPHKV_K_TOPK_NEIGHBORS, GRAPHKV_K_DECAY, GRAPHKV_K_TOPK_FINAL,
    GRAPHKV_K_GATHER, GRAPHKV_K_GENERIC_LOGITS, GRAPHKV_K_GENERIC_VOTES, GRAPHKV_K_GENERIC_COSINE,
    GRAPHKV_K_KNORM, GRAPHKV_K_COPY, GRAPHKV_K_COSINE_BOUND,
    GRAPHKV_K_COSINE_FILTER, GRAPHKV_K_NBR_SELECT, GRAPHKV_K_REDO_ROWS,
    GRAPHKV_K_MATCH_SOURCES,
    /* later rounds when neighbour lists are kept: source selection, and the bound, filter and
     * select passes over the few sources that have no list yet */
    GRAPHKV_K_TOPK_SOURCES_LATER, GRAPHKV_K_COSINE_BOUND_NEW, GRAPHKV_K_COSINE_FILTER_NEW,
    GRAPHKV_K_NBR_SELECT_LATER, GRAPHKV_N_KERNELS
};
int32_t graphkv_profile_begin(void);
int32_t graphkv_profile_end(double *ms, int64_t *launches);
const char *graphkv_kernel_name(int32_t id);

/* 1 if AUTO would run the MFMA kernels for these params, 0 otherwise. */
int32_t graphkv_uses_mfma(const graphkv_params *p);

#ifdef __cplusplus
}
#endif
#endif /* GRAPHKV_H */
