/*
 * CPU oracle for the GraphKV eviction pass.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, double-precision restatement of what the pass computes, used
 * by the test-suite, the smoke check and the benchmark's CPU-baseline leg to
 * judge the GPU library.  It shares no code, header, table or helper with the
 * GPU library and must never be called from a product path.
 *
 * What is computed, per KV head independently (the paper states the problem
 * for one n x d key/value matrix per layer -- Methodology, "Problem
 * Formulation"; heads are treated as independent instances of it):
 *
 *   stage I   initial importance score s_j of every prefix token (the paper
 *             leaves this to a host method -- "Sparse Graph Building", first
 *             paragraph; here the observation-window attention score that
 *             SnapKV uses, named in Related Works / Baseline Methods);
 *   stage II  source nodes = the S highest-scoring tokens (Eq. 2, Alg. 1) and
 *             cosine edges from every source to every other node (Eq. 1);
 *   stage III neighbourhood of a source = its m largest edges (Eq. 3); scores
 *             of neighbours are multiplied by (1 - alpha*e_ij) for every
 *             source that reaches them (Eq. 4, Eq. 5, Alg. 2), T rounds;
 *   stage IV  the budget's worth of highest refined scores is kept and the
 *             K/V rows are gathered ("Decay Signal Propagation", last
 *             paragraph before the closing remark).
 *
 * Readings taken where the paper is silent, garbled or ambiguous:
 *   R1  Eq. 4 and Alg. 2 are printed with a blank where a coefficient of
 *       e_ij s_j would stand; the Limitation section speaks of a decay-strength
 *       hyper-parameter.  Factor = (1 - alpha*e_ij); alpha = 1 gives Eq. 5 as
 *       printed.
 *   R2  Graph fixed across rounds (Eq. 2/5, Alg. 2 take a finished graph) or
 *       re-picked from the refined scores each round (Fig. 1's caption allows
 *       the pick-and-propagate step to run once or several times)?
 *       Both: reselect = 0 / 1.  Identical at T = 1.
 *   R3  Inside a round all sources act at once (Eq. 5's product).  Alg. 2's
 *       nested loops give the same real number because neighbourhoods depend
 *       on e only; the floating-point order is fixed to ascending source index.
 *   R4  A source may be decayed by another source (only j = i is excluded,
 *       Eq. 3 and Alg. 1's O \ {o_i}).
 *   R5  Eq. 3's ">=" would admit more than m neighbours on ties; here every
 *       top-k returns exactly k entries and ties go to the lowest index.
 *   R6  A negative cosine gives a factor above 1: literal, no clamp.
 *   R7  m and S are explicit arguments.
 *   R8  Stage I: logits q.k * scale (default 1/sqrt(d)); row r of the window
 *       sits at position P + r and sees columns 0 .. P + r (causal); softmax
 *       over all visible columns; only columns j < P collect votes; votes are
 *       summed over the window rows, pooled per query head (length-preserving,
 *       stride 1; average with zero padding and division by the kernel size,
 *       or max), then averaged over the G query heads of the KV head.
 *   R9  Graph nodes are the P = N - w prefix tokens; window tokens are always
 *       kept, are never sources and never neighbours.  The budget B counts
 *       them, so B - w tokens come from the prefix.
 *   R10 Retained rows are emitted in ascending token order, window last.
 *   R11 A zero-norm key has e = 0 with every node.
 *   R12 Besides the decay signal, the Discussion ("Diversity of Graph Signal")
 *       names an enhanced signal (+) and an evicted signal (-inf):
 *       signal 1 multiplies by (1 + alpha*e), signal 2 sets neighbours to -inf.
 *   R13 Source lists and neighbour lists are reported in ascending index order
 *       (their order carries no meaning in the paper).
 *   R14 The Discussion ("Exploration of similarity for Graph Edge") also tries
 *       query-to-key, query-to-query, key-to-value and value-to-value
 *       similarities as edges, without formulas.  Reading: e_ij = cosine of
 *       (row i of a first tensor, row j of a second tensor), the first tensor
 *       giving the source's feature and the second the other node's; key-to-key
 *       is first = second = keys.  edge_mode of the whole-pass function:
 *       0 key-key, 1 key-value, 2 value-value (pairings with queries need the
 *       prefix tokens' queries, which the pass does not receive; the two-tensor
 *       propagate takes any pair).
 *   R15 KNorm as the indicator that initialises the nodes (Sparse Graph Building,
 *       first paragraph; Baseline Methods describes it as the keys' L2 norm): that method keeps
 *       the keys of small norm, so s_j = -||k_j|| (scorer 1 of the whole-pass
 *       function; no queries are needed).
 *   R16 Scores of either sign.  Eq. 4 / Eq. 5 are written for a non-negative
 *       indicator; multiplied into a negative score, (1 - alpha e) would RAISE
 *       it, against what "Decay Signal Propagation" says the signal does
 *       (it lowers the score of a token that resembles a source, the more so
 *       the closer the two are).  Reading: the change of Eq. 4 is taken on the
 *       magnitude, s_j' = s_j - alpha e_ij |s_j|, i.e. the factor of Eq. 5 is
 *       (1 - alpha e) for s_j >= 0 and (1 + alpha e) for s_j < 0, the sign being
 *       that of the score at the start of the round; the enhanced signal mirrors
 *       it.  For s_j >= 0 this is Eq. 4 / Eq. 5 as printed.
 *
 * Arithmetic: every product, sum, exp, sqrt and division is done in double on
 * the exact values of the stored fp32/bf16 inputs.  No blocking, no fusion.
 *
 * Pins (tests, CPU only): brute force on a dense P x P cosine matrix for tiny
 * P; T = 0 / alpha = 0 reducing to plain top-(B-w); closed forms for zero
 * queries; softmax re-derived with a library routine; orthogonal keys; exact
 * duplicates; scale invariance; a hand-worked 6-node example (also with negative
 * scores); Eq. 4 iterated source by source on negative scores; the decay of -s
 * mirroring the enhanced signal on s; the value of the reported cut gaps.  The
 * choice among the readings R2, R6, R7, R8, R15, R16 cannot be pinned by the paper:
 * "parity unpinned" for those beyond agreement under the stated reading.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { GKV_FP32 = 0, GKV_BF16 = 1 };

static double load_elem(const void *base, int dtype, size_t i)
{
    if (dtype == GKV_FP32)
        return (double)((const float *)base)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)base)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static size_t elem_size(int dtype) { return dtype == GKV_FP32 ? 4 : 2; }

/* ---------------------------------------------------------------- top-k --- */

typedef struct { double v; int32_t i; } gkv_pair;

static int cmp_value_desc_index_asc(const void *a, const void *b)
{
    const gkv_pair *x = (const gkv_pair *)a, *y = (const gkv_pair *)b;
    if (x->v > y->v) return -1;
    if (x->v < y->v) return 1;
    return (x->i > y->i) - (x->i < y->i);
}

static int cmp_int32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * The k entries that come first when x[0..n) is sorted by value descending,
 * index ascending (reading R5).  idx_out receives them in ascending index
 * order (R13).  skip >= 0 removes that index from the candidates (Eq. 3's
 * j != i).  gap_out (optional) receives the relative gap at the cut:
 * (last kept - first dropped) / max(|last kept|, tiny); +inf when nothing is
 * dropped.
 */
void gkv_oracle_topk(const double *x, int32_t n, int32_t k, int32_t skip,
                     int32_t *idx_out, double *gap_out)
{
    gkv_pair *p = (gkv_pair *)malloc((size_t)(n > 0 ? n : 1) * sizeof *p);
    int32_t cnt = 0;
    for (int32_t j = 0; j < n; ++j) {
        if (j == skip) continue;
        p[cnt].v = x[j];
        p[cnt].i = j;
        ++cnt;
    }
    qsort(p, (size_t)cnt, sizeof *p, cmp_value_desc_index_asc);
    if (k > cnt) k = cnt;
    for (int32_t t = 0; t < k; ++t) idx_out[t] = p[t].i;
    qsort(idx_out, (size_t)k, sizeof *idx_out, cmp_int32);
    if (gap_out) {
        if (k == 0 || k == cnt) {
            *gap_out = INFINITY;
        } else {
            double in = p[k - 1].v, out = p[k].v;
            double den = fabs(in) > 1e-300 ? fabs(in) : 1e-300;
            *gap_out = (in - out) / den;
        }
    }
    free(p);
}

/* -------------------------------------------------------------- stage I --- */

/*
 * Initial importance score (reading R8).  Kc [Hkv,N,d], Qw [Hq,w,d] in the
 * storage type; s_out [Hkv,P] double.  votes_out (optional) [Hq,P] receives the
 * un-pooled per-query-head votes.
 */
int gkv_oracle_score(const void *Kc, const void *Qw, int dtype,
                     int32_t Hkv, int32_t Hq, int32_t d, int32_t N, int32_t w,
                     int32_t pool_kernel, int32_t pool_mode, double scale,
                     double *s_out, double *votes_out)
{
    if (Hkv < 1 || Hq < Hkv || Hq % Hkv || d < 1 || w < 1 || N <= w) return -1;
    if (pool_kernel < 1 || pool_kernel % 2 == 0) return -1;
    const int32_t P = N - w, G = Hq / Hkv, half = (pool_kernel - 1) / 2;
    if (scale == 0.0) scale = 1.0 / sqrt((double)d);

#pragma omp parallel for schedule(dynamic)
    for (int32_t h = 0; h < Hkv; ++h) {
        double *logit = (double *)malloc((size_t)N * sizeof(double));
        double *vote = (double *)malloc((size_t)P * sizeof(double));
        double *pooled = (double *)malloc((size_t)P * sizeof(double));
        double *s = s_out + (size_t)h * P;
        for (int32_t j = 0; j < P; ++j) s[j] = 0.0;

        for (int32_t g = 0; g < G; ++g) {
            const int32_t q = h * G + g;
            for (int32_t j = 0; j < P; ++j) vote[j] = 0.0;
            for (int32_t r = 0; r < w; ++r) {
                const int32_t last = P + r;            /* causal: columns 0..P+r */
                double mx = -INFINITY;
                for (int32_t j = 0; j <= last; ++j) {
                    double acc = 0.0;
                    for (int32_t c = 0; c < d; ++c)
                        acc += load_elem(Qw, dtype, ((size_t)q * w + r) * d + c) *
                               load_elem(Kc, dtype, ((size_t)h * N + j) * d + c);
                    logit[j] = acc * scale;
                    if (logit[j] > mx) mx = logit[j];
                }
                double z = 0.0;
                for (int32_t j = 0; j <= last; ++j) z += exp(logit[j] - mx);
                for (int32_t j = 0; j < P; ++j) vote[j] += exp(logit[j] - mx) / z;
            }
            if (votes_out)
                memcpy(votes_out + (size_t)q * P, vote, (size_t)P * sizeof(double));
            for (int32_t j = 0; j < P; ++j) {
                if (pool_mode == 0) {                  /* average, zero padding */
                    double acc = 0.0;
                    for (int32_t t = j - half; t <= j + half; ++t)
                        if (t >= 0 && t < P) acc += vote[t];
                    pooled[j] = acc / (double)pool_kernel;
                } else {                               /* max, -inf padding */
                    double mxp = -INFINITY;
                    for (int32_t t = j - half; t <= j + half; ++t)
                        if (t >= 0 && t < P && vote[t] > mxp) mxp = vote[t];
                    pooled[j] = mxp;
                }
            }
            for (int32_t j = 0; j < P; ++j) s[j] += pooled[j];
        }
        for (int32_t j = 0; j < P; ++j) s[j] /= (double)G;
        free(logit); free(vote); free(pooled);
    }
    return 0;
}

/*
 * KNorm-style initial score: the paper lists the L2 norm of keys as another
 * indicator that can initialise the nodes (Baseline Methods).  Tokens with a
 * small key norm are the ones that method keeps, so s_j = -||k_j||.
 */
int gkv_oracle_score_knorm(const void *Kc, int dtype, int32_t Hkv, int32_t d,
                           int32_t N, int32_t w, double *s_out)
{
    if (Hkv < 1 || d < 1 || w < 0 || N <= w) return -1;
    const int32_t P = N - w;
    for (int32_t h = 0; h < Hkv; ++h)
        for (int32_t j = 0; j < P; ++j) {
            double acc = 0.0;
            for (int32_t c = 0; c < d; ++c) {
                double v = load_elem(Kc, dtype, ((size_t)h * N + j) * d + c);
                acc += v * v;
            }
            s_out[(size_t)h * P + j] = -sqrt(acc);
        }
    return 0;
}

/* ------------------------------------------------------- stages II, III --- */

/* Eq. 1 for one source i of head h against every prefix node, with the feature of
 * the source taken from A and the feature of the other node from Bm (both
 * [Hkv,N,d]; reading R14: A = Bm = keys is the paper's main definition, the
 * Discussion's other pairings pass other tensors).  e[i] itself is left at 0 and
 * must be skipped by the caller.  Reading R11 for zero norms. */
void gkv_oracle_cosine_row2(const void *A, const void *Bm, int dtype, int32_t d, int32_t N,
                            int32_t P, int32_t h, int32_t i, double *e_out)
{
    double ni = 0.0;
    for (int32_t c = 0; c < d; ++c) {
        double v = load_elem(A, dtype, ((size_t)h * N + i) * d + c);
        ni += v * v;
    }
    ni = sqrt(ni);
    for (int32_t j = 0; j < P; ++j) {
        double dot = 0.0, nj = 0.0;
        for (int32_t c = 0; c < d; ++c) {
            double a = load_elem(A, dtype, ((size_t)h * N + i) * d + c);
            double b = load_elem(Bm, dtype, ((size_t)h * N + j) * d + c);
            dot += a * b;
            nj += b * b;
        }
        nj = sqrt(nj);
        e_out[j] = (ni == 0.0 || nj == 0.0) ? 0.0 : dot / (ni * nj);
    }
    e_out[i] = 0.0;
}

void gkv_oracle_cosine_row(const void *Kc, int dtype, int32_t d, int32_t N,
                           int32_t P, int32_t h, int32_t i, double *e_out)
{
    gkv_oracle_cosine_row2(Kc, Kc, dtype, d, N, P, h, i, e_out);
}

/*
 * T rounds of signal propagation on scores s [Hkv,P] (in place).
 *   forced_src (optional) [T,Hkv,S]: use these sources instead of Eq. 2's pick
 *     (ascending per list) -- lets a test hold the upstream selection fixed.
 *   dbg_src [T,Hkv,S], dbg_nbr [T,Hkv,S,m], dbg_e [T,Hkv,S,m] (optional):
 *     what was picked, ascending index order (R13), and the edge weights.
 *   gap_src [T,Hkv], gap_nbr [T,Hkv,S] (optional): relative gaps at the cuts.
 * signal: 0 decay (Eq. 5), 1 enhanced, 2 evicted (R12); negative scores: R16.
 * A, Bm: the tensors whose rows enter Eq. 1 for the source and for the other
 *   node (R14).
 */
int gkv_oracle_propagate_edges(const void *A, const void *Bm, int dtype, int32_t Hkv, int32_t d,
                               int32_t N, int32_t w, int32_t S, int32_t m, int32_t T,
                               double alpha, int32_t reselect, int32_t signal,
                               double *s, const int32_t *forced_src,
                               int32_t *dbg_src, int32_t *dbg_nbr, double *dbg_e,
                               double *gap_src, double *gap_nbr)
{
    const int32_t P = N - w;
    if (Hkv < 1 || d < 1 || P < 1 || T < 0) return -1;
    if (T > 0 && (S < 1 || S > P || m < 0 || m > P - 1)) return -1;

#pragma omp parallel for schedule(dynamic)
    for (int32_t h = 0; h < Hkv; ++h) {
        double *sh = s + (size_t)h * P;
        int32_t *src = (int32_t *)malloc((size_t)(S > 0 ? S : 1) * sizeof(int32_t));
        int32_t *nbr = (int32_t *)malloc((size_t)(S * m > 0 ? S * m : 1) * sizeof(int32_t));
        double *ev = (double *)malloc((size_t)(S * m > 0 ? S * m : 1) * sizeof(double));
        double *erow = (double *)malloc((size_t)P * sizeof(double));
        double *f = (double *)malloc((size_t)P * sizeof(double));
        char *hit = (char *)malloc((size_t)P);

        for (int32_t t = 0; t < T; ++t) {
            const size_t ts = ((size_t)t * Hkv + h) * S;
            if (t == 0 || reselect) {
                /* Eq. 2 / Alg. 1: source nodes */
                double g = INFINITY;
                if (forced_src) {
                    memcpy(src, forced_src + ts, (size_t)S * sizeof(int32_t));
                } else {
                    gkv_oracle_topk(sh, P, S, -1, src, &g);
                }
                if (gap_src) gap_src[(size_t)t * Hkv + h] = g;
                /* Eq. 1 + Eq. 3: edges of each source and its m nearest nodes */
                for (int32_t a = 0; a < S; ++a) {
                    double gn = INFINITY;
                    gkv_oracle_cosine_row2(A, Bm, dtype, d, N, P, h, src[a], erow);
                    gkv_oracle_topk(erow, P, m, src[a], nbr + (size_t)a * m, &gn);
                    for (int32_t u = 0; u < m; ++u)
                        ev[(size_t)a * m + u] = erow[nbr[(size_t)a * m + u]];
                    if (gap_nbr) gap_nbr[ts + a] = gn;
                }
            } else {
                if (gap_src) gap_src[(size_t)t * Hkv + h] = gap_src[h];
                if (gap_nbr)
                    for (int32_t a = 0; a < S; ++a) gap_nbr[ts + a] = gap_nbr[(size_t)h * S + a];
            }
            if (dbg_src) memcpy(dbg_src + ts, src, (size_t)S * sizeof(int32_t));
            if (dbg_nbr) memcpy(dbg_nbr + ts * m, nbr, (size_t)S * m * sizeof(int32_t));
            if (dbg_e) memcpy(dbg_e + ts * m, ev, (size_t)S * m * sizeof(double));

            /* Eq. 5: product over the sources that reach node j, ascending source index */
            for (int32_t j = 0; j < P; ++j) { f[j] = 1.0; hit[j] = 0; }
            for (int32_t a = 0; a < S; ++a)
                for (int32_t u = 0; u < m; ++u) {
                    const int32_t j = nbr[(size_t)a * m + u];
                    const double e = ev[(size_t)a * m + u];
                    hit[j] = 1;
                    /* R16: the signal acts on the magnitude of the score the round
                     * started with: decay lowers it, the enhanced signal raises it */
                    const double dir = ((signal == 1) != (sh[j] < 0.0)) ? 1.0 : -1.0;
                    f[j] *= (1.0 + dir * alpha * e);
                }
            for (int32_t j = 0; j < P; ++j) {
                if (!hit[j]) continue;
                if (signal == 2) sh[j] = -INFINITY;
                else             sh[j] *= f[j];
            }
        }
        free(src); free(nbr); free(ev); free(erow); free(f); free(hit);
    }
    return 0;
}

/* Key-to-key edges: the paper's main definition (Eq. 1). */
int gkv_oracle_propagate(const void *Kc, int dtype, int32_t Hkv, int32_t d,
                         int32_t N, int32_t w, int32_t S, int32_t m, int32_t T,
                         double alpha, int32_t reselect, int32_t signal,
                         double *s, const int32_t *forced_src,
                         int32_t *dbg_src, int32_t *dbg_nbr, double *dbg_e,
                         double *gap_src, double *gap_nbr)
{
    return gkv_oracle_propagate_edges(Kc, Kc, dtype, Hkv, d, N, w, S, m, T, alpha, reselect, signal,
                                      s, forced_src, dbg_src, dbg_nbr, dbg_e, gap_src, gap_nbr);
}

/* ------------------------------------------------------------ stage IV --- */

/* Final budgeted selection (R9, R10): idx [Hkv,B] = the B-w best prefix tokens
 * in ascending order followed by P .. N-1.  gap (optional) [Hkv]. */
int gkv_oracle_select(const double *s, int32_t Hkv, int32_t N, int32_t w,
                      int32_t B, int32_t *idx, double *gap)
{
    const int32_t P = N - w;
    if (B < w || B > N || P < 1) return -1;
    for (int32_t h = 0; h < Hkv; ++h) {
        double g = INFINITY;
        gkv_oracle_topk(s + (size_t)h * P, P, B - w, -1, idx + (size_t)h * B, &g);
        for (int32_t r = 0; r < w; ++r) idx[(size_t)h * B + (B - w) + r] = P + r;
        if (gap) gap[h] = g;
    }
    return 0;
}

/* Compacted cache: Kout[h,t,:] = Kc[h,idx[h,t],:], same for V (byte copies). */
int gkv_oracle_gather(const void *Kc, const void *Vc, int dtype, int32_t Hkv,
                      int32_t d, int32_t N, int32_t B, const int32_t *idx,
                      void *Kout, void *Vout)
{
    const size_t row = (size_t)d * elem_size(dtype);
    for (int32_t h = 0; h < Hkv; ++h)
        for (int32_t t = 0; t < B; ++t) {
            const int32_t j = idx[(size_t)h * B + t];
            if (j < 0 || j >= N) return -1;
            memcpy((char *)Kout + ((size_t)h * B + t) * row,
                   (const char *)Kc + ((size_t)h * N + j) * row, row);
            memcpy((char *)Vout + ((size_t)h * B + t) * row,
                   (const char *)Vc + ((size_t)h * N + j) * row, row);
        }
    return 0;
}

/*
 * The whole pass for one layer: stage I -> T rounds of II+III -> IV.
 * scorer: 0 the observation-window attention score (R8), 1 KNorm (R15; Qw unused).
 * scores_out (optional) [Hkv,P] double: the refined scores s^(T).
 * s0_out (optional) [Hkv,P] double: the initial scores.
 * What was picked and how close every cut was (all optional):
 *   src_out [T,Hkv,S], nbr_out [T,Hkv,S,m]: sources and neighbour lists per round;
 *   gap_src [T,Hkv], gap_nbr [T,Hkv,S], gap_final [Hkv]: the relative gap between
 *   the last entry kept and the first one dropped at the source cut, at each
 *   source's neighbour cut and at the final cut (see gkv_oracle_topk).
 */
int gkv_oracle_compress(const void *Kc, const void *Vc, const void *Qw, int dtype,
                        int32_t Hkv, int32_t Hq, int32_t d, int32_t N, int32_t w,
                        int32_t pool_kernel, int32_t pool_mode, double scale,
                        int32_t B, int32_t S, int32_t m, int32_t T, double alpha,
                        int32_t reselect, int32_t signal, int32_t edge_mode, int32_t scorer,
                        void *Kout, void *Vout, int32_t *idx,
                        double *scores_out, double *s0_out,
                        int32_t *src_out, int32_t *nbr_out,
                        double *gap_src, double *gap_nbr, double *gap_final)
{
    const int32_t P = N - w;
    if (P < 1 || B <= w || B > N) return -1;
    if (scorer != 0 && scorer != 1) return -1;
    double *s = (double *)malloc((size_t)Hkv * P * sizeof(double));
    int rc = scorer == 1
        ? gkv_oracle_score_knorm(Kc, dtype, Hkv, d, N, w, s)
        : gkv_oracle_score(Kc, Qw, dtype, Hkv, Hq, d, N, w, pool_kernel, pool_mode, scale, s, NULL);
    if (rc == 0 && s0_out) memcpy(s0_out, s, (size_t)Hkv * P * sizeof(double));
    if (rc == 0 && T > 0)
        rc = gkv_oracle_propagate_edges(edge_mode == 2 ? Vc : Kc, edge_mode == 0 ? Kc : Vc, dtype,
                                        Hkv, d, N, w, S, m, T, alpha, reselect, signal,
                                        s, NULL, src_out, nbr_out, NULL, gap_src, gap_nbr);
    if (rc == 0) rc = gkv_oracle_select(s, Hkv, N, w, B, idx, gap_final);
    if (rc == 0) rc = gkv_oracle_gather(Kc, Vc, dtype, Hkv, d, N, B, idx, Kout, Vout);
    if (rc == 0 && scores_out) memcpy(scores_out, s, (size_t)Hkv * P * sizeof(double));
    free(s);
    return rc;
}
