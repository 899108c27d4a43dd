// Host-side launchers of the GraphKV kernels.  Every launcher only enqueues
// work on `st` and returns hipGetLastError() of its launches.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.hpp"

namespace gkv {

// Kernels that use more than 64 KiB of dynamic LDS need a one-time opt-in per kernel and
// device.  Which (device, kernel) pairs have it is the library's only state besides the
// measurement aid; it is process-wide and guarded by a mutex, so first calls may come from
// several host threads at once.  Returns false if the opt-in failed.
bool allow_big_lds(const void *kernel, int bytes = 160 * 1024 - 8192);

// ---- selection (select.hip) -------------------------------------------------
// For each of `rows` rows of x (row r starts at x + r*ld, n entries): the k
// entries that come first by (value descending, index ascending), written in
// ascending index order to idx_out + r*idx_ld (and their values to val_out +
// r*val_ld when val_out != nullptr).  After the k picks, `append_count`
// consecutive integers starting at `append_from` are appended to idx_out.
// tau_out (optional) receives the k-th largest value of each row; idx_out may
// then be nullptr.  gate (optional): row r is skipped when gate[r / rows_per_gate] == 0.
hipError_t launch_topk_rows(const float *x, long ld, int n, int rows, int k,
                            int32_t *idx_out, long idx_ld, float *val_out, long val_ld,
                            float *tau_out, int append_from, int append_count,
                            const int32_t *gate, int rows_per_gate, hipStream_t st);

// Neighbourhoods of the heads whose overflow flag is set (filter route, bf16, d = 128): a fixed
// number of workgroups walk the (head, source) rows of those heads, each computing one row of
// edges into its own scratch row (rows: redo_rows_scratch_bytes()) and taking the exact top-m.
size_t redo_rows_scratch_bytes(int heads, int S, int P);
hipError_t launch_redo_rows(const void *Ac, const void *Kc, int heads, int N, int P, int S, int m,
                            const int32_t *src, const int32_t *overflow, float *rows, int32_t *nbr,
                            float *nbr_e, hipStream_t st);

// ---- scalar kernels for any dtype / shape (generic.hip) ----------------------
// logits [Hq*w, N] (fp32, scaled), then per-row max and sum of exp.
hipError_t launch_generic_logits(const void *Kc, const void *Qw, int dtype, int Hkv, int Hq, int d,
                                 int N, int w, float scale, float *logits, float *row_max,
                                 float *row_sum, hipStream_t st);
// votes [Hq, P]: softmax weights summed over the window rows.
hipError_t launch_generic_votes(const float *logits, const float *row_max, const float *row_sum,
                                int Hq, int N, int w, float *votes, hipStream_t st);
// E [Hkv, S, P] cosine of row src[h,a] of Ac against every prefix row of Kc; self = -inf.
// (Eq. 1: Ac = Kc = keys; other pairings of tensors give the Discussion's other edges.)
hipError_t launch_generic_cosine(const void *Ac, const void *Kc, int dtype, int Hkv, int d, int N, int P, int S,
                                 const int32_t *src, float *E, hipStream_t st);
// scores[h,j] = -||k_j||
hipError_t launch_knorm(const void *Kc, int dtype, int Hkv, int d, int N, int P, float *scores,
                        hipStream_t st);

// ---- pooling, signal propagation, gather (stages.hip) -----------------------
// votes [Hkv*Gv, P] -> scores [Hkv, P]: pool each of the Gv rows of a head, sum, divide by div.
hipError_t launch_pool_group(const float *votes, int Hkv, int Gv, int P, int pool_kernel,
                             int pool_mode, float div, float *scores, hipStream_t st);
// Eq. 5 for one round: scores[h, nbr] *= prod (1 -/+ alpha e), ascending source order.
hipError_t launch_decay(float *scores, int Hkv, int P, int S, int m, const int32_t *nbr,
                        const float *nbr_e, float alpha, int signal, hipStream_t st);
// Kout[q,t,:] = Kc[q, idx[q,t], :] for the heads q of a batch, same for V; packed
// outputs, per-layer budgets from the plan; row_bytes multiple of 16.
hipError_t launch_gather(const void *Kc, const void *Vc, const int32_t *idx, int heads, int N,
                         const LayerPlan &plan, int max_budget, int row_bytes, void *Kout, void *Vout,
                         hipStream_t st);
// Final selection of a batch: row q keeps budget[l] - w entries and writes them,
// followed by the window tokens P .. P + w - 1, to its packed idx row.
hipError_t launch_topk_final(const float *scores, int P, int rows, const LayerPlan &plan, int w,
                             int32_t *idx, hipStream_t st);
hipError_t launch_copy_i32(const int32_t *src, int32_t *dst, long n, hipStream_t st);
hipError_t launch_copy_f32(const float *src, float *dst, long n, hipStream_t st);

// ---- bf16 MFMA kernels, d = 128 (mfma_score.hip, mfma_cosine.hip) ----------
struct MfmaScorePlan {
    int chunks;        // key chunks per head in the streaming passes
    size_t part_bytes; // bytes of per-chunk row statistics
};
MfmaScorePlan mfma_score_plan(int Hkv, int rows, int N);
// Pass A: per (head, chunk, row) partial max and sum of exp2 over the chunk's visible keys.
// Pass B: votes [Hkv * rows, P] with rows = mfma_score_vote_rows(): partial sums over
// groups of query rows (to be added up), or one row per query head.
int mfma_score_vote_rows(int G, int w, int per_qhead_votes);
hipError_t launch_mfma_score_stats(const void *Kc, const void *Qw, int Hkv, int Hq, int N, int w,
                                  float scale, float *part, hipStream_t st);
// fused_pool_kernel > 0 (only if mfma_score_fuses_pool()): average pooling with that kernel
// size and the mean over the query heads are done in the same kernel; `votes` is then the
// score array [Hkv, P] and no pooling kernel follows.
bool mfma_score_fuses_pool(int G, int w, int per_qhead_votes, int pool_kernel);
hipError_t launch_mfma_score_votes(const void *Kc, const void *Qw, int Hkv, int Hq, int N, int w,
                                  float scale, int per_qhead_votes, int fused_pool_kernel,
                                  const float *part, float *votes, hipStream_t st);
// E [Hkv, S, P] from bf16 keys (same contract as launch_generic_cosine); heads with
// gate[h] == 0 are skipped when gate != nullptr.
hipError_t launch_mfma_cosine(const void *Ac, const void *Kc, int Hkv, int N, int P, int S, const int32_t *src,
                              float *E, const int32_t *gate, hipStream_t st);
// Neighbourhoods without the dense block (see mfma_cosine.hip):
bool mfma_filter_applies(int P, int m);
int mfma_sample_cols(int P);          // keys in the strided sample
int mfma_cand_cap(int P, int m);      // candidates per source the exact select can take
struct MfmaFilterGeom {
    int chunk_cols;   // keys per workgroup of the filter pass
    int chunks;       // workgroups (= candidate slices) per head
    int slice_cap;    // entries per (source, chunk) slice
};
MfmaFilterGeom mfma_filter_geom(int Hkv, int P, int S, int m);
// tau [Hkv, S]: a lower bound of each source's m-th largest edge, from the edges to every
// (P / sample_cols)-th key (within 1/256 of the m-th largest sampled edge); clears overflow [Hkv].
size_t mfma_bound_scratch_bytes(int Hkv, int P, int S);   // per-chunk histograms (0 if one chunk)
// n_src (bound and filter pass): null, or [Hkv] rows of each head's source list in use; the
// arrays keep their pitch of S rows.
hipError_t launch_mfma_cosine_bound(const void *Ac, const void *Kc, int Hkv, int N, int P, int S, int m,
                                    const int32_t *src, const int32_t *n_src, void *hist_part, float *tau,
                                    int32_t *overflow, hipStream_t st);
// Streams all keys; edges that reach tau[h, a] go to cand [Hkv, S, chunks, slice_cap] x 8
// bytes, their number per slice to cand_cnt [Hkv, S, chunks].
hipError_t launch_mfma_cosine_filter(const void *Ac, const void *Kc, int Hkv, int N, int P, int S, int m,
                                     const int32_t *src, const int32_t *n_src, const float *tau, void *cand,
                                     int32_t *cand_cnt, int32_t *overflow, hipStream_t st);
// Exact top-m over each source's slices -> nbr / nbr_e [Hkv, S, m]; skips heads with
// overflow[h], and raises overflow[h] itself if a source has more candidates than it can take.
// Neighbour lists kept from the previous round: Eq. 1 and Eq. 3 depend on the keys alone, so
// a source that was one in the previous round has the same neighbourhood.
struct SourceReuse {
    const int32_t *n_new;      // [Hkv] sources that were none in the previous round
    const int32_t *code;       // [Hkv, S] per source: its slot in the previous round, or -1 - r (r-th new one)
    const int32_t *new_pos;    // [Hkv, S] slot of the r-th new source in this round's list
};
bool source_reuse_applies(int S);
// prev, cur [Hkv, S] ascending -> code, new_pos as above, new_src [Hkv, S] (the new sources in
// order, n_new[h] of them); copies the lists of the sources that stay from prev_nbr / prev_e
// [Hkv, S, m] to their slots in nbr / nbr_e.
hipError_t launch_match_sources(const int32_t *prev, const int32_t *cur, int Hkv, int S, int m,
                                const int32_t *prev_nbr, const float *prev_e, int32_t *code, int32_t *new_src,
                                int32_t *new_pos, int32_t *n_new, int32_t *nbr, float *nbr_e, hipStream_t st);
// reuse: null, or the candidate rows are those of the new sources (src = new_src).
hipError_t launch_nbr_select(const void *cand, const int32_t *cand_cnt, int32_t *overflow,
                             const int32_t *src, int Hkv, int P, int S, int m, const SourceReuse *reuse,
                             int32_t *nbr, float *nbr_e, hipStream_t st);

}  // namespace gkv
