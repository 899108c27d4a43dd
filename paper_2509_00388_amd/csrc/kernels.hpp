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

// Source nodes (Eq. 2) plus the X nodes ranked right behind them: src [rows, S] gets the S
// best entries of each row (ascending index), ext [rows, S + X] the same S followed by the next
// X (ascending index), by (value descending, index ascending).  4096 < n, S + X <= kMaxExtSources.
hipError_t launch_pick_sources(const float *x, long ld, int n, int rows, int S, int X, int32_t *src,
                               int32_t *ext, hipStream_t st);

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
int mfma_bound_rank(int m, int stride);   // rank in the sample at which a row's bound is taken (<= m)
int mfma_cand_cap(int P, int m);      // candidates per source the exact select can take
bool source_reuse_applies(int S);     // lists can be kept from round to round
constexpr int kSpecRows = 32;         // speculative rows per head: one or two MFMA row blocks of 32
constexpr int kMaxExtSources = 256;   // largest S + kSpecRows the source selection splits
// Geometry of the filter route for one call.  The per-row buffers (tau [Hkv, pitch], cand
// [Hkv, pitch, chunks, slice_cap] x 8 bytes, cand_cnt [Hkv, pitch, chunks]) hold, per head,
// the S sources of the first round, then X speculative rows (the nodes ranked right behind the
// sources: the likeliest new sources of later rounds, whose candidate lists the first round's
// pass builds on the side), then fb_rows rows for new sources of later rounds that have no kept
// list.  Without speculation (X = 0) nothing outlives a round and later rounds reuse rows 0 .. S.
struct MfmaFilterPlan {
    int S, X;
    int sb;           // 32-row groups per workgroup in the passes over the full source list
    int pitch;        // S + X
    int chunk_cols;   // keys per workgroup of the filter pass
    int chunks;       // workgroups (= candidate slices) per head and source group
    int slice_cap;    // entries per (row, chunk) slice
    int cand_cap;     // entries the exact select can take per row
};
MfmaFilterPlan mfma_filter_plan(int Hkv, int P, int S, int m, bool keep_lists, bool speculate);
size_t mfma_bound_scratch_bytes(int Hkv, int P, const MfmaFilterPlan &g);   // per-chunk histograms (0 if one chunk)
// Bound pass: tau = a value that at least m of the row's edges reach (but for about one row in
// 10^7, which the select notices), from the edges to every (P / sample_cols)-th key; clears
// overflow [Hkv].  first_round: src is the extended list
// [Hkv, S + X] (all rows in use, rows 0 .. of the buffers); otherwise src is the list of new
// sources [Hkv, S], n_src [Hkv] of them in use, rows 0 .. of the buffers.
hipError_t launch_mfma_cosine_bound(const void *Ac, const void *Kc, int Hkv, int N, int P, int m,
                                    const MfmaFilterPlan &g, bool first_round, const int32_t *src,
                                    const int32_t *n_src, void *hist_part, float *tau, int32_t *overflow,
                                    hipStream_t st);
// Filter pass: streams all keys; edges that reach a row's tau go to its slices, their number
// per slice to cand_cnt.  Same source lists and rows as the bound pass.
hipError_t launch_mfma_cosine_filter(const void *Ac, const void *Kc, int Hkv, int N, int P, int m,
                                     const MfmaFilterPlan &g, bool first_round, const int32_t *src,
                                     const int32_t *n_src, const float *tau, void *cand, int32_t *cand_cnt,
                                     int32_t *overflow, hipStream_t st);
// From the second round on: which sources keep their list from the round before (copied from
// prev_nbr / prev_e to nbr / nbr_e), which are speculative rows of the first round (the last X
// entries of ext [Hkv, S + X]; not used for heads that overflowed then: spec_bad [Hkv], set by the first match of
// a call from the first round's overflow flags), and which need another bound and filter pass
// (new_src [Hkv, S], n_new [Hkv]).  sel_row / sel_pos [Hkv, S], n_sel [Hkv]: the selections to
// run as (candidate row, source slot).
hipError_t launch_match_sources(const int32_t *prev, const int32_t *cur, int Hkv, int m, const MfmaFilterPlan &g,
                                const int32_t *prev_nbr, const float *prev_e, int32_t *nbr, float *nbr_e,
                                const int32_t *ext, int32_t *spec_bad, const int32_t *overflow, bool first_match,
                                int32_t *new_src, int32_t *n_new, int32_t *sel_row, int32_t *sel_pos,
                                int32_t *n_sel, hipStream_t st);
// Exact top-m over candidate rows -> nbr / nbr_e [Hkv, S, m]; skips heads with overflow[h], and
// raises overflow[h] itself if a row has more candidates than it can take.  rows == nullptr:
// candidate row x -> source slot x for all S sources of src [Hkv, S]; otherwise the listed ones.
struct SelectRows {
    const int32_t *n_rows;   // [Hkv] selections per head
    const int32_t *row;      // [Hkv, S] candidate row of the x-th selection
    const int32_t *pos;      // [Hkv, S] its source slot in this round's list
};
hipError_t launch_nbr_select(const void *cand, const int32_t *cand_cnt, int32_t *overflow, const int32_t *src,
                             int Hkv, int m, const MfmaFilterPlan &g, const SelectRows *rows, int32_t *nbr,
                             float *nbr_e, hipStream_t st);

}  // namespace gkv
