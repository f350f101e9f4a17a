/*
 * CPU oracle for the lightning-indexer top-k step (StreamIndex, Sections 1, 3 and 4).
 *
 * TEST INFRASTRUCTURE ONLY.  This library is the slow, plain definition that the
 * GPU path is checked against.  It shares no code with the HIP library and is
 * never called by it.  Host pointers only.
 *
 * What it computes (Section 1 and Section 3, the indexer score; Section 4.1, the
 * total order; Section 4.2, the effective k):
 *
 *   I(t, s)   = sum_h  w[t,h] * max(0, sum_d q[t,h,d] * K[s,d])        (fp64)
 *   legal(t)  = T                      if mask_mode == 0
 *             = min(T, floor((t+1)/m)) if mask_mode == 1  (causal block mask)
 *   result(t) = the min(k, legal(t)) legal keys that are largest under
 *               (a,i) > (b,j)  <=>  a > b  or  (a == b and i < j),
 *               listed best first; remaining slots idx = -1, score = -inf.
 *
 * q and K are bfloat16 bit patterns (uint16_t), w is float.  Every product and
 * sum is done in double.
 *
 * Pins (tests/test_oracle_*.py): hand-worked integer fixture, planted keys,
 * w == 0 tie order, duplicated keys, pad structure and its closed-form count,
 * ReLU(x) - ReLU(-x) = x identity against a plain mat-vec, exact power-of-two
 * scaling, single-head non-negative case against a library sort, key
 * permutation invariance, Algorithm 1 and Algorithm 2 agreeing with the full
 * sort, footprint figures printed in the paper.  The attention consumer
 * (si_oracle_sparse_attention_rows): dense masked softmax attention in numpy,
 * constant-value rows, zero queries (uniform weights), window-only = local
 * attention, list order and duplicates, a huge scale (argmax), empty sets.
 * Absolute score values on random inputs have no figure in the paper to compare
 * with; they are pinned through the identities and the brute-force case only.
 */
#ifndef SI_ORACLE_H
#define SI_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Number of legal keys of query position t (Section 4.2). */
int64_t si_oracle_legal_count(int64_t t, int64_t T, int32_t m, int32_t mask_mode);

/* fp64 scores of one query against keys [0, n_keys).  q_row: [H, D] bf16 bits,
 * K: [T, D] bf16 bits (n_keys <= T), w_row: [H].  out: [n_keys]. */
int32_t si_oracle_score_row(const uint16_t* q_row, const uint16_t* K, const float* w_row,
                            int32_t H, int32_t D, int64_t n_keys, double* out);

/* fp64 scores of one query at the listed key indices (idx[i] < 0 gives NaN). */
int32_t si_oracle_score_at(const uint16_t* q_row, const uint16_t* K, const float* w_row,
                           int32_t H, int32_t D, const int32_t* idx, int64_t n_idx,
                           double* out);

/* Full sort of scores[0, L) under the total order; writes the best min(k, L)
 * then pads.  out_idx: [k], out_score: [k] (fp64, -inf pads). */
int32_t si_oracle_sort_topk(const double* scores, int64_t L, int32_t k,
                            int32_t* out_idx, double* out_score);

/* Top-k for a list of query rows.  q_rows: [n_rows, H, D], w_rows: [n_rows, H],
 * K: [B, T, D]; row r is query position t_of_row[r] of batch b_of_row[r].
 * out_idx: [n_rows, k] int32, out_score: [n_rows, k] fp64.
 * n_threads > 1 only fans rows out over threads; each row is computed by the
 * same single-threaded routine.  Returns 0, or a negative code on bad input. */
int32_t si_oracle_topk_rows(const uint16_t* q_rows, const float* w_rows, const uint16_t* K,
                            const int32_t* b_of_row, const int64_t* t_of_row, int64_t n_rows,
                            int32_t H, int32_t D, int64_t T, int32_t m, int32_t k,
                            int32_t mask_mode, int32_t* out_idx, double* out_score,
                            int32_t n_threads);

/* Algorithm 1: bounded min-heap under the total order, keys visited in the
 * order perm[0..L).  Returns the kept set sorted best first, padded. */
int32_t si_oracle_stream_topk(const double* scores, int64_t L, const int64_t* perm,
                              int32_t k, int32_t* out_idx, double* out_score);

/* Algorithm 2 for one query row, on precomputed scores over all T keys:
 * key tiles of c_T, per-tile mask from the legal count, per-tile
 * top-min(k, c_T), merge into a running buffer.
 * variant 0 = as stated; 1 = merge step dropped after the first tile
 * (ablation A1); 2 = tiles with c_T < k skipped (ablation A2). */
int32_t si_oracle_chunked_topk_row(const double* scores, int64_t T, int64_t legal,
                                   int32_t k, int64_t c_T, int32_t variant,
                                   int32_t* out_idx, double* out_score);

/* The consumer of the index lists (Section 3, step 4: "a sparse attention kernel reads only
 * TopK(t) U Window(t) for each query"), as this build reads it (the paper gives no formula):
 *   K_C is the compressed key/value cache: a key's row is also its value row (Section 3, step 1);
 *   TopK(t)   = the entries >= 0 of the query's index list (any order, -1 = pad);
 *   Window(t) = the last min(n_win, legal(t)) legal keys: legal(t)-n_win .. legal(t)-1;
 *   U(t)      = TopK(t) U Window(t) as a SET (a key in both counts once);
 *   out[t,h,:] = sum_{s in U} p_s K_C[s,:],  p = softmax over U of scale * <qa[t,h,:], K_C[s,:]>,
 *   and out = 0 when U is empty.
 * qa_rows: [n_rows, H, D] bf16 bits, K: [B, T, D] bf16 bits, idx_rows: [n_rows, k] (entries -1 or
 * in [0, T)), out: [n_rows, H, D] fp64.  Every product, exponential and sum in double; the set is
 * visited in ascending key order.  Returns 0, -1 on bad arguments, -2 on an index outside [-1, T). */
int32_t si_oracle_sparse_attention_rows(const uint16_t* qa_rows, const uint16_t* K,
                                        const int32_t* idx_rows, const int32_t* b_of_row,
                                        const int64_t* t_of_row, int64_t n_rows, int32_t H,
                                        int32_t D, int64_t T, int32_t m, int32_t k,
                                        int32_t mask_mode, int32_t n_win, double scale,
                                        double* out, int32_t n_threads);

/* Bytes of the [B, S, H, T] fp32 intermediate that the method avoids. */
uint64_t si_oracle_materialize_bytes(int64_t B, int64_t S, int64_t H, int64_t T);

/* Bytes of a [B, S, T] one-byte causal mask (Section 5, per-chunk mask). */
uint64_t si_oracle_mask_bytes(int64_t B, int64_t S, int64_t T);

#ifdef __cplusplus
}
#endif
#endif
