/*
 * libstreamindex -- the consumer of the index lists: sparse attention over TopK(t) U Window(t)
 * (StreamIndex, Section 3, step 4).  Same library, same conventions as streamindex.h: caller-owned
 * device pointers, contiguous row-major, 16-byte aligned; work is enqueued on `stream` and the
 * call returns without synchronising; nothing is allocated; argument errors are reported before
 * anything is launched.
 *
 * The paper names this step ("a sparse attention kernel reads only TopK(t) U Window(t) for each
 * query and returns the attention output") and gives no formula.  What is computed here:
 *
 *   K_C       the compressed key/value cache of Section 3, step 1: a key's row is also its value row;
 *   TopK(t)   the entries >= 0 of the query's index list, as si_indexer_topk writes it (-1 = pad);
 *             the entries of a row must be distinct and in [0, T);
 *   Window(t) the last min(n_win, legal(t)) legal keys, legal(t)-n_win .. legal(t)-1, with
 *             legal(t) of Section 4.2 (T for SI_MASK_NONE, min(T, floor((t+1)/m)) for the causal mode);
 *   U(t)      = TopK(t) U Window(t) as a set: a key in both counts once;
 *   out[b,t,h,:] = sum_{s in U(t)} p_s K_C[b,s,:],
 *             p = softmax over U(t) of  scale * <qa[b,t,h,:], K_C[b,s,:]>;   0 where U(t) is empty.
 *
 * bf16 operands, fp32 accumulation of the dot products, fp32 softmax statistics, weights carried
 * with 16 mantissa bits into the second product, fp32 output.
 */
#ifndef STREAMINDEX_ATTENTION_H
#define STREAMINDEX_ATTENTION_H

#include "streamindex.h"

#ifdef __cplusplus
extern "C" {
#endif

/*   qa   device [B,S,H_A,D] bf16   attention queries (dims->H_I carries H_A, 1..64; D = 64 or 128)
 *   Kc   device [B,T,D] bf16       compressed cache: keys and values
 *   idx  device [B,S,k] int32      index lists (k <= 4096; n_win <= 4096)
 *   out  device [B,S,H_A,D] f32
 * One workgroup per query; no workspace.  SI_ERR_UNSUPPORTED_SHAPE for other D, H_A > 64, k or
 * n_win above 4096; SI_ERR_INVALID_ARG for null pointers, non-positive sizes, a non-finite scale. */
si_status si_sparse_attention(const void* qa, const void* Kc, const int32_t* idx, const si_dims* dims,
                              int32_t m, int32_t k, si_mask_mode mask_mode, int32_t n_win, float scale,
                              float* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* STREAMINDEX_ATTENTION_H */
