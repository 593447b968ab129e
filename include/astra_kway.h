/*
 * astra_kway.h -- K-way merge of partial attention states: the K-term form of the paper's Table 1,
 * Kernel 1 (arxiv 2509.07506),
 *
 *     V_out = sum_k e^(S_k) V_k / sum_k e^(S_k),      S_out = log sum_k e^(S_k)        (natural log).
 *
 * The paper defines the two-way operator only; merging is associative, so this equals any chain of K-1
 * two-way merges (up to rounding) while reading every partial state once and writing one result:
 * (K+1) tensor passes instead of 3(K-1).  It is the combine step after a split-KV attention that left
 * K partial outputs per token.
 *
 *   v_parts   [K, T, num_heads, head_dim] dtype, device, read only (the K partial outputs, stacked)
 *   lse_parts [K, T, num_heads] binary32, device, read only (-inf marks an empty partition)
 *   v_out     [T, num_heads, head_dim] dtype, device, written
 *   lse_out   [T, num_heads] binary32, device, written
 *
 * Evaluated in binary32 with the (running) maximum score subtracted: the partitions are folded in order,
 * four at a time, into running sums that are rescaled when the maximum grows; one rounding at the end.
 * That equals the definition up to binary32 rounding.  A single non-empty partition is returned unchanged; all
 * partitions empty give V_out = 0 and S_out = -inf.  K = 2 computes what astra_merge_attn_states_lse
 * computes on the two slices.  Outputs must not overlap inputs (ASTRA_ERR_ALIAS).  K must be in
 * [1, 65536] and the output must hold at most 2^31 16-byte vectors, counting a partial last vector of a pair as
 * one (ASTRA_ERR_SHAPE otherwise).  Everything else -- ownership, stream, validation order,
 * alignment rules, the slower paths for a head_dim that is not a whole number of 16-byte vectors or for pointers that
 * are only element aligned -- is as in astra.h.
 */
#ifndef ASTRA_KWAY_H
#define ASTRA_KWAY_H

#include "astra.h"

#ifdef __cplusplus
extern "C" {
#endif

astra_status_t astra_merge_attn_states_lse_kway(void* v_out, float* lse_out, const void* v_parts,
                                                const float* lse_parts, int64_t K, int64_t T, int64_t num_heads,
                                                int64_t head_dim, astra_dtype_t dtype, hipStream_t stream);

#ifdef __cplusplus
}
#endif

#endif /* ASTRA_KWAY_H */
