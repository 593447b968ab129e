/*
 * astra_ablation.h -- the three operators of astra.h with ONE optimisation removed again, for measuring
 * what each of the optimisations the paper (arxiv 2509.07506) reports is worth on MI355X.  The paper's
 * case studies show a CUDA "baseline" pattern next to each optimised one: weights recomputed inside the
 * element loop (Fig. 2a), a shared-memory-only tree reduction (Fig. 3a), scalar 16-bit loads (Fig. 4a),
 * library expf plus a divide (Fig. 5a).  Each variant below puts one of these patterns back into the
 * tuned gfx950 kernel and leaves everything else alone.  Results are the same as the tuned operators'
 * within the operators' tolerances (the residual stays bit-exact).
 *
 * Arguments, layouts, ownership and validation are exactly those of the corresponding function in
 * astra.h.  In addition: a variant that does not apply to the operator, or a shape outside what the
 * variant supports (variants 1 to 4 need 16-byte aligned pointers and rows that are a multiple of 8 elements,
 * i.e. the fast path; scalar-load variants need fewer than 2^32 elements and, for rmsnorm, H <= 16384),
 * returns ASTRA_ERR_VARIANT and does nothing.
 */
#ifndef ASTRA_ABLATION_H
#define ASTRA_ABLATION_H

#include "astra.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ASTRA_VARIANT_TUNED = 0,              /* the kernel astra.h runs */
    ASTRA_VARIANT_SCALAR_LOADS = 1,       /* all three: one 16-bit element per load/store instead of 128-bit vectors */
    ASTRA_VARIANT_LDS_TREE_REDUCTION = 2, /* fused_add_rmsnorm: LDS tree with a barrier per step instead of DPP + one LDS float per wave */
    ASTRA_VARIANT_UNHOISTED_WEIGHTS = 3,  /* merge_attn_states_lse: mixing weights recomputed for every element */
    ASTRA_VARIANT_LIBM_EXP_DIVIDE = 4,    /* silu_and_mul: library expf and an IEEE divide instead of v_exp_f32 / v_rcp_f32 */
    ASTRA_VARIANT_ELEMENT_WISE = 5,       /* all three: the plain element-wise kernels that astra.h keeps for inputs beyond the
                                             limits of its other paths, here on any valid input (every storage type, any
                                             row length and alignment), so that they can be checked and timed at ordinary sizes */
    /* fused_add_rmsnorm only, every storage type: the tuned row kernel with its request pacing (ASTRA_PACE_* in
       astra_plan.h) forced instead of chosen by the launch policy, so that the policy's table can be re-measured.
       Same arithmetic and results as the tuned kernel.  ASTRA_ERR_VARIANT unless the shape runs one row per workgroup
       on the 16-byte path (rows of at most 4096 vectors, 16-byte aligned, fewer than 2^21 rows). */
    ASTRA_VARIANT_PACE_NONE = 6,          /* every request as early as possible */
    ASTRA_VARIANT_PACE_STORE_GAP = 7,     /* output store held until the residual store has completed */
    ASTRA_VARIANT_PACE_X_BEFORE_R = 8,    /* x arrived before r is requested */
    ASTRA_VARIANT_PACE_WEIGHT_X_R = 9,    /* weight, then x, then r, one after the other */
    /* fused_add_rmsnorm only, every storage type, the same shapes as variants 6 to 9: the tuned row kernel, paced as the
       launch policy says, with its two stores at device scope (the line goes on to memory instead of staying dirty in
       the L2) instead of plain non-temporal stores.  Not an optimisation of the paper: a choice this library measured
       and decided against (a small gain on some tensors far larger than the last-level cache, a loss of 2-15 % on
       cache-sized ones); the variants keep the measurement repeatable.  Same results as the tuned kernel. */
    ASTRA_VARIANT_STORE_DEVICE_SCOPE_WHOLE_LINES = 10, /* for rows that begin and end on 128-byte lines only */
    ASTRA_VARIANT_STORE_DEVICE_SCOPE = 11,             /* for every row (rows that share lines lose 15-25 % with it) */
    ASTRA_ENUM_SPANS_INT32(ASTRA_VARIANT)
} astra_variant_t;

/* ASTRA_ERR_VARIANT (astra.h): variant not applicable to this operator, shape or storage type (variants 1 to 4 exist
 * for the 16-bit types only). */

astra_status_t astra_ablation_fused_add_rmsnorm(void* input, void* residual, const void* weight, int64_t T, int64_t H,
                                                astra_dtype_t dtype, float eps, astra_variant_t variant,
                                                hipStream_t stream);

astra_status_t astra_ablation_silu_and_mul(void* out, const void* input, int64_t T, int64_t d, astra_dtype_t dtype,
                                           astra_variant_t variant, hipStream_t stream);

astra_status_t astra_ablation_merge_attn_states_lse(void* v_out, float* lse_out, const void* v_a, const float* lse_a,
                                                    const void* v_b, const float* lse_b, int64_t T, int64_t num_heads,
                                                    int64_t head_dim, astra_dtype_t dtype, astra_variant_t variant,
                                                    hipStream_t stream);

#ifdef __cplusplus
}
#endif

#endif /* ASTRA_ABLATION_H */
