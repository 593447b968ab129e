/*
 * astra_strided.h -- the three operators of astra.h (paper Table 1) for callers whose tensors are strided views
 * of larger buffers.  Arithmetic, rounding, ownership, stream and validation order are those of astra.h; strides
 * are in elements; a stride smaller than the extent it has to span is ASTRA_ERR_SHAPE; overlap is judged on the
 * bounding byte ranges of the views.  The fast path needs 16-byte aligned pointers and row lengths and strides
 * that are multiples of 16 bytes; anything else takes the ragged path of astra.h (same results up to the order of
 * binary32 roundings).  The silu_and_mul and merge_attn_states_lse views may hold at most 2^31 16-byte output
 * vectors, counting a partial last vector of a row as one (ASTRA_ERR_SHAPE otherwise).
 *
 * fused_add_rmsnorm (Kernel 2: y = (x+r)/sqrt(||x+r||^2/H + eps) (.) w) on row-strided views, with the results
 * written somewhere else than the operands if wanted.  Same arithmetic and rounding as astra_fused_add_rmsnorm (residual = one binary32 add rounded
 * once; statistics over the unrounded sum).
 *
 *   x      [T, H] dtype, device, read:    row t starts x_stride elements after row t-1
 *   r      [T, H] dtype, device, read:    row stride r_stride
 *   weight [H]    dtype, device, read
 *   y_out  [T, H] dtype, device, written: normalised, weighted rows; row stride y_stride
 *   r_out  [T, H] dtype, device, written: x + r; row stride r_out_stride
 *
 * Every stride is in elements and must be >= H (ASTRA_ERR_SHAPE otherwise).  y_out may be the very same
 * view as x (same pointer and stride) and r_out the very same view as r -- that is the in-place operator;
 * any other overlap between an output and an input or between the two outputs is ASTRA_ERR_ALIAS
 * (overlap is judged on the bounding byte ranges of the views).  The fast path needs 16-byte aligned
 * pointers and H and all strides multiples of 16 bytes (8 16-bit or 4 binary32 elements); anything else takes the
 * ragged path of astra_fused_add_rmsnorm (rows of up to 4096 vectors) or the element-wise path.
 */
#ifndef ASTRA_STRIDED_H
#define ASTRA_STRIDED_H

#include "astra.h"

#ifdef __cplusplus
extern "C" {
#endif

astra_status_t astra_fused_add_rmsnorm_strided(void* y_out, int64_t y_stride, void* r_out, int64_t r_out_stride,
                                               const void* x, int64_t x_stride, const void* r, int64_t r_stride,
                                               const void* weight, int64_t T, int64_t H, astra_dtype_t dtype, float eps,
                                               hipStream_t stream);

/*
 * silu_and_mul (Kernel 3: out = SiLU(x) (.) g) on row-strided views.
 *
 *   input [T, 2d] dtype, device, read:    row t starts in_stride elements after row t-1 (in_stride >= 2d);
 *                                         columns [0, d) of a row are x, columns [d, 2d) are g
 *   out   [T, d]  dtype, device, written: row stride out_stride >= d
 *
 * `out` must not overlap `input` (ASTRA_ERR_ALIAS).
 */
astra_status_t astra_silu_and_mul_strided(void* out, int64_t out_stride, const void* input, int64_t in_stride, int64_t T,
                                          int64_t d, astra_dtype_t dtype, hipStream_t stream);

/*
 * merge_attn_states_lse (Kernel 1: V_out = (e^Sa V_a + e^Sb V_b)/(e^Sa + e^Sb), S_out = log(e^Sa + e^Sb)) with
 * strided value tensors: element (t, h, k) of v_a lives at v_a[t*a_token_stride + h*a_head_stride + k], likewise
 * v_b and v_out (each head's head_dim values are dense; head_stride >= head_dim, token_stride >=
 * (num_heads-1)*head_stride + head_dim).  The scores lse_a, lse_b, lse_out stay dense [T, num_heads] binary32.
 * This covers head_dim slices of a wider per-head buffer and padded or interleaved head layouts.
 *
 * v_out may be the very same view as v_a or v_b (same pointer and strides); any other overlap of v_out with an
 * input, and any overlap of lse_out with lse_a or lse_b, is ASTRA_ERR_ALIAS.
 */
astra_status_t astra_merge_attn_states_lse_strided(void* v_out, int64_t out_token_stride, int64_t out_head_stride,
                                                   float* lse_out, const void* v_a, int64_t a_token_stride,
                                                   int64_t a_head_stride, const float* lse_a, const void* v_b,
                                                   int64_t b_token_stride, int64_t b_head_stride, const float* lse_b,
                                                   int64_t T, int64_t num_heads, int64_t head_dim, astra_dtype_t dtype,
                                                   hipStream_t stream);

#ifdef __cplusplus
}
#endif

#endif /* ASTRA_STRIDED_H */
