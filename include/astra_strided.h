/*
 * astra_strided.h -- fused_add_rmsnorm (paper Table 1, Kernel 2: y = (x+r)/sqrt(||x+r||^2/H + eps) (.) w)
 * for callers whose tensors are row-strided views or who want the results somewhere else than in the
 * operands.  Same arithmetic and rounding as astra_fused_add_rmsnorm (residual = one binary32 add rounded
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
 * pointers and H and all strides multiples of 16 bytes (8 16-bit or 4 binary32 elements); anything else takes the element-wise path.  Everything
 * else -- ownership, stream, validation order, error codes -- is as in astra.h.
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

#ifdef __cplusplus
}
#endif

#endif /* ASTRA_STRIDED_H */
