/*
 * astra.h -- C ABI of the MI355X (gfx950) implementation of the three LLM-serving operators that the
 * Astra paper (arxiv 2509.07506) optimises: Table 1 of the paper defines each computation, Section 6.1
 * gives the tensor shapes ([seq_len, num_heads, head_dim] for the merge, [batch, hidden] for the others).
 *
 * General rules for every entry point
 *   - All data pointers are DEVICE pointers (HIP global memory on the current device).  The caller owns
 *     every buffer; the library allocates nothing, keeps no state between calls and is re-entrant.
 *   - Tensors are dense, row-major, without strides.  `dtype` names the storage type of the activation
 *     tensors: IEEE binary16 (ASTRA_F16), bfloat16 (ASTRA_BF16) -- the types the serving workloads use --
 *     or IEEE binary32 (ASTRA_F32, a convenience).  Scores are always IEEE binary32.
 *   - Arithmetic is binary32 inside the kernels; each stored 16-bit value is rounded once,
 *     round-to-nearest-even, subnormals preserved; binary32 storage is written unrounded.
 *   - The work is enqueued on `stream` (NULL = the default stream) and the call returns without
 *     synchronising.
 *   - Errors are reported by return value only.  Arguments are validated, in the order
 *     null -> shape -> dtype -> eps -> alignment -> aliasing, before any HIP call is made, so a bad call
 *     never touches the device.  T == 0 is valid and does nothing.
 *   - Pointers must be aligned to their element size (2 or 4 bytes, scores 4 bytes).  The fast path needs
 *     16-byte aligned pointers and a row length that is a multiple of 16 bytes (8 16-bit or 4 binary32
 *     elements); anything else is served by other paths that compute the same thing.  The usual one works on the
 *     16-byte aligned chunks of memory the OUTPUT covers, at nearly the fast path's rate: silu_and_mul and
 *     merge_attn_states_lse for any element-aligned dense tensors with rows of at least eight vectors (d) / one
 *     vector (head_dim),
 *     fused_add_rmsnorm when its activation tensors are in step with each other (congruent modulo 16 bytes, as all
 *     16-byte aligned dense tensors are).  Otherwise 16-byte accesses at element alignment (fused_add_rmsnorm tensors
 *     out of step, shorter rows), and plain element-wise kernels for fused_add_rmsnorm rows of more than 4096
 *     vectors or less than one and for inputs beyond 2^31 vectors.  Equal up to the order of binary32 roundings; the
 *     residual of fused_add_rmsnorm is bit-identical on every path.
 *   - Nothing outside a tensor is ever written.  One path READS outside: the chunked path of fused_add_rmsnorm loads
 *     whole 16-byte aligned chunks, so at the two ends of a tensor that does not start or end on the 16-byte grid it
 *     reads up to 14 bytes outside it; such a read stays inside the 16-byte aligned block (hence the page) that holds
 *     the tensor's first or last element.
 *   - Element counts (T*H, T*2d, T*num_heads*head_dim) may exceed 2^31; they must fit in int64.
 */
#ifndef ASTRA_H
#define ASTRA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Same declaration as in the HIP runtime headers; repeating a typedef is legal in C11 and C++. */
typedef struct ihipStream_t* hipStream_t;

/* Every enumeration of this interface also lists the two ends of the 32-bit integer range.  They are not values to
 * pass: they make every int a representable value of the type, so that a call with an unknown code is a well-defined
 * input in C and in C++ alike, which the library answers with an error code. */
#define ASTRA_ENUM_SPANS_INT32(prefix) prefix##_INT32_MIN_ = -0x7fffffff - 1, prefix##_INT32_MAX_ = 0x7fffffff

typedef enum { ASTRA_F16 = 0, ASTRA_BF16 = 1, ASTRA_F32 = 2, ASTRA_ENUM_SPANS_INT32(ASTRA_DTYPE) } astra_dtype_t;

typedef enum {
    ASTRA_OK = 0,
    ASTRA_ERR_NULL = 1,   /* a required pointer is NULL */
    ASTRA_ERR_SHAPE = 2,  /* T < 0, a row dimension <= 0, or an element count overflows int64 */
    ASTRA_ERR_DTYPE = 3,  /* dtype is not one of astra_dtype_t */
    ASTRA_ERR_EPS = 4,    /* eps is negative or NaN */
    ASTRA_ERR_ALIGN = 5,  /* a pointer is not aligned to its element size */
    ASTRA_ERR_ALIAS = 6,  /* an output overlaps an input it must not overlap */
    ASTRA_ERR_LAUNCH = 7, /* the HIP runtime refused the kernel launch */
    ASTRA_ERR_VARIANT = 8, /* astra_ablation.h only: the variant does not apply to this operator, shape or storage type */
    ASTRA_ENUM_SPANS_INT32(ASTRA_STATUS)
} astra_status_t;

/*
 * fused_add_rmsnorm -- Table 1, Kernel 2:  y = (x + r) / sqrt(||x + r||^2 / H + eps) (.) w.
 *
 *   input    [T, H] dtype, device, read and written:  on return holds y
 *   residual [T, H] dtype, device, read and written:  on return holds x + r
 *   weight   [H]    dtype, device, read only
 *   eps      >= 0, added to the mean square inside the square root
 *
 * Per row: s = float(x) + float(r) (one binary32 add); residual <- round(s); the mean square is taken
 * over the unrounded s; input <- round(s * rsqrt(ms + eps) * float(w)).  `input` and `residual` must
 * not overlap each other or `weight`.
 */
astra_status_t astra_fused_add_rmsnorm(void* input, void* residual, const void* weight, int64_t T, int64_t H,
                                       astra_dtype_t dtype, float eps, hipStream_t stream);

/*
 * silu_and_mul -- Table 1, Kernel 3:  out = SiLU(x) (.) g,  SiLU(z) = z / (1 + e^-z).
 *
 *   input [T, 2d] dtype, device, read only:  columns [0, d) are x, columns [d, 2d) are g
 *   out   [T, d]  dtype, device, written
 *
 * out[t, j] = round(silu(float(x[t, j])) * float(g[t, j])).  `out` must not overlap `input`
 * (ASTRA_ERR_ALIAS).
 */
astra_status_t astra_silu_and_mul(void* out, const void* input, int64_t T, int64_t d, astra_dtype_t dtype,
                                  hipStream_t stream);

/*
 * merge_attn_states_lse -- Table 1, Kernel 1:
 *   V_out = (e^Sa V_a + e^Sb V_b) / (e^Sa + e^Sb),   S_out = log(e^Sa + e^Sb)      (natural log).
 *
 *   v_a, v_b  [T, num_heads, head_dim] dtype, device, read only
 *   lse_a, lse_b [T, num_heads] binary32, device, read only (the scores S; -inf marks an empty partition)
 *   v_out     [T, num_heads, head_dim] dtype, device, written
 *   lse_out   [T, num_heads] binary32, device, written
 *
 * Evaluated with the maximum score subtracted so that nothing overflows.  One empty side returns the
 * other side unchanged; two empty sides give V_out = 0 and S_out = -inf.  v_out may be exactly the same
 * buffer as v_a or v_b (every element is read before it is written, by the same work-item); any other
 * overlap of v_out with an input, and any overlap of lse_out with lse_a or lse_b, is ASTRA_ERR_ALIAS.
 */
astra_status_t astra_merge_attn_states_lse(void* v_out, float* lse_out, const void* v_a, const float* lse_a,
                                           const void* v_b, const float* lse_b, int64_t T, int64_t num_heads,
                                           int64_t head_dim, astra_dtype_t dtype, hipStream_t stream);

/*
 * Measurement aid, not one of the paper's operators: copies `nbytes` bytes (device to device, both
 * pointers 16-byte aligned, nbytes a multiple of 16) with the same 16-byte-per-lane access pattern the
 * operators use.  It gives the streaming ceiling of the machine and the scale of the profiler's
 * FETCH_SIZE / WRITE_SIZE counters.  Errors: ASTRA_ERR_NULL, ASTRA_ERR_SHAPE (nbytes < 0 or not a
 * multiple of 16), ASTRA_ERR_ALIGN, ASTRA_ERR_LAUNCH.
 */
astra_status_t astra_stream_copy(void* dst, const void* src, int64_t nbytes, hipStream_t stream);

/*
 * Measurement aid, not one of the paper's operators: moves `nbytes` bytes per stream with the traffic mix of an
 * operator and none of its arithmetic, with the launch geometry the operators use, so that an operator's time can be
 * set against what the machine does for the same bytes.  a, b, c: device buffers of nbytes each, 16-byte aligned,
 * pairwise disjoint, nbytes a multiple of 16; a buffer the mode does not touch may be NULL.
 */
typedef enum {
    ASTRA_PROBE_COPY = 0,         /* c <- a: one read stream, one write stream */
    ASTRA_PROBE_READ2 = 1,        /* a and b are read, nothing is written */
    ASTRA_PROBE_WRITE1 = 2,       /* c is written; 256-lane workgroups at every size (a single-wave workgroup per
                                     1 KiB store would measure the workgroup launch rate, not memory) */
    ASTRA_PROBE_READ2_WRITE1 = 3, /* c <- a ^ b: the mix of silu_and_mul and merge_attn_states_lse */
    ASTRA_PROBE_UPDATE2 = 4,      /* a <- a ^ b, b <- a + b, in place: the mix of fused_add_rmsnorm */
    ASTRA_ENUM_SPANS_INT32(ASTRA_PROBE)
} astra_probe_t;

/* Errors: ASTRA_ERR_NULL (a buffer the mode uses is NULL), ASTRA_ERR_SHAPE (nbytes < 0, not a multiple of 16, more than
 * 2^31 vectors, or an unknown mode), ASTRA_ERR_ALIGN, ASTRA_ERR_ALIAS, ASTRA_ERR_LAUNCH. */
astra_status_t astra_stream_probe(void* a, void* b, void* c, int64_t nbytes, astra_probe_t mode, hipStream_t stream);

/* Static, NUL-terminated description of a status code. */
const char* astra_status_string(astra_status_t status);

#ifdef __cplusplus
}
#endif

#endif /* ASTRA_H */
