/*
 * astra_plan.h -- introspection of the host-side dispatch of the astra library: which kernel variant
 * and launch geometry a call with the given shape would use.  Pure host arithmetic, no HIP call, so it
 * can be exercised on a machine without a GPU.  The operators themselves are declared in astra.h.
 */
#ifndef ASTRA_PLAN_H
#define ASTRA_PLAN_H

#include <stdint.h>

#include "astra.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ASTRA_PATH_NONE = 0,    /* nothing to launch (T == 0) */
    ASTRA_PATH_VECTOR = 1,  /* 16-byte-per-lane fast path */
    ASTRA_PATH_GENERIC = 2, /* element-wise path: rmsnorm rows of more than 4096 vectors or less than one, inputs beyond
                               the 32-bit vector index */
    ASTRA_PATH_RAGGED = 3,  /* 16-byte accesses at element alignment, loads and stores alike, the partial last vector of a row
                               element-wise: fused_add_rmsnorm with its activation tensors at unrelated offsets into the
                               16-byte grid; silu_and_mul with rows (d) under eight vectors and merge_attn_states_lse
                               with rows (head_dim) under one, row-strided views, or more than 2^31 (2^32) elements */
    ASTRA_PATH_PHASED = 4   /* row lengths that are no whole number of vectors, or pointers that are only element aligned:
                               lanes own the 16-byte aligned chunks of memory the output covers, so every store is an
                               aligned one (the partial chunk at an end element-wise); runs at nearly the vector path's
                               rate.  silu_and_mul and merge_attn_states_lse: any dense tensors with rows of at least
                               eight vectors / one vector, loads at element alignment.  fused_add_rmsnorm (in place, so loads and stores
                               share their chunks): activation tensors in step with each other (congruent modulo 16
                               bytes -- every dense call on 16-byte aligned tensors is); it also takes this path for
                               16-byte aligned rows of whole vectors that are no whole number of 128-byte lines, on
                               streaming grids: its chunks are counted from the line, so its waves stay on whole lines */
} astra_path_t;

typedef struct {
    int32_t path;             /* astra_path_t */
    int32_t block;            /* work-items per workgroup */
    int32_t vectors_per_lane; /* 16-byte vectors each lane keeps in flight (0 on the generic path) */
    int32_t log2_xcd_chunk;   /* workgroups an XCD runs back to back cover 2^this consecutive work units */
    int64_t grid;             /* workgroups launched (padded to a multiple of 8 * 2^log2_xcd_chunk) */
    int32_t pace;             /* fused_add_rmsnorm fast path only: ASTRA_PACE_* bits, when a wave issues its requests */
    int32_t rows_per_block;   /* fused_add_rmsnorm on rows of at most 32 vectors: rows one workgroup handles; otherwise 0 */
    int32_t access_bytes;     /* bytes one lane moves per access on the vector path: 16, or 8 for small silu_and_mul problems;
                                 0 on the other paths */
    int32_t non_temporal;     /* 1: activations are moved with the non-temporal hint (streaming sizes); 0: plain cached
                                 accesses (small silu_and_mul / merge problems, where the launch ends sooner with them) */
} astra_launch_info_t;

/* Request pacing of the fused_add_rmsnorm row kernel.  Same arithmetic and bytes for every value; the order in time of
 * a wave's requests changes the streaming rate by a few per cent, so the library picks it per shape from measurements. */
enum {
    ASTRA_PACE_NONE = 0,         /* every request as early as possible (few rows: shortest dependent chain) */
    ASTRA_PACE_WEIGHT_FIRST = 1, /* the weight has arrived before the activations are requested */
    ASTRA_PACE_X_BEFORE_R = 2,   /* x has arrived before r is requested */
    ASTRA_PACE_STORE_GAP = 4,    /* the residual store has completed before the output store is issued */
    ASTRA_PACE_ONE_RESIDENT = 8  /* not a wait: the workgroup reserves 96 KiB of LDS so that a compute unit holds one
                                    workgroup at a time (long rows: two resident ones keep too many loads in flight) */
};

/* `dtype` is the storage type of the call.  `aligned16` tells how the tensor pointers of the call sit on the 16-byte
 * grid: 1 = every pointer is 16-byte aligned; 2 = not, but the activation tensors (input and residual; input and out;
 * v_a, v_b and v_out) are congruent modulo 16 bytes; 0 = element alignment only (1 against the rest decides for
 * silu_and_mul and merge_attn_states_lse, 2 against 0 matters to fused_add_rmsnorm only).  Each function validates like its operator does
 * (ASTRA_ERR_NULL for `info`, ASTRA_ERR_SHAPE, ASTRA_ERR_DTYPE). */
astra_status_t astra_plan_fused_add_rmsnorm(int64_t T, int64_t H, astra_dtype_t dtype, int aligned16,
                                            astra_launch_info_t* info);
astra_status_t astra_plan_silu_and_mul(int64_t T, int64_t d, astra_dtype_t dtype, int aligned16, astra_launch_info_t* info);
astra_status_t astra_plan_merge_attn_states_lse(int64_t T, int64_t num_heads, int64_t head_dim, astra_dtype_t dtype,
                                                int aligned16, astra_launch_info_t* info);

/* The map from workgroup index to work unit that the kernels apply when log2_xcd_chunk > 0 (the same
 * function the device code runs): workgroup b executes on XCD b % 8, and the workgroups of one XCD are
 * given runs of 2^log2_chunk consecutive units.  A permutation of [0, G) for every G that is a multiple
 * of 8 * 2^log2_chunk.  log2_chunk outside [0, 8] returns `workgroup` unchanged. */
uint32_t astra_plan_xcd_chunked(uint32_t workgroup, int log2_chunk);

/* What the HIP runtime reports about device `device`'s memory system: memory clock in kHz and bus width in
 * bits (HBM3E moves four bits per pin and reported clock: bandwidth = 4 * clock * width / 8).  The only function of this
 * header that calls the runtime.  ASTRA_ERR_NULL for a NULL output, ASTRA_ERR_LAUNCH if the query fails. */
astra_status_t astra_device_memory_info(int device, int* memory_clock_khz, int* memory_bus_bits);

#ifdef __cplusplus
}
#endif

#endif /* ASTRA_PLAN_H */
