// Streaming copy with the operators' access pattern (16 bytes per lane, UNROLL vectors in flight per
// lane).  A measurement aid: its rate is the ceiling a one-pass kernel can reach on this machine and
// its known byte counts calibrate the profiler's memory counters.
#pragma once

#include "device_common.h"

namespace astra {

template <int UNROLL, bool NTL, bool NTS>
__global__ __launch_bounds__(256) void stream_copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src,
                                                          uint32_t nvec, int log2_chunk)
{
    const uint32_t first = xcd_chunked(blockIdx.x, log2_chunk) * (256u * UNROLL) + threadIdx.x;
    u32x4 v[UNROLL];
#pragma unroll
    for (int k = 0; k < UNROLL; ++k) {
        const uint32_t i = first + 256u * k;
        if (i < nvec) v[k] = load_vec<NTL>(src + i);
    }
#pragma unroll
    for (int k = 0; k < UNROLL; ++k) {
        const uint32_t i = first + 256u * k;
        if (i < nvec) store_vec<NTS>(dst + i, v[k]);
    }
}

// Streaming probes: the traffic of an operator without its arithmetic, with the flat kernels' geometry (one 16-byte
// vector per lane, BLOCK lanes per workgroup, XCD-aware order, non-temporal hint).  MODE (astra_probe_t in astra.h):
//   0 c <- a                      one read stream, one write stream
//   1 a and b are read only       two read streams (the loaded registers are consumed by an empty asm statement)
//   2 c <- a pattern              one write stream
//   3 c <- a ^ b                  two read streams, one write stream: the mix of silu_and_mul and merge_attn_states_lse
//   4 a <- a ^ b, b <- a + b      two streams updated in place: the mix of fused_add_rmsnorm
template <int MODE, int BLOCK>
__global__ __launch_bounds__(BLOCK) void stream_probe_kernel(u32x4* a, u32x4* b, u32x4* c, uint32_t nvec, int log2_chunk)
{
    const uint32_t i = xcd_chunked(blockIdx.x, log2_chunk) * uint32_t(BLOCK) + threadIdx.x;
    if (i >= nvec) return;
    u32x4 x = u32x4{i, i, i, i}, y = x;
    if constexpr (MODE != 2) x = load_vec<true>(a + i);
    if constexpr (MODE == 1 || MODE == 3 || MODE == 4) y = load_vec<true>(b + i);
    if constexpr (MODE == 1) {
        asm volatile("" : : "v"(x), "v"(y));
    } else if constexpr (MODE == 4) {
        store_vec<true>(a + i, x ^ y);
        store_vec<true>(b + i, x + y);
    } else {
        store_vec<true>(c + i, MODE == 3 ? (x ^ y) : x);
    }
}

}  // namespace astra
