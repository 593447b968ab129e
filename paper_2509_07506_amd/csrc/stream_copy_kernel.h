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

}  // namespace astra
