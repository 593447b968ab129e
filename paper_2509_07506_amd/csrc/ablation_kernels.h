// Ablation kernels: the tuned kernels with ONE of the paper's optimisations taken out again, so that its
// worth on gfx950 can be measured (the paper's Figs. 2a, 3a, 4a, 5a show the corresponding CUDA
// "baseline" patterns).  The hoisting, reduction and fast-math toggles are template flags of the tuned
// kernels; this file holds the remaining toggle, scalar 16-bit loads and stores (Fig. 4a): the same
// work decomposition as the tuned kernels, but one element per lane access instead of eight.
#pragma once

#include "device_common.h"
#include "merge_attn_states_lse_kernels.h"
#include "silu_and_mul_kernels.h"

namespace astra {

// silu_and_mul, one element per lane; flat element index over [T, d], n = T*d < 2^32.
template <int DT>
__global__ __launch_bounds__(256) void silu_and_mul_scalar_kernel(uint16_t* __restrict__ out,
                                                                  const uint16_t* __restrict__ in, uint32_t n, uint32_t d,
                                                                  FastDiv by_d)
{
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i >= n) return;
    const uint32_t t = by_d.div(i);
    const uint32_t j = i - t * d;
    const uint16_t* row = in + (size_t)t * 2u * d;
    const float x = Storage<DT>::widen(row[j]);
    const float g = Storage<DT>::widen(row[d + j]);
    out[i] = Storage<DT>::narrow(silu_fast(x) * g);
}

// merge, one element per lane; flat element index over [pairs, D], n = pairs*D < 2^32.  Weights are
// still computed once per lane (i.e. per element here: a lane has only one).
template <int DT>
__global__ __launch_bounds__(256) void merge_attn_states_lse_scalar_kernel(uint16_t* v_out, float* lse_out,
                                                                           const uint16_t* v_a, const float* lse_a,
                                                                           const uint16_t* v_b, const float* lse_b,
                                                                           uint32_t n, uint32_t D, FastDiv by_D)
{
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i >= n) return;
    const uint32_t p = by_D.div(i);
    const MergeWeights w = merge_weights(lse_a[p], lse_b[p]);
    const float a = Storage<DT>::widen(v_a[i]);
    const float b = Storage<DT>::widen(v_b[i]);
    v_out[i] = Storage<DT>::narrow(blend(w, a, b));
    if (i == p * D) lse_out[p] = w.lse;
}

// fused_add_rmsnorm, one workgroup per row, the row resident in registers as in the tuned kernel, but
// every access is a single 16-bit element: lane t owns elements t, t + blockDim.x, ... (at most EPT).
template <int DT, int EPT>
__global__ __launch_bounds__(1024) void fused_add_rmsnorm_scalar_kernel(uint16_t* input, uint16_t* residual,
                                                                        const uint16_t* __restrict__ weight, int64_t T,
                                                                        uint32_t H, float inv_h, float eps)
{
    __shared__ float partials[2][16];
    int parity = 0;
    for (int64_t row = blockIdx.x; row < T; row += gridDim.x, parity ^= 1) {
        uint16_t* x = input + row * H;
        uint16_t* r = residual + row * H;
        float s[EPT];
        float acc = 0.0f;
#pragma unroll
        for (int k = 0; k < EPT; ++k) {
            const uint32_t j = threadIdx.x + k * blockDim.x;
            s[k] = 0.0f;
            if (j < H) {
                s[k] = Storage<DT>::widen(x[j]) + Storage<DT>::widen(r[j]);
                acc += s[k] * s[k];
                r[j] = Storage<DT>::narrow(s[k]);
            }
        }
        const float total = block_sum(acc, partials[parity], blockDim.x >> 6);
        const float scale = rsqrt_full_range(total * inv_h + eps);
#pragma unroll
        for (int k = 0; k < EPT; ++k) {
            const uint32_t j = threadIdx.x + k * blockDim.x;
            if (j < H) x[j] = Storage<DT>::narrow((s[k] * scale) * Storage<DT>::widen(weight[j]));
        }
    }
}

}  // namespace astra
