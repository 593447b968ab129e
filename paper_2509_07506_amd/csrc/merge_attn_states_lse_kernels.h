// merge_attn_states_lse for gfx950 -- paper Table 1, Kernel 1:
//   V_out = (e^Sa V_a + e^Sb V_b) / (e^Sa + e^Sb),  S_out = log(e^Sa + e^Sb).
//
// One lane owns one 16-byte vector (8 elements) of one (token, head) pair.  The two mixing weights
// depend only on the pair, so a lane computes them once for its 8 elements (the hoisting of the
// paper's Fig. 2b); the lanes that share a pair read the same two scores from one cache line.
// Per lane that is 4 transcendental ops against 48 bytes of traffic, far below the memory time.
#pragma once

#include "device_common.h"

namespace astra {

struct MergeWeights {
    float a, b, lse;
};

// Dividing numerator and denominator by e^m, m = max(Sa, Sb):  a = e^(Sa-m) / (e^(Sa-m) + e^(Sb-m)),
// S_out = m + log(e^(Sa-m) + e^(Sb-m)).  The larger exponential is exactly 1 so the denominator is in
// [1, 2].  Two empty partitions (both scores -inf) give a = b = 0 and S_out = -inf.
__device__ __forceinline__ MergeWeights merge_weights(float sa, float sb)
{
    const float ninf = -__builtin_inff();
    const float m = fmaxf(sa, sb);
    const bool empty = (m == ninf);
    const float m0 = empty ? 0.0f : m;
    const float wa = fast_exp(sa - m0);
    const float wb = fast_exp(sb - m0);
    const float den = wa + wb;
    const float inv = fast_rcp(den);
    MergeWeights w;
    w.a = empty ? 0.0f : wa * inv;
    w.b = empty ? 0.0f : wb * inv;
    w.lse = empty ? ninf : m + fast_log(den);
    return w;
}

// Fast path: head_dim % 8 == 0, 16-byte aligned v pointers.  Flat list of vectors, dvec = head_dim/8
// per pair.  The pair index is a shift when dvec is a power of two (LOG2_DVEC >= 0), otherwise a
// multiply-high division.  v_out may alias v_a or v_b exactly: all loads of a lane precede its stores.
// lse_out must not alias the input scores: the lanes of one pair can sit in different waves.
template <int DT, int UNROLL, bool NTL, bool NTS, bool HOIST = true>
__global__ __launch_bounds__(256) void merge_attn_states_lse_vec_kernel(u32x4* v_out, float* lse_out, const u32x4* v_a,
                                                                        const float* lse_a, const u32x4* v_b,
                                                                        const float* lse_b, uint32_t total_vecs,
                                                                        uint32_t dvec, int log2_dvec, FastDiv by_dvec,
                                                                        int log2_chunk)
{
    const uint32_t first = xcd_chunked(blockIdx.x, log2_chunk) * (256u * UNROLL) + threadIdx.x;
    u32x4 av[UNROLL], bv[UNROLL];
    float sa[UNROLL], sb[UNROLL];
    uint32_t pair[UNROLL];
#pragma unroll
    for (int k = 0; k < UNROLL; ++k) {
        const uint32_t i = first + 256u * k;
        if (i < total_vecs) {
            pair[k] = log2_dvec >= 0 ? (i >> log2_dvec) : by_dvec.div(i);
            av[k] = load_vec<NTL>(v_a + i);
            bv[k] = load_vec<NTL>(v_b + i);
            sa[k] = lse_a[pair[k]];
            sb[k] = lse_b[pair[k]];
        }
    }
#pragma unroll
    for (int k = 0; k < UNROLL; ++k) {
        const uint32_t i = first + 256u * k;
        if (i < total_vecs) {
            const MergeWeights w = merge_weights(sa[k], sb[k]);
            float a[8], b[8], o[8];
            unpack8<DT>(av[k], a);
            unpack8<DT>(bv[k], b);
            if constexpr (HOIST) {
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = w.a * a[e] + w.b * b[e];
            } else {
                // ablation only (the pattern of the paper's Fig. 2a): the weights are worked out again for
                // every element.  The empty asm makes the score opaque so the compiler cannot merge the
                // eight evaluations back into one.
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float s = sa[k];
                    asm volatile("" : "+v"(s));
                    const MergeWeights we = merge_weights(s, sb[k]);
                    o[e] = we.a * a[e] + we.b * b[e];
                }
            }
            store_vec<NTS>(v_out + i, pack8<DT>(o));
            if (i == pair[k] * dvec) lse_out[pair[k]] = w.lse;  // first vector of the pair
        }
    }
}

// Element-wise path for any head_dim and 2-byte aligned pointers: one block per (token, head) pair.
template <int DT>
__global__ __launch_bounds__(256) void merge_attn_states_lse_generic_kernel(uint16_t* v_out, float* lse_out,
                                                                            const uint16_t* v_a, const float* lse_a,
                                                                            const uint16_t* v_b, const float* lse_b,
                                                                            int64_t pairs, int64_t D)
{
    for (int64_t p = blockIdx.x; p < pairs; p += gridDim.x) {
        const MergeWeights w = merge_weights(lse_a[p], lse_b[p]);
        for (int64_t k = threadIdx.x; k < D; k += blockDim.x) {
            float a = Storage<DT>::widen(v_a[p * D + k]);
            float b = Storage<DT>::widen(v_b[p * D + k]);
            v_out[p * D + k] = Storage<DT>::narrow(w.a * a + w.b * b);
        }
        if (threadIdx.x == 0) lse_out[p] = w.lse;
    }
}

}  // namespace astra
