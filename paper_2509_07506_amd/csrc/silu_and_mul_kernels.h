// silu_and_mul for gfx950 -- paper Table 1, Kernel 3: out = SiLU(x) (.) g, SiLU(z) = z / (1 + e^-z).
//
// The operator is a pure stream: 2 input vectors and 1 output vector per N results (N = 8 for the
// 16-bit storage types, 4 for binary32), no reuse.  The
// fast kernel gives every lane 16-byte accesses and `UNROLL` independent vector pairs so that enough
// bytes are in flight per CU, and keeps the transcendental cost at one v_exp_f32 and one v_rcp_f32
// per element (the reciprocal-multiply form of the paper's Fig. 5b; the plain divide of Fig. 5a
// expands to a long IEEE division sequence).
#pragma once

#include "device_common.h"

namespace astra {

// SiLU(x) = x * 1/(1 + e^-x).  LIBM = false (every kernel of the library): e^-x as one hardware 2^(-x log2 e) and the
// reciprocal as one hardware v_rcp_f32.  x << 0: 2^(+big) = inf, 1/inf = 0, x * 0 = -0, the limit value.
// LIBM = true (ablation entry point only): the same expression with the library expf and an IEEE-rounded divide,
// the costlier pair that the paper's Fig. 5 measures against the fast one.
template <bool LIBM>
__device__ __forceinline__ float silu_form(float x)
{
    const float e = LIBM ? expf(-x) : __builtin_amdgcn_exp2f(x * -kLog2e);
    const float inv = LIBM ? 1.0f / (1.0f + e) : fast_rcp(1.0f + e);
    return x * inv;
}

__device__ __forceinline__ float silu_fast(float x) { return silu_form<false>(x); }

// Fast path: d % N == 0 and 16-byte aligned pointers.  Work is the flat list of output vectors
// (dv = d/N per row); a block owns BLOCK*UNROLL consecutive ones.  For output vector (t, j):
//   x = in[t*2dv + j], g = in[t*2dv + dv + j], out index = t*dv + j.
// LANE_DIV = false (rows of at least 32 vectors): the row of the block's first vector comes from one scalar
// fast division; lanes then step to the next row when they run past the end of a row (a few steps at most).
// LANE_DIV = true (short rows, e.g. a tensor-parallel slice of a small expert): every lane divides for itself.
template <int DT, int UNROLL, bool NTL, bool NTS, bool LIBM = false, int BLOCK = 256, bool LANE_DIV = false>
__global__ __launch_bounds__(BLOCK) void silu_and_mul_vec_kernel(u32x4* __restrict__ out, const u32x4* __restrict__ in,
                                                               uint32_t total_vecs, uint32_t dv, FastDiv by_dv,
                                                               int log2_chunk)
{
    constexpr int N = Storage<DT>::kN;
    constexpr uint32_t kSpan = uint32_t(BLOCK) * UNROLL;
    const uint32_t first = xcd_chunked(blockIdx.x, log2_chunk) * kSpan;
    if (first >= total_vecs) return;  // grid padding
    uint32_t t0 = 0, j0 = 0;
    if constexpr (!LANE_DIV) {
        t0 = by_dv.div(first);
        j0 = first - t0 * dv;
    }

    u32x4 xv[UNROLL], gv[UNROLL];
    uint32_t oidx[UNROLL];
#pragma unroll
    for (int k = 0; k < UNROLL; ++k) {
        const uint32_t off = threadIdx.x + uint32_t(BLOCK) * k;
        oidx[k] = first + off;
        uint32_t t, j;
        if constexpr (LANE_DIV) {
            t = by_dv.div(oidx[k]);
            j = oidx[k] - t * dv;
        } else {
            t = t0;
            j = j0 + off;
            while (j >= dv) {
                j -= dv;
                ++t;
            }
        }
        if (oidx[k] < total_vecs) {
            const u32x4* px = in + (t * 2u * dv + j);  // the host keeps 2*T*dv within 32 bits
            xv[k] = load_vec<NTL>(px);
            gv[k] = load_vec<NTL>(px + dv);
        }
    }
#pragma unroll
    for (int k = 0; k < UNROLL; ++k) {
        if (oidx[k] < total_vecs) {
            float x[N], g[N], o[N];
            unpack_vec<DT>(xv[k], x);
            unpack_vec<DT>(gv[k], g);
#pragma unroll
            for (int e = 0; e < N; ++e) o[e] = silu_form<LIBM>(x[e]) * g[e];
            store_vec<NTS>(out + oidx[k], pack_vec<DT>(o));
        }
    }
}

// Small problems (fewer than 2^15 output vectors, about 1.5 MiB moved: decode-sized launches, bound by launch latency
// and one memory round trip).  Two differences from the streaming kernel, both measured on MI355X by HIP-graph replay
// on the paper's Table 4 shapes, cold: plain (cached) accesses instead of non-temporal ones -- the kernel ends as soon
// as its stores are in the L2, 0.10-0.17 us sooner -- and 8 bytes per lane, which spreads the work over twice as many
// lanes and compute units (T=32 d=5120: 1.97 us against 2.08 with 16 bytes per lane, 2.14 non-temporal; T=16
// d=12288: 1.98 / 2.09 / 2.15).  From 2^15 vectors on non-temporal wins again (T=64 d=8192: 2.29 against 2.47).
// Work is the flat list of half vectors, dh = 2 * d / N per row; every lane divides for itself.
template <int DT>
__global__ __launch_bounds__(256) void silu_and_mul_small_kernel(u32x2* __restrict__ out, const u32x2* __restrict__ in,
                                                                 uint32_t total_halves, uint32_t dh, FastDiv by_dh)
{
    constexpr int M = Storage<DT>::kN / 2;
    const uint32_t o = blockIdx.x * 256u + threadIdx.x;
    if (o >= total_halves) return;
    const uint32_t t = by_dh.div(o), j = o - t * dh;
    const u32x2* px = in + (t * 2u * dh + j);  // below 2^17 half vectors in all
    const u32x2 xv = px[0], gv = px[dh];
    float x[M], g[M], r[M];
    unpack_half_vec<DT>(xv, x);
    unpack_half_vec<DT>(gv, g);
#pragma unroll
    for (int e = 0; e < M; ++e) r[e] = silu_fast(x[e]) * g[e];
    out[o] = pack_half_vec<DT>(r);
}

// Phased path: dense tensors, any d >= N (the host sends rows of eight vectors or more) and any element-aligned pointers.  The work is the list of 16-byte aligned
// chunks of memory the OUTPUT covers: lane c owns flat output elements [c*N - phase, c*N - phase + N), `phase` = the
// output pointer's offset into the 16-byte grid in elements, and stores them with one aligned 16-byte access.  Its
// operands are loaded with 16-byte accesses at element alignment: on MI355X it is the unaligned STORE that costs (the
// ragged kernel below, which also stores at element alignment, runs at 0.91-0.95 of the fast path's rate on odd d;
// this kernel at 0.98-0.99: T=16384, bf16, d=11009 78.2 -> 83.3 % of the HBM peak, d=11012 80.3 -> 84.1 %, d=14337
// 78.9 -> 84.7 %, d=11008 behind offset pointers 73.1 -> 81.3 %; aligned loads measured the same as unaligned ones).
// All but one chunk per row lie inside one row (two loads, one store).  The chunk across the end of row t holds the
// last k elements of row t and the first N - k of row t + 1 (d >= N: never a third row); its operands sit in three
// 16-byte pieces of the input, because what follows x's row t in memory is g's row t, and so on:
//     A1 at x[t] + d - k:   x[t, d-k..d) | g[t, 0..N-k)
//     A2 at g[t] + d - k:   g[t, d-k..d) | x[t+1, 0..N-k)
//     A3 at x[t+1] + d - k: x[t+1, d-k..d) | g[t+1, 0..N-k)
// so positions i < k are SiLU(A1[i]) * A2[i] and positions i >= k are SiLU(A2[i]) * A3[i]: one load more, still one
// aligned store.  The first and the last chunk of the whole output (positions outside the tensor) go element by
// element, so nothing outside either tensor is read or written.
template <int DT, bool NTL, bool NTS, int BLOCK>
__global__ __launch_bounds__(BLOCK) void silu_and_mul_phased_kernel(typename Storage<DT>::elem_t* out,
                                                                    const typename Storage<DT>::elem_t* __restrict__ in,
                                                                    uint32_t T, uint32_t d, FastDiv by_d,
                                                                    uint32_t total_chunks, int phase, int log2_chunk)
{
    typedef typename Storage<DT>::elem_t E;
    constexpr int N = Storage<DT>::kN;
    const uint32_t c = xcd_chunked(blockIdx.x, log2_chunk) * uint32_t(BLOCK) + threadIdx.x;
    if (c >= total_chunks) return;
    const int64_t f0 = (int64_t)c * N - phase;  // first flat output element of the chunk; negative only for chunk 0
    // t: the row of the chunk's first position (-1: before the tensor); k: how many positions that row still holds
    int64_t t = -1;
    int64_t k = phase;
    if (f0 >= 0) {
        t = by_d.div((uint32_t)f0);
        k = (t + 1) * (int64_t)d - f0;
    }
    float x[N], g[N], o[N];
    if (k >= N) {  // inside row t
        const E* px = in + (t * 2 * (int64_t)d + (d - k));
        const u32x4 xv = load_vec_elem_aligned<DT, NTL>(px);
        const u32x4 gv = load_vec_elem_aligned<DT, NTL>(px + d);
        unpack_vec<DT>(xv, x);
        unpack_vec<DT>(gv, g);
#pragma unroll
        for (int e = 0; e < N; ++e) o[e] = silu_fast(x[e]) * g[e];
        store_vec<NTS>(reinterpret_cast<u32x4*>(out + f0), pack_vec<DT>(o));
        return;
    }
    if (t < 0 || t + 1 >= (int64_t)T) {
        // the first or the last chunk of the output: some of its positions lie outside the tensor (rows -1 and T do
        // not exist), so these two lanes of the grid go element by element
#pragma unroll
        for (int e = 0; e < N; ++e) {
            const int64_t f = f0 + e;
            if (f >= 0 && f < (int64_t)T * d) {
                const int64_t row = e < k ? t : t + 1, col = e < k ? (int64_t)d - k + e : e - k;
                const E* pr = in + row * 2 * (int64_t)d;
                out[f] = Storage<DT>::narrow(silu_fast(Storage<DT>::widen(pr[col])) * Storage<DT>::widen(pr[d + col]));
            }
        }
        return;
    }
    // across the end of row t
    const E* a2 = in + ((t + 1) * 2 * (int64_t)d - k);
    const u32x4 v1 = load_vec_elem_aligned<DT, NTL>(a2 - d);
    const u32x4 v2 = load_vec_elem_aligned<DT, NTL>(a2);
    const u32x4 v3 = load_vec_elem_aligned<DT, NTL>(a2 + d);
    float m[N];
    unpack_vec<DT>(v1, x);
    unpack_vec<DT>(v2, m);
    unpack_vec<DT>(v3, g);
#pragma unroll
    for (int e = 0; e < N; ++e) o[e] = e < k ? silu_fast(x[e]) * m[e] : silu_fast(m[e]) * g[e];
    store_vec<NTS>(reinterpret_cast<u32x4*>(out + f0), pack_vec<DT>(o));
}

// Ragged path (rows shorter than eight vectors, row-strided views, tensors beyond the phased kernel's 32-bit element index):
// any d, pointers and row strides only element aligned (dense tensors: out_stride = d, in_stride = 2d).
// A row is dv = ceil(d/N) vectors, the last one possibly partial; one lane per vector, row and column from a
// per-lane fast division, 64-bit element offsets.  Full vectors are 16-byte accesses at element alignment; the
// partial one reads the whole vector that ends at the row end and stores its own elements one by one.
template <int DT, bool NTL, bool NTS>
__global__ __launch_bounds__(256) void silu_and_mul_ragged_kernel(typename Storage<DT>::elem_t* __restrict__ out,
                                                                  int64_t out_stride,
                                                                  const typename Storage<DT>::elem_t* __restrict__ in,
                                                                  int64_t in_stride, uint32_t total_vecs, uint32_t dv,
                                                                  int64_t d, FastDiv by_dv)
{
    constexpr int N = Storage<DT>::kN;
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i >= total_vecs) return;
    const uint32_t t = by_dv.div(i), j = i - t * dv;
    const int64_t e0 = (int64_t)j * N;
    const int count = d - e0 < N ? (int)(d - e0) : N;
    const typename Storage<DT>::elem_t* xrow = in + (int64_t)t * in_stride;  // the gate row follows d elements later
    float x[N], g[N], o[N];
    const int shift = load_row_elems<DT, NTL>(xrow, d, e0, count, x);
    load_row_elems<DT, NTL>(xrow + d, d, e0, count, g);
#pragma unroll
    for (int e = 0; e < N; ++e) o[e] = silu_fast(x[e]) * g[e];  // positions outside [shift, shift + count) are not stored
    store_row_elems<DT, NTS>(out + (int64_t)t * out_stride, e0, count, shift, o);
}

// Element-wise path (inputs too large for the ragged kernel's 32-bit vector index): one block walks one row at a time.
template <int DT>
__global__ __launch_bounds__(256) void silu_and_mul_generic_kernel(typename Storage<DT>::elem_t* __restrict__ out,
                                                                   const typename Storage<DT>::elem_t* __restrict__ in,
                                                                   int64_t T, int64_t d)
{
    typedef typename Storage<DT>::elem_t E;
    for (int64_t t = blockIdx.x; t < T; t += gridDim.x) {
        const E* row = in + t * 2 * d;
        E* orow = out + t * d;
        for (int64_t j = threadIdx.x; j < d; j += blockDim.x) {
            float x = Storage<DT>::widen(row[j]);
            float g = Storage<DT>::widen(row[d + j]);
            orow[j] = Storage<DT>::narrow(silu_fast(x) * g);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Row-strided views: input row t starts in_stride vectors (elements for the element-wise kernel) after row
// t-1, likewise the output (views with odd strides or extents take the ragged kernel above).  One lane per output vector, row and column from a per-lane fast division,
// 64-bit offsets (a strided view has no 32-bit bound on its extent).

template <int DT, bool NTL, bool NTS, int BLOCK = 256>
__global__ __launch_bounds__(BLOCK) void silu_and_mul_strided_vec_kernel(u32x4* __restrict__ out, int64_t out_stride,
                                                                       const u32x4* __restrict__ in, int64_t in_stride,
                                                                       uint32_t total_vecs, uint32_t dv, FastDiv by_dv,
                                                                       int log2_chunk)
{
    constexpr int N = Storage<DT>::kN;
    const uint32_t o = xcd_chunked(blockIdx.x, log2_chunk) * uint32_t(BLOCK) + threadIdx.x;
    if (o >= total_vecs) return;
    const uint32_t t = by_dv.div(o);
    const uint32_t j = o - t * dv;
    const u32x4* px = in + ((int64_t)t * in_stride + j);
    const u32x4 xv = load_vec<NTL>(px);
    const u32x4 gv = load_vec<NTL>(px + dv);
    float x[N], g[N], r[N];
    unpack_vec<DT>(xv, x);
    unpack_vec<DT>(gv, g);
#pragma unroll
    for (int e = 0; e < N; ++e) r[e] = silu_fast(x[e]) * g[e];
    store_vec<NTS>(out + ((int64_t)t * out_stride + j), pack_vec<DT>(r));
}

}  // namespace astra
