// merge_attn_states_lse for gfx950 -- paper Table 1, Kernel 1:
//   V_out = (e^Sa V_a + e^Sb V_b) / (e^Sa + e^Sb),  S_out = log(e^Sa + e^Sb).
//
// One lane owns one 16-byte vector (N = 8 16-bit or 4 binary32 elements) of one (token, head) pair.  The
// two mixing weights depend only on the pair, so a lane computes them once for its N elements (the hoisting of the
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

// One element of the blend a*va + b*vb.  A term whose weight is exactly zero is left out and its value not looked
// at: an empty partition (score -inf) has no value vector, so NaN or inf left in its buffer must not reach the
// output, and one empty side returns the other side's value bit for bit.  The sum is one fused multiply-add in
// every kernel, so all paths give the same bits.  The selects cost three v_cndmask per element, far below the
// memory time.
__device__ __forceinline__ float blend(const MergeWeights& w, float va, float vb)
{
    const float pa = w.a * va, pb = w.b * vb;
    const float both = __builtin_fmaf(w.a, va, pb);
    return w.a == 0.0f ? (w.b == 0.0f ? 0.0f : pb) : (w.b == 0.0f ? pa : both);
}

// The same for one 16-byte vector of each side, with fewer instructions: the weighted sum is formed for all N
// elements (one multiply and one fused multiply-add each), then the packed result is replaced as a whole when a
// weight is zero -- by the other side's vector unchanged (its weight is then exactly 1: e^0 / (1 + 0)), or by zero
// when both weights are zero.  Equal to blend() element by element for every finite live value.
template <int DT>
__device__ __forceinline__ u32x4 blend_vec(const MergeWeights& w, u32x4 av, u32x4 bv)
{
    constexpr int N = Storage<DT>::kN;
    float a[N], b[N], o[N];
    unpack_vec<DT>(av, a);
    unpack_vec<DT>(bv, b);
#pragma unroll
    for (int e = 0; e < N; ++e) o[e] = __builtin_fmaf(w.a, a[e], w.b * b[e]);
    u32x4 r = pack_vec<DT>(o);
    const bool a0 = (w.a == 0.0f), b0 = (w.b == 0.0f);
    const u32x4 other = a0 ? bv : av;
    r = (a0 != b0) ? other : r;
    r = (a0 && b0) ? u32x4{0u, 0u, 0u, 0u} : r;
    return r;
}

// Fast path: head_dim % N == 0, 16-byte aligned v pointers.  Flat list of vectors, dvec = head_dim/N
// per pair.  The pair index is a shift when dvec is a power of two (LOG2_DVEC >= 0), otherwise a
// multiply-high division.  v_out may alias v_a or v_b exactly: all loads of a lane precede its stores.
// lse_out must not alias the input scores: the lanes of one pair can sit in different waves.
template <int DT, int UNROLL, bool NTL, bool NTS, bool HOIST = true, int BLOCK = 256>
__global__ __launch_bounds__(BLOCK) void merge_attn_states_lse_vec_kernel(u32x4* v_out, float* lse_out, const u32x4* v_a,
                                                                        const float* lse_a, const u32x4* v_b,
                                                                        const float* lse_b, uint32_t total_vecs,
                                                                        uint32_t dvec, int log2_dvec, FastDiv by_dvec,
                                                                        int log2_chunk)
{
    constexpr int N = Storage<DT>::kN;
    const uint32_t first = xcd_chunked(blockIdx.x, log2_chunk) * (uint32_t(BLOCK) * UNROLL) + threadIdx.x;
    u32x4 av[UNROLL], bv[UNROLL];
    float sa[UNROLL], sb[UNROLL];
    uint32_t pair[UNROLL];
#pragma unroll
    for (int k = 0; k < UNROLL; ++k) {
        const uint32_t i = first + uint32_t(BLOCK) * k;
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
        const uint32_t i = first + uint32_t(BLOCK) * k;
        if (i < total_vecs) {
            const MergeWeights w = merge_weights(sa[k], sb[k]);
            if constexpr (HOIST) {
                store_vec<NTS>(v_out + i, blend_vec<DT>(w, av[k], bv[k]));
            } else {
                float a[N], b[N], o[N];
                unpack_vec<DT>(av[k], a);
                unpack_vec<DT>(bv[k], b);
                // ablation only (the pattern of the paper's Fig. 2a): the weights are worked out again for
                // every element.  The empty asm makes the score opaque so the compiler cannot merge the
                // N evaluations back into one.
#pragma unroll
                for (int e = 0; e < N; ++e) {
                    float s = sa[k];
                    asm volatile("" : "+v"(s));
                    const MergeWeights we = merge_weights(s, sb[k]);
                    o[e] = blend(we, a[e], b[e]);
                }
                store_vec<NTS>(v_out + i, pack_vec<DT>(o));
            }
            if (i == pair[k] * dvec) lse_out[pair[k]] = w.lse;  // first vector of the pair
        }
    }
}

// Strides of the value tensors of a strided call: element (t, h, k) lives at t*token + h*head + k
struct ValueStrides {
    int64_t out_token, out_head, a_token, a_head, b_token, b_head;
};

// Ragged path: any head_dim, value pointers (and, STRIDED, token and head strides) only element aligned.  A pair is
// dvec = ceil(D/N) vectors, the last one possibly partial; one lane per vector, pair and position from a per-lane
// fast division, 64-bit element offsets.  Full vectors are 16-byte accesses at element alignment; the partial one
// reads the whole vector that ends at the end of the pair and stores its own elements one by one.  v_out may alias
// v_a or v_b exactly (a lane loads before it stores; what it reads of its neighbour's elements it ignores).  STRIDED = false: dense [pairs, D] tensors, `vs`, `by_heads` and `heads` are not looked at.
template <int DT, bool NTL, bool NTS, bool STRIDED = false>
__global__ __launch_bounds__(256) void merge_attn_states_lse_ragged_kernel(
    typename Storage<DT>::elem_t* v_out, float* lse_out, const typename Storage<DT>::elem_t* v_a, const float* lse_a,
    const typename Storage<DT>::elem_t* v_b, const float* lse_b, uint32_t total_vecs, uint32_t dvec, int64_t D,
    FastDiv by_dvec, ValueStrides vs = ValueStrides{0, 0, 0, 0, 0, 0}, FastDiv by_heads = FastDiv{0, 0, 0}, uint32_t heads = 1)
{
    constexpr int N = Storage<DT>::kN;
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i >= total_vecs) return;
    const uint32_t pair = by_dvec.div(i), jv = i - pair * dvec;
    const int64_t e0 = (int64_t)jv * N;
    const int count = D - e0 < N ? (int)(D - e0) : N;
    int64_t oa, ob, oo;  // where the pair's head_dim elements start
    if constexpr (STRIDED) {
        const uint32_t t = by_heads.div(pair), h = pair - t * heads;
        oa = (int64_t)t * vs.a_token + (int64_t)h * vs.a_head;
        ob = (int64_t)t * vs.b_token + (int64_t)h * vs.b_head;
        oo = (int64_t)t * vs.out_token + (int64_t)h * vs.out_head;
    } else {
        oa = ob = oo = (int64_t)pair * D;
    }
    float a[N], b[N], o[N];
    const int shift = load_row_elems<DT, NTL>(v_a + oa, D, e0, count, a);
    load_row_elems<DT, NTL>(v_b + ob, D, e0, count, b);
    const MergeWeights w = merge_weights(lse_a[pair], lse_b[pair]);
#pragma unroll
    for (int e = 0; e < N; ++e) o[e] = blend(w, a[e], b[e]);  // positions outside [shift, shift + count) are not stored
    store_row_elems<DT, NTS>(v_out + oo, e0, count, shift, o);
    if (jv == 0) lse_out[pair] = w.lse;
}

// Phased path: head_dim no whole number of vectors, or pointers offset by some elements; dense tensors, head_dim >= N.
// The work is the list of 16-byte aligned chunks of memory the OUTPUT covers: lane c owns flat elements
// [c*N - phase, c*N - phase + N), `phase` = v_out's offset into the 16-byte grid in elements, and stores them with one
// aligned 16-byte access; v_a and v_b are loaded with 16-byte accesses at element alignment (aligned ones whenever the
// inputs are in step with the output, as all 16-byte aligned tensors are).  It is the unaligned store that costs on
// MI355X: a kernel that also stores at element alignment, like the ragged one above, runs 25-30 % below the fast path,
// unaligned loads measure the same as aligned ones.  Only the first and the last chunk of the whole tensor can be
// partial (element by element; nothing outside a tensor is read or written).  A chunk can straddle the end of a
// (token, head) pair -- at most one, since head_dim >= N -- so a lane evaluates the weights of the pair of its first
// and of its last element and takes, per element, those of the pair the element belongs to; the lane that holds a
// pair's first element stores that pair's S_out.
template <int DT, bool NTL, bool NTS, int BLOCK = 256>
__global__ __launch_bounds__(BLOCK) void merge_attn_states_lse_phased_kernel(
    typename Storage<DT>::elem_t* v_out, float* lse_out, const typename Storage<DT>::elem_t* v_a, const float* lse_a,
    const typename Storage<DT>::elem_t* v_b, const float* lse_b, uint32_t n_elems, uint32_t D, FastDiv by_D,
    uint32_t total_chunks, int phase, int log2_chunk)
{
    constexpr int N = Storage<DT>::kN;
    const uint32_t c = xcd_chunked(blockIdx.x, log2_chunk) * uint32_t(BLOCK) + threadIdx.x;
    if (c >= total_chunks) return;
    const int64_t e0 = (int64_t)c * N - phase;  // first flat element of the chunk; negative only for chunk 0
    const bool whole = e0 >= 0 && e0 + N <= (int64_t)n_elems;
    const uint32_t first = e0 < 0 ? 0u : (uint32_t)e0;
    const uint32_t last = e0 + N <= (int64_t)n_elems ? (uint32_t)(e0 + N - 1) : n_elems - 1u;
    const uint32_t p0 = by_D.div(first), p1 = by_D.div(last);
    u32x4 av, bv;
    if (whole) {  // (aligned whenever the input is in step with the output)
        av = load_vec_elem_aligned<DT, NTL>(v_a + e0);
        bv = load_vec_elem_aligned<DT, NTL>(v_b + e0);
    } else {
        av = load_chunk_partial<DT>(v_a, n_elems, e0);
        bv = load_chunk_partial<DT>(v_b, n_elems, e0);
    }
    const MergeWeights w0 = merge_weights(lse_a[p0], lse_b[p0]);
    const MergeWeights w1 = merge_weights(lse_a[p1], lse_b[p1]);
    const int64_t turn = (int64_t)(p0 + 1u) * D - e0;  // chunk positions from `turn` on belong to pair p1
    float a[N], b[N], o[N];
    unpack_vec<DT>(av, a);
    unpack_vec<DT>(bv, b);
#pragma unroll
    for (int i = 0; i < N; ++i) o[i] = blend(i < turn ? w0 : w1, a[i], b[i]);
    if (whole) store_vec<NTS>(reinterpret_cast<u32x4*>(v_out + e0), pack_vec<DT>(o));
    else store_chunk_partial<DT>(v_out, n_elems, e0, o);
    if (first == p0 * D) lse_out[p0] = w0.lse;  // the chunk holds the first element of pair p0 ...
    if (p1 != p0) lse_out[p1] = w1.lse;         // ... and that of p1 whenever it reaches into p1
}

// Element-wise path (inputs too large for the ragged kernel's 32-bit vector index): one block per (token, head) pair.
template <int DT>
__global__ __launch_bounds__(256) void merge_attn_states_lse_generic_kernel(typename Storage<DT>::elem_t* v_out, float* lse_out,
                                                                            const typename Storage<DT>::elem_t* v_a,
                                                                            const float* lse_a,
                                                                            const typename Storage<DT>::elem_t* v_b,
                                                                            const float* lse_b, int64_t pairs, int64_t D)
{
    for (int64_t p = blockIdx.x; p < pairs; p += gridDim.x) {
        const MergeWeights w = merge_weights(lse_a[p], lse_b[p]);
        for (int64_t k = threadIdx.x; k < D; k += blockDim.x) {
            float a = Storage<DT>::widen(v_a[p * D + k]);
            float b = Storage<DT>::widen(v_b[p * D + k]);
            v_out[p * D + k] = Storage<DT>::narrow(blend(w, a, b));
        }
        if (threadIdx.x == 0) lse_out[p] = w.lse;
    }
}

// ---------------------------------------------------------------------------------------------
// Strided views of the value tensors: element (t, h, k) of a tensor lives at t*token_stride + h*head_stride + k
// (strides in vectors for the fast kernel, in elements for the ragged and the element-wise one); the scores stay dense [T, NH].
// One lane per output vector; pair, token and head from per-lane fast divisions; 64-bit offsets.

template <int DT, bool NTL, bool NTS, int BLOCK = 256>
__global__ __launch_bounds__(BLOCK) void merge_attn_states_lse_strided_vec_kernel(u32x4* v_out, float* lse_out, const u32x4* v_a,
                                                                                const float* lse_a, const u32x4* v_b,
                                                                                const float* lse_b, ValueStrides vs,
                                                                                uint32_t total_vecs, uint32_t dvec,
                                                                                FastDiv by_dvec, FastDiv by_heads,
                                                                                uint32_t heads, int log2_chunk)
{
    const uint32_t i = xcd_chunked(blockIdx.x, log2_chunk) * uint32_t(BLOCK) + threadIdx.x;
    if (i >= total_vecs) return;
    const uint32_t pair = by_dvec.div(i), jv = i - pair * dvec;
    const uint32_t t = by_heads.div(pair), h = pair - t * heads;
    const u32x4 av = load_vec<NTL>(v_a + ((int64_t)t * vs.a_token + (int64_t)h * vs.a_head + jv));
    const u32x4 bv = load_vec<NTL>(v_b + ((int64_t)t * vs.b_token + (int64_t)h * vs.b_head + jv));
    const MergeWeights w = merge_weights(lse_a[pair], lse_b[pair]);
    store_vec<NTS>(v_out + ((int64_t)t * vs.out_token + (int64_t)h * vs.out_head + jv), blend_vec<DT>(w, av, bv));
    if (jv == 0) lse_out[pair] = w.lse;
}

// ---------------------------------------------------------------------------------------------
// K-way merge: V_out = sum_k e^(S_k) V_k / sum_k e^(S_k), S_out = log sum_k e^(S_k).

// Fast path: one lane per output vector; part k of vector i lives at v_parts[k * total_vecs + i].
// Streaming form: the parts are taken in groups of G.  All G scores and G vectors of a group are
// requested together (one wait per group; loads return in order, so a score load issued after a
// vector load cannot be consumed earlier anyway), then folded into a running maximum m, a running
// denominator and running accumulators that are rescaled by e^(m_old - m_new) whenever the maximum
// grows.  Equal to the definition up to binary32 rounding; a three-pass form (maximum, denominator,
// weights) measured 10-14 % slower because every pass waits on memory again.
template <int DT, int G, bool NTL, bool NTS, int BLOCK = 256>
__global__ __launch_bounds__(BLOCK) void merge_attn_states_lse_kway_vec_kernel(u32x4* __restrict__ v_out,
                                                                             float* __restrict__ lse_out,
                                                                             const u32x4* __restrict__ v_parts,
                                                                             const float* __restrict__ lse_parts,
                                                                             uint32_t K, uint32_t total_vecs, uint32_t pairs,
                                                                             uint32_t dvec, int log2_dvec, FastDiv by_dvec,
                                                                             int log2_chunk)
{
    constexpr int N = Storage<DT>::kN;
    const uint32_t i = xcd_chunked(blockIdx.x, log2_chunk) * uint32_t(BLOCK) + threadIdx.x;
    if (i >= total_vecs) return;
    const uint32_t pair = log2_dvec >= 0 ? (i >> log2_dvec) : by_dvec.div(i);
    const float ninf = -__builtin_inff();
    float m = ninf, den = 0.0f;
    float acc[N];
#pragma unroll
    for (int e = 0; e < N; ++e) acc[e] = 0.0f;
    for (uint32_t k0 = 0; k0 < K; k0 += G) {
        u32x4 pv[G];
        float s[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const uint32_t k = k0 + g;
            if (k < K) {
                pv[g] = load_vec<NTL>(v_parts + ((size_t)k * total_vecs + i));
                s[g] = lse_parts[(size_t)k * pairs + pair];
            } else {
                pv[g] = u32x4{0u, 0u, 0u, 0u};
                s[g] = ninf;
            }
        }
        float gm = s[0];
#pragma unroll
        for (int g = 1; g < G; ++g) gm = fmaxf(gm, s[g]);
        const float mn = fmaxf(m, gm);
        if (mn != ninf) {  // otherwise every partition so far is empty: nothing to add
            const float rescale = fast_exp(m - mn);  // first live group: m = -inf, e^-inf = 0, sums are 0 anyway
            den *= rescale;
#pragma unroll
            for (int e = 0; e < N; ++e) acc[e] *= rescale;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float w = fast_exp(s[g] - mn);
                den += w;
                float v[N];
                // a part with weight zero (an empty partition) is not looked at: its vector is read as zeros
                unpack_vec<DT>(w == 0.0f ? u32x4{0u, 0u, 0u, 0u} : pv[g], v);
#pragma unroll
                for (int e = 0; e < N; ++e) acc[e] = __builtin_fmaf(w, v[e], acc[e]);
            }
            m = mn;
        }
    }
    const bool empty = (m == ninf);
    const float inv = empty ? 0.0f : fast_rcp(den);
#pragma unroll
    for (int e = 0; e < N; ++e) acc[e] *= inv;
    store_vec<NTS>(v_out + i, pack_vec<DT>(acc));
    if (i == pair * dvec) lse_out[pair] = empty ? ninf : m + fast_log(den);
}

// Ragged path of the K-way merge: any head_dim, value pointers only element aligned.  The streaming form above with
// dvec = ceil(D/N) vectors per pair; a partial last vector is read as the whole vector that ends at the end of the
// pair (the same positions for every part) and only its own elements are stored.
template <int DT, int G, bool NTL, bool NTS>
__global__ __launch_bounds__(256) void merge_attn_states_lse_kway_ragged_kernel(
    typename Storage<DT>::elem_t* __restrict__ v_out, float* __restrict__ lse_out,
    const typename Storage<DT>::elem_t* __restrict__ v_parts, const float* __restrict__ lse_parts, uint32_t K,
    uint32_t total_vecs, int64_t pairs, uint32_t dvec, int64_t D, FastDiv by_dvec)
{
    constexpr int N = Storage<DT>::kN;
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i >= total_vecs) return;
    const uint32_t pair = by_dvec.div(i), jv = i - pair * dvec;
    const int64_t e0 = (int64_t)jv * N;
    const int count = D - e0 < N ? (int)(D - e0) : N;
    const float ninf = -__builtin_inff();
    float m = ninf, den = 0.0f;
    float acc[N];
#pragma unroll
    for (int e = 0; e < N; ++e) acc[e] = 0.0f;
    int shift = 0;
    for (uint32_t k0 = 0; k0 < K; k0 += G) {
        u32x4 pv[G];
        float s[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const uint32_t k = k0 + g;
            if (k < K) {
                pv[g] = load_row_vec<DT, NTL>(v_parts + ((int64_t)k * pairs + pair) * D, D, e0, count, &shift);
                s[g] = lse_parts[(int64_t)k * pairs + pair];
            } else {
                pv[g] = u32x4{0u, 0u, 0u, 0u};
                s[g] = ninf;
            }
        }
        float gm = s[0];
#pragma unroll
        for (int g = 1; g < G; ++g) gm = fmaxf(gm, s[g]);
        const float mn = fmaxf(m, gm);
        if (mn != ninf) {
            const float rescale = fast_exp(m - mn);
            den *= rescale;
#pragma unroll
            for (int e = 0; e < N; ++e) acc[e] *= rescale;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float w = fast_exp(s[g] - mn);
                den += w;
                float v[N];
                // a part with weight zero (an empty partition) is not looked at: its vector is read as zeros
                unpack_vec<DT>(w == 0.0f ? u32x4{0u, 0u, 0u, 0u} : pv[g], v);
#pragma unroll
                for (int e = 0; e < N; ++e) acc[e] = __builtin_fmaf(w, v[e], acc[e]);
            }
            m = mn;
        }
    }
    const bool empty = (m == ninf);
    const float inv = empty ? 0.0f : fast_rcp(den);
#pragma unroll
    for (int e = 0; e < N; ++e) acc[e] *= inv;
    store_row_elems<DT, NTS>(v_out + (int64_t)pair * D, e0, count, shift, acc);
    if (jv == 0) lse_out[pair] = empty ? ninf : m + fast_log(den);
}

}  // namespace astra
