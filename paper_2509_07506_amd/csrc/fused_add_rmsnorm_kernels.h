// fused_add_rmsnorm for gfx950 -- paper Table 1, Kernel 2:
//   y = (x + r) / sqrt(||x + r||^2 / H + eps) (.) w,  input <- y, residual <- x + r (both in place).
//
// One pass over HBM: a workgroup holds a whole row of binary32 sums in registers (VPT vectors of N = 8
// 16-bit or 4 binary32 elements per lane), so x and r are read once and each written once.  The sum of
// squares is reduced inside each wave with DPP (registers only) and across waves through one LDS float
// per wave and a single barrier -- the register-first reduction of the paper's Fig. 3b, on 64-lane waves.
#pragma once

#include "device_common.h"

namespace astra {

// Fast path: H % N == 0, 16-byte aligned pointers, hv = H/N <= VPT * blockDim.x (VPT is 1, 2 or 4).
// blockDim.x is a multiple of 64 and at most MAX_THREADS.  Lane `tid` owns vectors tid + k*blockDim.x.
//
// ROW_LOOP = false: one row per workgroup, row = xcd_chunked(blockIdx.x) (the grid covers all rows).
// ROW_LOOP = true:  a workgroup walks rows r0, r0 + gridDim.x, ... (only for more rows than the grid limit).
// They are separate instantiations so that the common single-row form carries no loop bookkeeping.
//
// PACE selects when a wave issues its memory requests.  The arithmetic is the same for every value; what changes
// is how the requests of the thousands of resident waves interleave at the memory controllers, which is worth
// 1-4 % of the streaming rate on MI355X (table in the host's launch plan).  Bits (device_common.h):
//   kPaceWeightFirst  the weight must have arrived before the activations are requested
//   kPaceXBeforeR     the x vectors must have arrived before the r vectors are requested
//   kPaceStoreGap     the residual store must have completed before the output store is issued
//   kPaceOneResident  not a wait: the workgroup reserves 96 KiB of LDS it never touches, so that a compute unit holds
//                     one workgroup at a time.  Two resident workgroups of a two-vector row keep 2048 lanes x 2 x 32
//                     bytes = 128 KiB of loads in flight per compute unit, twice what the one-vector rows do, and
//                     the streaming rate is best at 56 to 80 KiB (T=8192, bf16, two -> one resident workgroup:
//                     H=16384 78.0 -> 79.6 % of the HBM peak, H=14336 78.6 -> 79.5 %; H=10240, whose rows are
//                     20 KiB, 79.1 -> 73.6 %)
// With PACE = 0 every request goes out as early as possible: the shortest dependent chain, used for few rows.
// Both results go out through store_row_vec (device_common.h): the plain non-temporal store; `store_scope` lets the
// ablation entry point run the same kernel with device-scope stores.
// The empty asm statements (`arrive`) consume the loaded registers at a chosen point, which fixes where the wait
// for that load is placed; no instruction is emitted for them.  All loads are consumed before the arithmetic
// starts, so the compiler has no reason to add a wait of its own later on.
template <int VPT>
__device__ __forceinline__ void arrive(u32x4 (&v)[VPT])
{
#pragma unroll
    for (int k = 0; k < VPT; ++k) asm volatile("" : "+v"(v[k]));
}

// STRIDED = false: dense in-place operator; `input` and `residual` are read and overwritten, `views`, `y_out` and
// `r_out` are not looked at.  STRIDED = true: rows of x (= `input`), r (= `residual`), y_out and r_out start
// views.*_stride vectors apart and the results go to y_out / r_out (which may be the input views themselves).
struct RowViews {
    int64_t y_stride, r_out_stride, x_stride, r_stride;
};

template <int DT, int VPT, int MAX_THREADS, bool NTL, bool NTS, bool LDS_TREE = false, bool ROW_LOOP = false,
          int PACE = kPaceNone, bool STRIDED = false>
__global__ __launch_bounds__(MAX_THREADS) void fused_add_rmsnorm_row_kernel(u32x4* input, u32x4* residual,
                                                                            const u32x4* __restrict__ weight,
                                                                            int64_t T, uint32_t hv, float inv_h, float eps,
                                                                            int log2_chunk, u32x4* y_out = nullptr,
                                                                            u32x4* r_out = nullptr,
                                                                            RowViews views = RowViews{0, 0, 0, 0},
                                                                            int store_scope = kStoreScopeNone)
{
    constexpr int N = Storage<DT>::kN;
    __shared__ float partials[2][16];
    __shared__ float tree[LDS_TREE ? 1024 : 1];  // ablation only
    if constexpr ((PACE & kPaceOneResident) != 0) {
        __shared__ char reserved[kOneResidentLdsBytes];  // never accessed; its address is consumed so that it is allocated
        asm volatile("" : : "v"((uint32_t)(uintptr_t)&reserved[0]));
    }
    const int nwaves = blockDim.x >> 6;
    const int64_t first_row = xcd_chunked(blockIdx.x, log2_chunk);
    if (first_row >= T) return;  // grid padding; uniform for the whole workgroup
    int parity = 0;

    // the weight does not depend on the row: requested first (L2 resident, shared by all blocks), used last
    u32x4 wv[VPT];
#pragma unroll
    for (int k = 0; k < VPT; ++k) {
        const uint32_t v = threadIdx.x + k * blockDim.x;
        wv[k] = u32x4{0u, 0u, 0u, 0u};
        if (v < hv) wv[k] = weight[v];
    }
    if constexpr ((PACE & kPaceWeightFirst) != 0) arrive<VPT>(wv);

    int64_t row = first_row;
    do {
        const u32x4* xrow = input + row * (STRIDED ? views.x_stride : (int64_t)hv);
        const u32x4* rrow = residual + row * (STRIDED ? views.r_stride : (int64_t)hv);
        u32x4* yrow = STRIDED ? y_out + row * views.y_stride : input + row * hv;
        u32x4* sumrow = STRIDED ? r_out + row * views.r_out_stride : residual + row * hv;
        u32x4 xv[VPT], rv[VPT];
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            const uint32_t v = threadIdx.x + k * blockDim.x;
            xv[k] = u32x4{0u, 0u, 0u, 0u};
            if (v < hv) xv[k] = load_vec<NTL>(xrow + v);
        }
        if constexpr ((PACE & kPaceXBeforeR) != 0) arrive<VPT>(xv);
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            const uint32_t v = threadIdx.x + k * blockDim.x;
            rv[k] = u32x4{0u, 0u, 0u, 0u};
            if (v < hv) rv[k] = load_vec<NTL>(rrow + v);
        }
        // everything requested so far is consumed here, so the only later wait is the optional store gap
        arrive<VPT>(xv);
        arrive<VPT>(rv);
        arrive<VPT>(wv);

        float s[VPT][N];
        float acc = 0.0f;
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            const uint32_t v = threadIdx.x + k * blockDim.x;
            if (v < hv) {
                float x[N], r[N];
                unpack_vec<DT>(xv[k], x);
                unpack_vec<DT>(rv[k], r);
#pragma unroll
                for (int e = 0; e < N; ++e) {
                    s[k][e] = x[e] + r[e];
                    acc += s[k][e] * s[k][e];
                }
                store_row_vec<NTS>(sumrow, hv, v, pack_vec<DT>(s[k]), store_scope);
            }
        }

        const float total = LDS_TREE ? block_sum_lds_only(acc, tree, nwaves) : block_sum(acc, partials[parity], nwaves);
        const float scale = rsqrt_full_range(total * inv_h + eps);
        if constexpr ((PACE & kPaceStoreGap) != 0) wait_vector_memory();

#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            const uint32_t v = threadIdx.x + k * blockDim.x;
            if (v < hv) {
                float w[N], y[N];
                unpack_vec<DT>(wv[k], w);
#pragma unroll
                for (int e = 0; e < N; ++e) y[e] = (s[k][e] * scale) * w[e];
                store_row_vec<NTS>(yrow, hv, v, pack_vec<DT>(y), store_scope);
            }
        }
        row += gridDim.x;
        parity ^= 1;
    } while (ROW_LOOP && row < T);
}

// Short rows (at most 32 vectors: H <= 256 in 16 bits): one row per workgroup would leave most of a wave idle, so a
// row takes G = 8, 16 or 32 lanes (the smallest that holds it) and a workgroup of BLOCK lanes BLOCK/G rows; the sum of
// squares stays inside the wave (group_sum: no LDS, no barrier).  Measured on MI355X with T*H = 2^28: H = 64
// 3040 -> 6507 GB/s, H = 128 4659 -> 6409, H = 256 6365 -> 6415 against one row per 64-lane workgroup.
// STRIDED as in the row kernel.
template <int DT, int G, bool NTL, bool NTS, bool STRIDED = false, int BLOCK = 256>
__global__ __launch_bounds__(BLOCK) void fused_add_rmsnorm_short_row_kernel(u32x4* input, u32x4* residual,
                                                                          const u32x4* __restrict__ weight, int64_t T,
                                                                          uint32_t hv, float inv_h, float eps, int log2_chunk,
                                                                          u32x4* y_out = nullptr, u32x4* r_out = nullptr,
                                                                          RowViews views = RowViews{0, 0, 0, 0})
{
    constexpr int N = Storage<DT>::kN;
    constexpr uint32_t kRows = BLOCK / G;  // rows per workgroup
    const int64_t row = (int64_t)xcd_chunked(blockIdx.x, log2_chunk) * kRows + threadIdx.x / G;
    const uint32_t v = threadIdx.x % G;
    const bool live = row < T && v < hv;  // whole waves stay together: group_sum needs every lane
    u32x4 wv = u32x4{0u, 0u, 0u, 0u}, xv = wv, rv = wv;
    const int64_t xo = row * (STRIDED ? views.x_stride : (int64_t)hv) + v;
    const int64_t ro = row * (STRIDED ? views.r_stride : (int64_t)hv) + v;
    if (live) {
        wv = weight[v];
        xv = load_vec<NTL>(input + xo);
        rv = load_vec<NTL>(residual + ro);
    }
    float x[N], r[N], s[N];
    unpack_vec<DT>(xv, x);
    unpack_vec<DT>(rv, r);
    float acc = 0.0f;
#pragma unroll
    for (int e = 0; e < N; ++e) {
        s[e] = x[e] + r[e];
        acc += s[e] * s[e];
    }
    if (live) store_vec<NTS>(STRIDED ? r_out + (row * views.r_out_stride + v) : residual + ro, pack_vec<DT>(s));
    const float total = group_sum<G>(acc);
    const float scale = rsqrt_full_range(total * inv_h + eps);
    float w[N], y[N];
    unpack_vec<DT>(wv, w);
#pragma unroll
    for (int e = 0; e < N; ++e) y[e] = (s[e] * scale) * w[e];
    if (live) store_vec<NTS>(STRIDED ? y_out + (row * views.y_stride + v) : input + xo, pack_vec<DT>(y));
}

// ---------------------------------------------------------------------------------------------
// Phased path: rows that do not start on the 16-byte grid (H no whole number of vectors, so the phase changes from row
// to row, or pointers offset by some elements), with x, r, y_out and r_out all at the SAME phase in every row (the
// host checks: pointers congruent modulo 16 bytes, row strides congruent modulo a vector -- true for every dense in
// place call on 16-byte aligned tensors).  A row is cut into the 16-byte aligned chunks of memory it covers, counted
// from the start of the 128-byte line the row begins in: lane c owns chunk c of that line-aligned run, i.e. row elements
// [c*N - phase, c*N - phase + N) with phase = elements between the line start and the row start (up to 128 bytes' worth;
// the chunks before the row stay idle), and moves it with aligned 16-byte accesses exactly like the fast path.  Counting
// from the line rather than from the row's first chunk keeps every wave's 1 KiB access on whole 128-byte lines, which
// measured 3-7 points of the HBM peak faster for row lengths that are no multiple of the vector (T=16384, bf16:
// H=8196 70.9 -> 78.2 %, H=11012 71.1 -> 78.0 %, H=4100 76.1 -> 79.5 %, H=5124 74.5 -> 77.5 %; the fast path on the
// neighbouring aligned H: 78.7-81.4 %).  The chunk at either end of the row can be partial (it also holds elements of
// the neighbouring row, which another workgroup is updating).
//
// What decides the speed here is the NUMBER of memory instructions a workgroup issues, not their bytes: on MI355X a
// streaming kernel pays about as much for a 2-byte store of one lane as for a 1 KiB store of a whole wave (measured:
// T=16384, H=4096 one element off the grid -- 84 us with the partial chunks left out, 112-131 us with them loaded and
// stored element by element or in 8/4/2-byte pieces, i.e. with 16-40 more instructions per row on top of 45).  So:
//   * a partial chunk is LOADED whole, with the same instruction as every other chunk, and the positions outside the
//     row are cleared in registers (they are bytes of the neighbouring row or, at the ends of a tensor, at most 14
//     bytes outside it -- an aligned 16-byte access lies inside one page, so it cannot fault);
//   * its elements are STORED by the first 16 lanes of the workgroup, one element per lane (lane j < N: position j of
//     the first chunk, lane N + j: position j of the last chunk), so that the whole boundary costs one element-wide
//     store instruction per output and one element-wide weight load: the two owner lanes hand the unrounded sums to
//     those lanes through LDS (written before the reduction's barrier, read after it).
// That is 3 memory instructions per row more than the fast path.  The weight is indexed by row position, so its
// 16-byte loads are at element alignment (it is cache resident).  One workgroup per row in the XCD-aware order;
// ROW_LOOP as in the row kernel; VPT chunks per lane; VPT * blockDim.x >= the most chunk slots a row can need,
// ceil((128 / sizeof(element) - 1 + H) / N).
template <int DT, int VPT, bool NTL, bool NTS, bool ROW_LOOP = false>
__global__ __launch_bounds__(1024) void fused_add_rmsnorm_phased_row_kernel(
    typename Storage<DT>::elem_t* y_out, typename Storage<DT>::elem_t* r_out, const typename Storage<DT>::elem_t* x,
    const typename Storage<DT>::elem_t* r, const typename Storage<DT>::elem_t* __restrict__ weight, RowViews sv, int64_t T,
    int64_t H, float inv_h, float eps, int log2_chunk)
{
    typedef typename Storage<DT>::elem_t E;
    constexpr int N = Storage<DT>::kN;
    __shared__ float partials[2][16];
    __shared__ float edge[2][2 * N];  // unrounded sums of the first chunk [0, N) and of the last chunk [N, 2N)
    const int nwaves = blockDim.x >> 6;
    int parity = 0;
    const int64_t first_row = xcd_chunked(blockIdx.x, log2_chunk);
    if (first_row >= T) return;  // grid padding; uniform for the whole workgroup
    const int len = (int)H;      // at most 4096 vectors

    int64_t row = first_row;
    do {
        const E* xr = x + row * sv.x_stride;
        const E* rr = r + row * sv.r_stride;
        E* yr = y_out + row * sv.y_stride;
        E* sr = r_out + row * sv.r_out_stride;
        // elements from the start of the enclosing 128-byte line to the row start; modulo N the same for rr, yr, sr
        const int phase = (int)((reinterpret_cast<uintptr_t>(xr) & (kLineBytes - 1)) / sizeof(E));
        const int first = phase / N;                  // index of the row's first chunk; uniform
        const int last = (phase + len - 1) / N;       // index of the row's last chunk; uniform
        const bool head_cut = phase % N != 0, tail_cut = (phase + len) % N != 0;

        // the boundary elements' weights, one per lane of the first 16 (requested first, like the weight vectors)
        const int j = (int)threadIdx.x;
        const int edge_e = (j < N ? first * N + j : last * N + (j - N)) - phase;  // row element of this lane's boundary position
        const bool edge_lane = j < 2 * N && edge_e >= 0 && edge_e < len && (j < N ? head_cut : tail_cut);  // H >= N: the two chunks differ
        float edge_w = 0.0f;
        if (edge_lane) edge_w = Storage<DT>::widen(weight[edge_e]);

        u32x4 xa[VPT], ra[VPT], wa[VPT];
        int e0[VPT];
        bool whole[VPT], cut[VPT];
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            const int c = (int)(threadIdx.x + k * blockDim.x);
            e0[k] = c * N - phase;  // first row element of the chunk (negative for chunk 0 when phase > 0)
            whole[k] = e0[k] >= 0 && e0[k] + N <= len;
            cut[k] = !whole[k] && c >= first && c <= last;
            wa[k] = u32x4{0u, 0u, 0u, 0u};
            if (whole[k]) wa[k] = load_vec_elem_aligned<DT, false>(weight + e0[k]);
        }
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            xa[k] = ra[k] = u32x4{0u, 0u, 0u, 0u};
            if (whole[k] || cut[k]) {  // one aligned access, also for a partial chunk
                xa[k] = load_vec<NTL>(reinterpret_cast<const u32x4*>(xr + e0[k]));
                ra[k] = load_vec<NTL>(reinterpret_cast<const u32x4*>(rr + e0[k]));
            }
        }

        float s[VPT][N];
        float acc = 0.0f;
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            float a[N], b[N];
            unpack_vec<DT>(xa[k], a);
            unpack_vec<DT>(ra[k], b);
            if (cut[k]) {  // clear the positions that belong to the neighbouring row
#pragma unroll
                for (int e = 0; e < N; ++e) {
                    const bool mine = e0[k] + e >= 0 && e0[k] + e < len;
                    a[e] = mine ? a[e] : 0.0f;
                    b[e] = mine ? b[e] : 0.0f;
                }
            }
#pragma unroll
            for (int e = 0; e < N; ++e) {
                s[k][e] = a[e] + b[e];
                acc += s[k][e] * s[k][e];
            }
            if (whole[k]) store_vec<NTS>(reinterpret_cast<u32x4*>(sr + e0[k]), pack_vec<DT>(s[k]));
            if (cut[k]) {
                float* slot = edge[parity] + (e0[k] < 0 ? 0 : N);  // first chunk, or last chunk
#pragma unroll
                for (int e = 0; e < N; ++e) slot[e] = s[k][e];
            }
        }
        const float total = block_sum(acc, partials[parity], nwaves);
        if (nwaves == 1) __syncthreads();  // block_sum has no barrier of its own then; the boundary sums pass through LDS
        const float scale = rsqrt_full_range(total * inv_h + eps);
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            if (whole[k]) {
                float w[N], y[N];
                unpack_vec<DT>(wa[k], w);
#pragma unroll
                for (int e = 0; e < N; ++e) y[e] = (s[k][e] * scale) * w[e];
                store_vec<NTS>(reinterpret_cast<u32x4*>(yr + e0[k]), pack_vec<DT>(y));
            }
        }
        if (edge_lane) {  // the boundary elements, one per lane: a single store instruction per output
            const float se = edge[parity][j];
            sr[edge_e] = Storage<DT>::narrow(se);
            yr[edge_e] = Storage<DT>::narrow((se * scale) * edge_w);
        }
        row += gridDim.x;
        parity ^= 1;
    } while (ROW_LOOP && row < T);
}

// ---------------------------------------------------------------------------------------------
// Ragged path: any H of 1 to 4096 whole vectors plus (TAIL) a tail of fewer than N elements, pointers and row strides
// only element aligned; in place (y_out = x, r_out = r, strides H) or out of place.  One workgroup per row in the
// XCD-aware order, rows gridDim.x apart, the whole vectors in registers as in the row kernel above, as 16-byte
// accesses at element alignment.  The tail rides in the workgroup's last lane (which has the fewest vectors, so it
// costs no extra wave) as the whole vector that ends at the row end, of which only the last `tail` positions are
// summed and stored; every request of a row is issued before the first is used.  A lane loads
// its elements of x and r before it stores to the same positions, so exact aliasing of an output with an input is
// safe.  `sv` holds the row strides in elements.
template <int DT, int VPT, bool TAIL, bool NTL, bool NTS>
__global__ __launch_bounds__(1024) void fused_add_rmsnorm_ragged_row_kernel(
    typename Storage<DT>::elem_t* y_out, typename Storage<DT>::elem_t* r_out, const typename Storage<DT>::elem_t* x,
    const typename Storage<DT>::elem_t* r, const typename Storage<DT>::elem_t* __restrict__ weight, RowViews sv, int64_t T,
    int64_t H, float inv_h, float eps, int log2_chunk)
{
    constexpr int N = Storage<DT>::kN;
    __shared__ float partials[2][16];
    const int nwaves = blockDim.x >> 6;
    int parity = 0;
    const int64_t first_row = xcd_chunked(blockIdx.x, log2_chunk);
    if (first_row >= T) return;  // grid padding; uniform for the whole workgroup
    const uint32_t whole = (uint32_t)(H / N);  // whole vectors per row
    const uint32_t tail0 = whole * N;          // first element of the tail
    const int tail = TAIL && threadIdx.x == blockDim.x - 1 ? (int)(H - tail0) : 0;  // tail elements this lane handles

    u32x4 wv[VPT], wt = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
    for (int k = 0; k < VPT; ++k) {
        const uint32_t v = threadIdx.x + k * blockDim.x;
        wv[k] = u32x4{0u, 0u, 0u, 0u};
        if (v < whole) wv[k] = load_vec_elem_aligned<DT, false>(weight + v * N);
    }
    if (TAIL && tail > 0) wt = load_vec_elem_aligned<DT, false>(weight + (H - N));  // the vector that ends at the row end

    for (int64_t row = first_row; row < T; row += gridDim.x, parity ^= 1) {
        const typename Storage<DT>::elem_t* xr = x + row * sv.x_stride;
        const typename Storage<DT>::elem_t* rr = r + row * sv.r_stride;
        typename Storage<DT>::elem_t* yr = y_out + row * sv.y_stride;
        typename Storage<DT>::elem_t* sr = r_out + row * sv.r_out_stride;
        u32x4 xa[VPT], ra[VPT], xt = u32x4{0u, 0u, 0u, 0u}, rt = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            const uint32_t v = threadIdx.x + k * blockDim.x;
            xa[k] = ra[k] = u32x4{0u, 0u, 0u, 0u};
            if (v < whole) {
                xa[k] = load_vec_elem_aligned<DT, NTL>(xr + v * N);
                ra[k] = load_vec_elem_aligned<DT, NTL>(rr + v * N);
            }
        }
        if (TAIL && tail > 0) {
            xt = load_vec_elem_aligned<DT, NTL>(xr + (H - N));
            rt = load_vec_elem_aligned<DT, NTL>(rr + (H - N));
        }

        float s[VPT][N], st[TAIL ? N : 1];
        float acc = 0.0f;
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            const uint32_t v = threadIdx.x + k * blockDim.x;
            if (v < whole) {
                float a[N], b[N];
                unpack_vec<DT>(xa[k], a);
                unpack_vec<DT>(ra[k], b);
#pragma unroll
                for (int e = 0; e < N; ++e) {
                    s[k][e] = a[e] + b[e];
                    acc += s[k][e] * s[k][e];
                }
                store_row_elems<DT, NTS>(sr, (int64_t)v * N, N, 0, s[k]);
            }
        }
        if constexpr (TAIL) {
            if (tail > 0) {
                float a[N], b[N];
                unpack_vec<DT>(xt, a);
                unpack_vec<DT>(rt, b);
#pragma unroll
                for (int e = 0; e < N; ++e) {
                    st[e] = e >= N - tail ? a[e] + b[e] : 0.0f;  // the other positions belong to the neighbouring lane
                    acc += st[e] * st[e];
                }
                store_row_elems<DT, NTS>(sr, tail0, tail, N - tail, st);
            }
        }
        const float total = block_sum(acc, partials[parity], nwaves);
        const float scale = rsqrt_full_range(total * inv_h + eps);
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            const uint32_t v = threadIdx.x + k * blockDim.x;
            if (v < whole) {
                float w[N], y[N];
                unpack_vec<DT>(wv[k], w);
#pragma unroll
                for (int e = 0; e < N; ++e) y[e] = (s[k][e] * scale) * w[e];
                store_row_elems<DT, NTS>(yr, (int64_t)v * N, N, 0, y);
            }
        }
        if constexpr (TAIL) {
            if (tail > 0) {
                float w[N], y[N];
                unpack_vec<DT>(wt, w);
#pragma unroll
                for (int e = 0; e < N; ++e) y[e] = (st[e] * scale) * w[e];
                store_row_elems<DT, NTS>(yr, tail0, tail, N - tail, y);
            }
        }
    }
}

// Element-wise path (rows of more than 4096 vectors), any H and element-aligned pointers: two passes over the row.  The first pass
// only reads (it needs the unrounded sums, so the residual cannot be written yet); the second
// recomputes x + r, stores it and the normalised value.  Each element is read and written by the
// same lane, so the in-place update is safe.
template <int DT>
__global__ __launch_bounds__(256) void fused_add_rmsnorm_generic_kernel(typename Storage<DT>::elem_t* input,
                                                                        typename Storage<DT>::elem_t* residual,
                                                                        const typename Storage<DT>::elem_t* __restrict__ weight,
                                                                        int64_t T, int64_t H, float inv_h, float eps)
{
    typedef typename Storage<DT>::elem_t E;
    __shared__ float partials[2][16];
    int parity = 0;
    for (int64_t row = blockIdx.x; row < T; row += gridDim.x, parity ^= 1) {
        E* x = input + row * H;
        E* r = residual + row * H;
        float acc = 0.0f;
        for (int64_t j = threadIdx.x; j < H; j += blockDim.x) {
            float s = Storage<DT>::widen(x[j]) + Storage<DT>::widen(r[j]);
            acc += s * s;
        }
        const float total = block_sum(acc, partials[parity], blockDim.x >> 6);
        const float scale = rsqrt_full_range(total * inv_h + eps);
        for (int64_t j = threadIdx.x; j < H; j += blockDim.x) {
            float s = Storage<DT>::widen(x[j]) + Storage<DT>::widen(r[j]);
            r[j] = Storage<DT>::narrow(s);
            x[j] = Storage<DT>::narrow((s * scale) * Storage<DT>::widen(weight[j]));
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Row-strided, out-of-place form, element-wise path (the fast path is the row kernel above with STRIDED = true):
// separate input and output views, each with its own row stride in elements.

template <int DT>
__global__ __launch_bounds__(256) void fused_add_rmsnorm_strided_generic_kernel(
    typename Storage<DT>::elem_t* y_out, typename Storage<DT>::elem_t* r_out, const typename Storage<DT>::elem_t* x,
    const typename Storage<DT>::elem_t* r, const typename Storage<DT>::elem_t* __restrict__ weight, RowViews sv, int64_t T,
    int64_t H, float inv_h, float eps)
{
    typedef typename Storage<DT>::elem_t E;
    __shared__ float partials[2][16];
    int parity = 0;
    for (int64_t row = blockIdx.x; row < T; row += gridDim.x, parity ^= 1) {
        const E* xr = x + row * sv.x_stride;
        const E* rr = r + row * sv.r_stride;
        float acc = 0.0f;
        for (int64_t j = threadIdx.x; j < H; j += blockDim.x) {
            float s = Storage<DT>::widen(xr[j]) + Storage<DT>::widen(rr[j]);
            acc += s * s;
        }
        const float total = block_sum(acc, partials[parity], blockDim.x >> 6);
        const float scale = rsqrt_full_range(total * inv_h + eps);
        for (int64_t j = threadIdx.x; j < H; j += blockDim.x) {
            float s = Storage<DT>::widen(xr[j]) + Storage<DT>::widen(rr[j]);
            r_out[row * sv.r_out_stride + j] = Storage<DT>::narrow(s);
            y_out[row * sv.y_stride + j] = Storage<DT>::narrow((s * scale) * Storage<DT>::widen(weight[j]));
        }
    }
}

}  // namespace astra
