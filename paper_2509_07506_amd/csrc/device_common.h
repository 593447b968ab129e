// Device-side building blocks shared by the three gfx950 kernels: 16-byte vector access, 16-bit
// storage-type conversion, wave64 and workgroup sum reductions, and the fast transcendental forms.
//
// gfx950 only.  A wavefront is 64 lanes; one lane moves 16 bytes (8 16-bit or 4 binary32 storage
// elements) per access so a wave covers 1 KiB of contiguous memory per instruction.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace astra {

constexpr int kWave = 64;
constexpr int kVecBytes = 16;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

enum : int { kF16 = 0, kBF16 = 1, kF32 = 2 };

// ---------------------------------------------------------------------------------------------
// global memory access.  Activations are touched exactly once, so they are moved with the
// non-temporal hint; small reused tensors (the rmsnorm weight, the scores) use plain loads.

// the unit in which the memory system moves data: a wave's 64 x 16 bytes are eight whole lines when line aligned
constexpr int kLineBytes = 128;

template <bool NT>
__device__ __forceinline__ u32x4 load_vec(const u32x4* p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

template <bool NT>
__device__ __forceinline__ void store_vec(u32x4* p, u32x4 v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// Store of vector `v` of the row that starts at `row` and holds `row_vecs` vectors, for the fused_add_rmsnorm row
// kernel.  `scope` (uniform over the wave) 0, what the library uses: the plain non-temporal store.  The other two
// values exist for the ablation entry point: the same store at device scope (the `sc1` bit of the CDNA3/CDNA4 memory
// instructions), which sends the line on to memory instead of leaving it dirty in the L2 -- 1: for rows that begin
// and end on 128-byte lines only, 2: for every row.  Measured on MI355X (`bench.py --stores`, 12 placements): for an
// in-place update of tensors far larger than the last-level cache device scope is worth between -0.9 and +1.4 %,
// depending on the row length and the run (T*H = 2^28: H=4096 +1.1 to +1.4 %, H=8192 and 2048 0 to +0.5 %, H=5120 -0.6
// to -0.9 %, H=14336 -0.7 to +0.4 %); on cache-sized tensors that are reused launch after launch it COSTS 3-14 %
// (T=4096 H=4096 23.1 against 21.6 us, T=512 H=8192 7.1 against 6.2 us, T=257 H=7168 5.1 against 4.5 us),
// because the data has to go out to memory; and a row that shares its first or last line with the neighbouring row
// loses 15-25 % with it (H=4104 77 -> 60 % of the HBM peak, H=8200 73 -> 59 %).  Stores to lines the kernel has not
// read (silu_and_mul, merge_attn_states_lse) gain nothing either (-0.5 to +0.4 points).  Hence scope 0 everywhere.
// The scope bits are reachable through the buffer form of the store only: `row` must be uniform over the wave (it
// becomes the scalar buffer descriptor, bounds = the row), `v` is the per-lane part.
enum : int { kStoreScopeNone = 0, kStoreScopeWholeLineRows = 1, kStoreScopeAlways = 2 };

template <bool NT>
__device__ __forceinline__ void store_row_vec(u32x4* row, uint32_t row_vecs, uint32_t v, u32x4 value, int scope = kStoreScopeNone)
{
    if constexpr (NT) {
        const bool whole_lines = ((reinterpret_cast<uintptr_t>(row) | (uintptr_t)(row_vecs * 16u)) & (kLineBytes - 1)) == 0;
        if (scope == kStoreScopeAlways || (scope == kStoreScopeWholeLineRows && whole_lines)) {
            constexpr int kNonTemporal = 2, kDeviceScope = 16;  // cache-policy bits of the buffer instructions: nt, sc1
            constexpr int kRawBuffer = 0x00020000;              // descriptor word 3: untyped 32-bit data, no swizzle
            const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(row, 0, row_vecs * 16u, kRawBuffer);
            __builtin_amdgcn_raw_buffer_store_b128(value, rsrc, v * 16u, 0, kNonTemporal | kDeviceScope);
            return;
        }
    }
    store_vec<NT>(row + v, value);
}

// Request pacing of the fused_add_rmsnorm row kernel (a template parameter there, chosen by the host's launch plan;
// the values are those of ASTRA_PACE_* in include/astra_plan.h)
enum : int { kPaceNone = 0, kPaceWeightFirst = 1, kPaceXBeforeR = 2, kPaceStoreGap = 4, kPaceOneResident = 8 };
// kPaceOneResident: the workgroup reserves this much LDS, more than half of a compute unit's 160 KiB, so that a compute
// unit holds one workgroup at a time (the longest rows of two vectors per lane: see the host's launch plan)
constexpr int kOneResidentLdsBytes = 96 << 10;

// Waits until every global load and store this wave has issued so far has completed (s_waitcnt vmcnt(0);
// the LDS / scalar and export counters are left alone).  Used to pace a wave's second store behind its first.
__device__ __forceinline__ void wait_vector_memory() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// ---------------------------------------------------------------------------------------------
// storage types.  kN: elements per 16-byte vector; elem_t: the element as an integer or float word.
// 16-bit types: unpack2 turns one dword holding two values into two floats (exact), pack2 turns two
// floats into one dword, round-to-nearest-even (v_cvt_pk_bf16_f32 / v_cvt_pk_f16_f32).  binary32
// storage needs no conversion at all.

template <int DT>
struct Storage;

template <>
struct Storage<kBF16> {
    static constexpr int kN = 8;
    typedef uint16_t elem_t;
    static __device__ __forceinline__ f32x2 unpack2(uint32_t w)
    {
        f32x2 r;
        r.x = __builtin_bit_cast(float, w << 16);
        r.y = __builtin_bit_cast(float, w & 0xffff0000u);
        return r;
    }
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi)
    {
        f32x2 v = {lo, hi};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    }
    static __device__ __forceinline__ float widen(uint16_t h) { return __builtin_bit_cast(float, (uint32_t)h << 16); }
    static __device__ __forceinline__ uint16_t narrow(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
};

template <>
struct Storage<kF16> {
    static constexpr int kN = 8;
    typedef uint16_t elem_t;
    static __device__ __forceinline__ f32x2 unpack2(uint32_t w)
    {
        return __builtin_convertvector(__builtin_bit_cast(f16x2, w), f32x2);
    }
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi)
    {
        f32x2 v = {lo, hi};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
    }
    static __device__ __forceinline__ float widen(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }
    static __device__ __forceinline__ uint16_t narrow(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }
};

template <>
struct Storage<kF32> {
    static constexpr int kN = 4;
    typedef float elem_t;
    static __device__ __forceinline__ float widen(float f) { return f; }
    static __device__ __forceinline__ float narrow(float f) { return f; }
};

// by-value helpers: the bit cast is applied to a plain scalar, never to a vector-element expression
__device__ __forceinline__ float word_as_float(uint32_t w) { return __builtin_bit_cast(float, w); }
__device__ __forceinline__ uint32_t float_as_word(float f) { return __builtin_bit_cast(uint32_t, f); }

// one 16-byte vector <-> its Storage<DT>::kN values as floats
template <int DT>
__device__ __forceinline__ void unpack_vec(u32x4 v, float (&f)[Storage<DT>::kN])
{
    if constexpr (DT == kF32) {
        f[0] = word_as_float(v.x); f[1] = word_as_float(v.y);
        f[2] = word_as_float(v.z); f[3] = word_as_float(v.w);
    } else {
        f32x2 a = Storage<DT>::unpack2(v.x), b = Storage<DT>::unpack2(v.y);
        f32x2 c = Storage<DT>::unpack2(v.z), d = Storage<DT>::unpack2(v.w);
        f[0] = a.x; f[1] = a.y; f[2] = b.x; f[3] = b.y;
        f[4] = c.x; f[5] = c.y; f[6] = d.x; f[7] = d.y;
    }
}

template <int DT>
__device__ __forceinline__ u32x4 pack_vec(const float (&f)[Storage<DT>::kN])
{
    u32x4 v;
    if constexpr (DT == kF32) {
        v.x = float_as_word(f[0]); v.y = float_as_word(f[1]);
        v.z = float_as_word(f[2]); v.w = float_as_word(f[3]);
    } else {
        v.x = Storage<DT>::pack2(f[0], f[1]);
        v.y = Storage<DT>::pack2(f[2], f[3]);
        v.z = Storage<DT>::pack2(f[4], f[5]);
        v.w = Storage<DT>::pack2(f[6], f[7]);
    }
    return v;
}

// half a vector (8 bytes: 4 16-bit or 2 binary32 elements), for the small-problem kernels
template <int DT>
__device__ __forceinline__ void unpack_half_vec(u32x2 v, float (&f)[Storage<DT>::kN / 2])
{
    if constexpr (DT == kF32) {
        f[0] = word_as_float(v.x); f[1] = word_as_float(v.y);
    } else {
        f32x2 a = Storage<DT>::unpack2(v.x), b = Storage<DT>::unpack2(v.y);
        f[0] = a.x; f[1] = a.y; f[2] = b.x; f[3] = b.y;
    }
}

template <int DT>
__device__ __forceinline__ u32x2 pack_half_vec(const float (&f)[Storage<DT>::kN / 2])
{
    u32x2 v;
    if constexpr (DT == kF32) {
        v.x = float_as_word(f[0]); v.y = float_as_word(f[1]);
    } else {
        v.x = Storage<DT>::pack2(f[0], f[1]);
        v.y = Storage<DT>::pack2(f[2], f[3]);
    }
    return v;
}

// ---------------------------------------------------------------------------------------------
// fast transcendental forms: one hardware op each (v_exp_f32 is 2^x, v_log_f32 is log2), about 1 ulp.

constexpr float kLog2e = 1.44269504088896340736f;
constexpr float kLn2 = 0.69314718055994530942f;

__device__ __forceinline__ float fast_exp(float x) { return __builtin_amdgcn_exp2f(x * kLog2e); }
__device__ __forceinline__ float fast_log(float x) { return __builtin_amdgcn_logf(x) * kLn2; }
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
__device__ __forceinline__ float fast_rsqrt(float x) { return __builtin_amdgcn_rsqf(x); }

// 1/sqrt(x) for every x >= 0.  The hardware op reads a subnormal argument as zero and would return inf; arguments
// below 2^-100 are scaled by 2^64 first and the result by 2^32 (exact powers of two), so a row whose mean square is
// that small (eps = 0 or tiny, |x + r| around 1e-19 or less) still gets a finite scale.  x = 0 gives inf.
__device__ __forceinline__ float rsqrt_full_range(float x)
{
    const bool tiny = x < 0x1p-100f;
    const float r = fast_rsqrt(tiny ? x * 0x1p+64f : x);
    return tiny ? r * 0x1p+32f : r;
}

// ---------------------------------------------------------------------------------------------
// kN elements at element alignment (the "ragged" kernels: row lengths that are no multiple of a vector,
// pointers that are only element aligned).  A 16-byte global access needs no 16-byte alignment on this
// target (code objects for the HSA runtime run with unaligned access mode on, and the compiler itself turns
// a 16-byte copy from a 2-byte-aligned address into one 128-bit instruction), so a full vector is still one
// instruction; measured it streams at 91-95 % of the aligned rate.  The last, partial vector of a row is
// touched element by element and never past `count`.

typedef u32x4 u32x4_align2 __attribute__((aligned(2)));
typedef u32x4 u32x4_align4 __attribute__((aligned(4)));

template <int DT>
struct ElemAlignedVec {
    typedef u32x4_align2 type;
};
template <>
struct ElemAlignedVec<kF32> {
    typedef u32x4_align4 type;
};

// one whole vector at element alignment
template <int DT, bool NT>
__device__ __forceinline__ u32x4 load_vec_elem_aligned(const typename Storage<DT>::elem_t* p)
{
    typedef typename ElemAlignedVec<DT>::type V;
    if constexpr (NT) return __builtin_nontemporal_load(reinterpret_cast<const V*>(p));
    else return *reinterpret_cast<const V*>(p);
}

// Elements [e0, e0 + count) of a row of `len` elements, 1 <= count <= kN, e0 + count <= len, into f.  Returns the
// position `shift` of element e0 in f: element e0 + i sits in f[shift + i]; the other positions of f hold
// other elements of the row (or repeats) and must be ignored.
//   count == kN           one 16-byte access at e0, shift 0;
//   count < kN <= len     (the partial last vector of a row: e0 + count == len) the whole vector that ends at the
//                         row end, one 16-byte access, shift kN - count; the positions before `shift` belong to the
//                         neighbouring lane and are only read;
//   len < kN              element loads with the index clamped into the row (independent of each other, so they go
//                         out together; a guarded load per element would wait for memory count times), shift 0.
template <int DT, bool NT>
__device__ __forceinline__ u32x4 load_row_vec(const typename Storage<DT>::elem_t* row, int64_t len, int64_t e0, int count,
                                              int* shift)
{
    constexpr int N = Storage<DT>::kN;
    if (count == N) {
        *shift = 0;
        return load_vec_elem_aligned<DT, NT>(row + e0);
    }
    if (len >= N) {
        *shift = N - count;
        return load_vec_elem_aligned<DT, NT>(row + (len - N));
    }
    float f[N];
#pragma unroll
    for (int e = 0; e < N; ++e) f[e] = Storage<DT>::widen(row[e0 + (e < count ? e : count - 1)]);
    *shift = 0;
    return pack_vec<DT>(f);  // widening and narrowing again is exact
}

// the same, unpacked
template <int DT, bool NT>
__device__ __forceinline__ int load_row_elems(const typename Storage<DT>::elem_t* row, int64_t len, int64_t e0, int count,
                                              float (&f)[Storage<DT>::kN])
{
    int shift;
    unpack_vec<DT>(load_row_vec<DT, NT>(row, len, e0, count, &shift), f);
    return shift;
}

// row[e0 + i] <- f[shift + i] narrowed for 0 <= i < count; nothing else is written
template <int DT, bool NT>
__device__ __forceinline__ void store_row_elems(typename Storage<DT>::elem_t* row, int64_t e0, int count, int shift,
                                                const float (&f)[Storage<DT>::kN])
{
    constexpr int N = Storage<DT>::kN;
    typedef typename ElemAlignedVec<DT>::type V;
    if (count == N) {
        const u32x4 v = pack_vec<DT>(f);
        if constexpr (NT) __builtin_nontemporal_store(v, reinterpret_cast<V*>(row + e0));
        else *reinterpret_cast<V*>(row + e0) = v;
    } else {
#pragma unroll
        for (int p = 0; p < N; ++p)
            if (p >= shift && p < shift + count) row[e0 + (p - shift)] = Storage<DT>::narrow(f[p]);
    }
}

// A 16-byte aligned chunk of memory that only partly belongs to the row (the "phased" kernels: rows that start off the
// 16-byte grid are cut into the aligned chunks of memory they cover, so every interior access is an aligned 16-byte
// one, and only the chunk at each end of a row is partial).  Chunk positions e0 .. e0 + N - 1 are row elements; e0 may
// be negative and e0 + N may exceed len.  Positions outside [0, len) read as zero and are not written; nothing outside
// the row is touched.  The element loads are independent of each other (clamped index), so they go out together.
template <int DT>
__device__ __forceinline__ u32x4 load_chunk_partial(const typename Storage<DT>::elem_t* row, int64_t len, int64_t e0)
{
    constexpr int N = Storage<DT>::kN;
    float f[N];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int64_t e = e0 + i;
        const int64_t ec = e < 0 ? 0 : (e >= len ? len - 1 : e);
        const float v = Storage<DT>::widen(row[ec]);
        f[i] = (e >= 0 && e < len) ? v : 0.0f;
    }
    return pack_vec<DT>(f);  // widening and narrowing again is exact
}

template <int DT>
__device__ __forceinline__ void store_chunk_partial(typename Storage<DT>::elem_t* row, int64_t len, int64_t e0,
                                                    const float (&f)[Storage<DT>::kN])
{
    constexpr int N = Storage<DT>::kN;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int64_t e = e0 + i;
        if (e >= 0 && e < len) row[e] = Storage<DT>::narrow(f[i]);  // plain stores: the L2 merges them with the neighbouring row's part of the chunk
    }
}

// ---------------------------------------------------------------------------------------------
// index arithmetic

// n / d for a 32-bit n and a fixed divisor d >= 1, as a multiply-high and two shifts (Granlund and
// Montgomery, "Division by invariant integers using multiplication", PLDI 1994, the unsigned
// round-up variant).  Exact for every 32-bit n.  Built on the host, used on the device.
struct FastDiv {
    uint32_t mul;
    uint32_t sh1;
    uint32_t sh2;
    __host__ __device__ __forceinline__ uint32_t div(uint32_t n) const
    {
#if defined(__HIP_DEVICE_COMPILE__)
        uint32_t t = __umulhi(n, mul);
#else
        uint32_t t = (uint32_t)(((uint64_t)n * mul) >> 32);
#endif
        return (t + ((n - t) >> sh1)) >> sh2;
    }
};

inline FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f;
    uint32_t l = 0;
    while (l < 32 && (uint64_t(1) << l) < d) ++l;  // l = ceil(log2 d)
    f.mul = (uint32_t)(((uint64_t(1) << 32) * ((uint64_t(1) << l) - d)) / d + 1);
    f.sh1 = l < 1 ? l : 1;
    f.sh2 = l < 1 ? 0 : l - 1;
    return f;
}

// Workgroups are handed to the chip's 8 XCDs (each with its own L2) round-robin: workgroup b runs on
// XCD b % 8.  With the plain mapping an XCD therefore touches every 8th unit of work.  This remap makes
// the workgroups that one XCD runs back to back cover 2^log2_chunk consecutive units, then the next
// XCD the following 2^log2_chunk, and so on: XCD x first gets units [x*C, (x+1)*C), then
// [(8+x)*C, (8+x+1)*C), ...  It is a permutation of [0, G) whenever G is a multiple of 8*C; the host
// pads the grid to such a G and surplus workgroups exit.  log2_chunk = 0 is the identity.
constexpr int kXcds = 8;
__host__ __device__ __forceinline__ uint32_t xcd_chunked(uint32_t b, int log2_chunk)
{
    const uint32_t q = b >> 3, x = b & 7u;
    const uint32_t c = q >> log2_chunk, j = q & ((1u << log2_chunk) - 1u);
    return (((c << 3) + x) << log2_chunk) + j;
}

// ---------------------------------------------------------------------------------------------
// reductions

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    // all rows, all banks, lanes without a source read 0 (never happens for the permutations used)
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

// Sum over the 64 lanes of a wave; the result is wave-uniform.  Four DPP steps leave every lane of
// a 16-lane row with the row's sum (lane^1, lane^2, mirror within 8, mirror within 16); the four row
// sums are then read through the scalar unit.  The order of additions is fixed, so the result is
// reproducible from run to run.
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_move<0xB1>(v);   // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);   // quad_perm [2,3,0,1]
    v += dpp_move<0x141>(v);  // row_half_mirror
    v += dpp_move<0x140>(v);  // row_mirror
    int iv = __builtin_bit_cast(int, v);
    float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 0));
    float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 16));
    float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 32));
    float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 48));
    return (r0 + r1) + (r2 + r3);
}

// Sum over each aligned group of G = 8, 16 or 32 consecutive lanes; every lane gets its group's sum.  The same DPP
// steps as wave_sum, stopped early; for 32 lanes the two 16-lane row sums are combined through the scalar unit.
template <int G>
__device__ __forceinline__ float group_sum(float v)
{
    static_assert(G == 8 || G == 16 || G == 32, "group of 8, 16 or 32 lanes");
    v += dpp_move<0xB1>(v);   // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);   // quad_perm [2,3,0,1]
    v += dpp_move<0x141>(v);  // row_half_mirror
    if constexpr (G == 8) return v;
    v += dpp_move<0x140>(v);  // row_mirror
    if constexpr (G == 16) return v;
    int iv = __builtin_bit_cast(int, v);
    float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 0));
    float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 16));
    float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 32));
    float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 48));
    return (threadIdx.x & 32u) ? r2 + r3 : r0 + r1;
}

// Sum over a workgroup of `nwaves` full waves (blockDim.x == nwaves * 64, at most 16 waves).  One LDS
// float per wave and one barrier; every lane then adds the partials in the same order.  `lds` must
// hold 16 floats and must not be reused before the next barrier of the caller.
__device__ __forceinline__ float block_sum(float v, float* lds, int nwaves)
{
    float w = wave_sum(v);
    if (nwaves == 1) return w;
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) lds[wave] = w;
    __syncthreads();
    float total = lds[0];
    for (int i = 1; i < nwaves; ++i) total += lds[i];
    return total;
}

// Ablation only: the workgroup sum with the register-level step taken out again, to measure what reducing in
// registers first is worth (the paper's Fig. 3 compares a shared-memory-only reduction with a shuffle-first one).
// Same two levels as block_sum -- per wave, then across waves -- but the per-wave level goes through LDS: every lane
// stores its value and each 64-lane segment is halved six times with a workgroup barrier before every halving; the
// segment sums are then added by every lane in wave order, as in block_sum.  `lds` holds blockDim.x floats
// (blockDim.x a multiple of 64, at most 1024) and is free again on return.
__device__ __forceinline__ float block_sum_lds_only(float v, float* lds, int nwaves)
{
    const uint32_t t = threadIdx.x, lane = t & 63u;
    lds[t] = v;
#pragma unroll
    for (uint32_t width = 32; width >= 1; width >>= 1) {
        __syncthreads();
        if (lane < width) lds[t] += lds[t + width];  // lanes >= width are only read in this step
    }
    __syncthreads();
    float total = lds[0];
    for (int w = 1; w < nwaves; ++w) total += lds[64 * w];
    __syncthreads();  // the next row overwrites lds
    return total;
}

}  // namespace astra
