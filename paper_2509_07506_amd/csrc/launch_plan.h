// Host-side dispatch of the astra library: shape x alignment x storage type -> kernel variant and launch
// geometry, and the argument checks every entry point shares.  Plain host arithmetic, no HIP runtime call,
// so all of it can be exercised on a machine without a GPU (include/astra_plan.h exposes the plans).
#pragma once

#include <cstdint>
#include <limits>
#include <type_traits>

#include "astra.h"
#include "astra_plan.h"
#include "device_common.h"

namespace astra {

// ---- tuning constants (measured on MI355X) ------------------------------------------------------
constexpr bool kNTLoad = true;    // non-temporal hint on the once-read activation streams
constexpr bool kNTStore = true;   // and on the once-written outputs
// Vector pairs per lane.  One is fastest on MI355X for every streaming kernel measured: the finest
// interleaving of loads and stores, full occupancy (32 waves per CU) supplies the bytes in flight.
constexpr int kSiluUnroll = 1;
constexpr int kMergeUnroll = 1;
constexpr int kCopyUnroll = 1;
constexpr int64_t kSiluLaneDivBelow = 32;  // silu rows shorter than this many vectors: each lane divides for itself
constexpr int kKwayGroup = 4;     // partitions folded per step of the streaming K-way merge

constexpr int64_t kMaxVecIndex = int64_t(1) << 31;  // 32-bit vector indices with head-room for the tail
constexpr int64_t kMaxGenericGrid = int64_t(1) << 20;
constexpr int64_t kMaxRowGrid = int64_t(1) << 21;  // grid * 1024 work-items stays below 2^32; a multiple of 8 * 2^8

// XCD-aware launch order (device_common.h, xcd_chunked): the workgroups one XCD runs back to back
// cover a contiguous run of memory.  Measured on MI355X the best run is about 256 KiB per stream for
// the row kernel (+3 to +10 % over the plain order) and 256 workgroups (1 MiB of output) for the flat
// streaming kernels (+2 to +4 %).  Small grids keep the plain order (see fit_chunk_log2).
constexpr int kRowChunkBytesLog2 = 18;
constexpr int kFlatChunkLog2 = 8;
constexpr int kMaxChunkLog2 = 8;
constexpr int64_t kRowChunkMinRows = 1024;    // two rounds of resident 1024-lane workgroups
constexpr int64_t kFlatChunkMinBlocks = 4096; // two rounds of resident 256-lane workgroups

inline int fit_chunk_log2(int64_t grid, int target, int64_t min_grid)
{
    // Grids that are resident almost at once gain nothing from the reordering and measured up to 20 % slower
    // with it (256 rows of H=4096: 3.5 us plain, 4.5 us chunked), so they keep the plain order.
    if (grid < min_grid) return 0;
    int lc = target < 0 ? 0 : (target > kMaxChunkLog2 ? kMaxChunkLog2 : target);
    while (lc > 0 && grid < (int64_t(64) << lc)) --lc;  // at least eight chunks per XCD
    return lc;
}

inline int64_t pad_grid(int64_t grid, int log2_chunk)
{
    if (log2_chunk == 0) return grid;  // identity order: nothing to pad
    const int64_t m = int64_t(kXcds) << log2_chunk;
    return (grid + m - 1) / m * m;
}

inline int floor_log2(int64_t v)
{
    int l = 0;
    while ((int64_t(2) << l) <= v) ++l;
    return l;
}

inline bool mul_overflows(int64_t a, int64_t b, int64_t* out) { return __builtin_mul_overflow(a, b, out); }

inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// half-open byte ranges [p, p+n) and [q, q+m)
inline bool overlaps(const void* p, int64_t n, const void* q, int64_t m)
{
    const uintptr_t a = reinterpret_cast<uintptr_t>(p), b = reinterpret_cast<uintptr_t>(q);
    return n > 0 && m > 0 && a < b + (uintptr_t)m && b < a + (uintptr_t)n;
}

inline bool valid_dtype(int dt) { return dt == ASTRA_F16 || dt == ASTRA_BF16 || dt == ASTRA_F32; }

// bytes per storage element; anything that is not binary32 counts as 16-bit so that shape checks, which come
// before the dtype check, are well defined for an invalid dtype too
inline int elem_bytes(int dt) { return dt == ASTRA_F32 ? 4 : 2; }

// calls f with the storage type as a compile-time constant
template <class F>
inline void for_dtype(astra_dtype_t dt, F&& f)
{
    if (dt == ASTRA_BF16) f(std::integral_constant<int, kBF16>{});
    else if (dt == ASTRA_F16) f(std::integral_constant<int, kF16>{});
    else f(std::integral_constant<int, kF32>{});
}


inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

// ---- fused_add_rmsnorm plan -----------------------------------------------------------------------
// The row lives in registers: hv = H/N vectors (N = 16 / element size) spread over `block` lanes, `vpt` per lane.
// Measured on MI355X: the fewest vectors per lane that fit the row in one workgroup are fastest, for few rows
// (one dependent load-reduce-store chain per lane, the row's bytes requested at once) and for many rows (finest
// interleaving of loads and stores): one vector per lane up to 1024 vectors (H <= 8192 in 16 bits; 81-85 % of
// peak), two up to 2048 (78-79 %; four per lane in half-sized workgroups measured 74-75 % there), four up to
// 4096.  The block is the smallest multiple of 64 lanes that covers the row.
struct RowPlan {
    int vpt;
    int block;
};

inline bool rmsnorm_row_plan(int64_t hv, RowPlan* plan)
{
    int vpt;
    if (hv <= 1024) vpt = 1;
    else if (hv <= 2048) vpt = 2;
    else if (hv <= 4096) vpt = 4;
    else return false;
    plan->vpt = vpt;
    plan->block = round_up((int)((hv + vpt - 1) / vpt), kWave);
    return true;
}

// When the waves of the row kernel issue their requests (fused_add_rmsnorm_kernels.h, PACE).  Few rows: nothing is
// held back (the shortest dependent chain).  Streaming grids: measured on MI355X with T*H = 2^28 16-bit elements,
// microseconds per launch averaged over 16 placements of x and r inside one 6 GiB allocation (10 for the two-vector
// rows), worst placement in brackets; "gap" = output store held until the residual store has completed, "x" = x
// arrived before r is requested, "w,x" = weight, then x, then r one after the other:
//                 none        gap         x           w,x
//   H =  2048   342 (362)   328 (346)   326 (337)   323 (339)
//   H =  4096   337 (349)   320 (338)   322 (325)   320 (326)
//   H =  5120   326 (331)   326 (332)   332 (335)   355 (358)
//   H =  6144   329 (334)   329 (334)   332 (339)   340 (346)
//   H =  8192   331 (342)   329 (332)   325 (332)   323 (329)
//   H =   512   324 (335)   324 (341)   320 (326)   322 (330)
//   H =  1024   327 (341)   326 (341)   327 (340)   323 (336)
//   H =  3072   336 (345)   333 (341)   328 (333)   336 (342)
//   H =  7168   329 (331)   330 (332)   328 (331)   329 (332)
//   H = 10240   342 (345)   341 (343)   339 (342)   336 (338)     two vectors per lane
//   H = 11008   342 (345)   342 (345)   344 (347)   336 (340)     two vectors per lane
//   H = 12288   339 (340)   339 (340)   338 (339)   337 (339)     two vectors per lane
//   H = 14336   341 (342)   341 (343)   338 (339)   336 (337)     two vectors per lane
//   H = 16384   347 (353)   346 (351)   338 (341)   345 (350)     two vectors per lane
//   H = 20480   354 (355)   355 (356)   352 (352)   350 (352)     four vectors per lane
//   H = 28672   353 (359)   354 (357)   353 (358)   374 (382)     four vectors per lane
//   H = 32768   360 (372)   356 (365)   346 (355)   360 (365)     four vectors per lane
// (floor at 8 TB/s: 268 us).  "gap" is never far from the best and has no bad case, so it is the default; the other
// two are taken only where they measured at least 1.5 % better: "w,x" for rows of 256, 512 or 1024 vectors (4, 8,
// 16 KiB) and for two-vector rows, "x" for rows of 384, 2048 and 4096 vectors.  Serialising x and r can lose 8 %
// on other row lengths (H = 5120), and waiting for the weight 6 % (H = 28672), so neither is used outside the
// measured cases.
inline int rmsnorm_pace(int64_t T, int64_t hv, int vpt)
{
    if (T < kRowChunkMinRows) return kPaceNone;
    if (hv == 384 || hv == 2048 || hv == 4096) return kPaceXBeforeR;
    if (vpt == 2 || hv == 256 || hv == 512 || hv == 1024) return kPaceWeightFirst | kPaceXBeforeR;
    return kPaceStoreGap;
}

inline astra_status_t plan_rmsnorm(int64_t T, int64_t H, int eb, bool aligned16, astra_launch_info_t* info)
{
    const int64_t ne = kVecBytes / eb;  // elements per 16-byte vector
    int64_t n;
    if (T < 0 || H <= 0 || mul_overflows(T, H, &n) || n > std::numeric_limits<int64_t>::max() / 4) return ASTRA_ERR_SHAPE;
    *info = astra_launch_info_t{ASTRA_PATH_NONE, 0, 0, 0, 0, 0, 0};
    if (T == 0) return ASTRA_OK;
    RowPlan rp;
    if (aligned16 && H % ne == 0 && rmsnorm_row_plan(H / ne, &rp)) {
        const int64_t rows = T < kMaxRowGrid ? T : kMaxRowGrid;
        const int lc = fit_chunk_log2(rows, kRowChunkBytesLog2 - floor_log2(H * eb), kRowChunkMinRows);
        const int pace = T < kMaxRowGrid ? rmsnorm_pace(T, H / ne, rp.vpt) : kPaceNone;  // the row-loop kernel is not paced
        *info = astra_launch_info_t{ASTRA_PATH_VECTOR, rp.block, rp.vpt, lc, T < kMaxRowGrid ? pad_grid(rows, lc) : rows, pace, 0};
    } else {
        *info = astra_launch_info_t{ASTRA_PATH_GENERIC, 256, 0, 0, T < kMaxGenericGrid ? T : kMaxGenericGrid, 0, 0};
    }
    return ASTRA_OK;
}

inline astra_status_t plan_silu(int64_t T, int64_t d, int eb, bool aligned16, astra_launch_info_t* info)
{
    const int64_t ne = kVecBytes / eb;
    int64_t two_d, n;
    if (T < 0 || d <= 0 || mul_overflows(d, 2, &two_d) || mul_overflows(T, two_d, &n) ||
        n > std::numeric_limits<int64_t>::max() / 4)
        return ASTRA_ERR_SHAPE;
    *info = astra_launch_info_t{ASTRA_PATH_NONE, 0, 0, 0, 0, 0, 0};
    if (T == 0) return ASTRA_OK;
    const int64_t dv = d / ne;
    // the input holds 2*T*dv vectors and is indexed with 32 bits
    if (aligned16 && d % ne == 0 && 2 * T * dv <= kMaxVecIndex) {  // rows under kSiluLaneDivBelow vectors: per-lane division
        const int64_t span = 256 * kSiluUnroll;
        const int64_t blocks = (T * dv + span - 1) / span;
        const int lc = fit_chunk_log2(blocks, kFlatChunkLog2, kFlatChunkMinBlocks);
        *info = astra_launch_info_t{ASTRA_PATH_VECTOR, 256, kSiluUnroll, lc, pad_grid(blocks, lc), 0, 0};
    } else {
        *info = astra_launch_info_t{ASTRA_PATH_GENERIC, 256, 0, 0, T < kMaxGenericGrid ? T : kMaxGenericGrid, 0, 0};
    }
    return ASTRA_OK;
}

inline astra_status_t plan_merge(int64_t T, int64_t NH, int64_t D, int eb, bool aligned16, astra_launch_info_t* info)
{
    const int64_t ne = kVecBytes / eb;
    int64_t pairs, n;
    if (T < 0 || NH <= 0 || D <= 0 || mul_overflows(T, NH, &pairs) || mul_overflows(pairs, D, &n) ||
        n > std::numeric_limits<int64_t>::max() / 4)
        return ASTRA_ERR_SHAPE;
    *info = astra_launch_info_t{ASTRA_PATH_NONE, 0, 0, 0, 0, 0, 0};
    if (T == 0) return ASTRA_OK;
    const int64_t dvec = D / ne;
    if (aligned16 && D % ne == 0 && pairs * dvec <= kMaxVecIndex) {
        const int64_t span = 256 * kMergeUnroll;
        const int64_t blocks = (pairs * dvec + span - 1) / span;
        const int lc = fit_chunk_log2(blocks, kFlatChunkLog2, kFlatChunkMinBlocks);
        *info = astra_launch_info_t{ASTRA_PATH_VECTOR, 256, kMergeUnroll, lc, pad_grid(blocks, lc), 0, 0};
    } else {
        *info = astra_launch_info_t{ASTRA_PATH_GENERIC, 256, 0, 0, pairs < kMaxGenericGrid ? pairs : kMaxGenericGrid, 0, 0};
    }
    return ASTRA_OK;
}

}  // namespace astra
