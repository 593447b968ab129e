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
    if (n <= 0 || m <= 0) return false;
    if ((uintptr_t)n > ~a || (uintptr_t)m > ~b) return true;  // an extent that wraps around the address space is no tensor: refuse it
    return a < b + (uintptr_t)m && b < a + (uintptr_t)n;
}

// How the tensor pointers of a call sit on the 16-byte grid (the `aligned16` argument of the plan functions):
//   kAlignNone   element alignment only, the tensors' offsets into the grid unrelated
//   kAlign16     every pointer (and row stride) a multiple of 16 bytes
//   kAlignPhased the activation tensors congruent modulo 16 bytes (and their row strides congruent modulo a vector):
//                they share one phase in every row, so they can be cut into the same aligned chunks
enum : int { kAlignNone = 0, kAlign16 = 1, kAlignPhased = 2 };

template <class... P>
inline int align_class(const void* first, P... rest)
{
    const uintptr_t ph = reinterpret_cast<uintptr_t>(first) & 15u;
    bool same = true;
    for (const void* p : {static_cast<const void*>(rest)...}) same = same && ((reinterpret_cast<uintptr_t>(p) & 15u) == ph);
    return !same ? kAlignNone : (ph == 0 ? kAlign16 : kAlignPhased);
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

// a launch description; the vector and ragged paths move 16 bytes per lane with the non-temporal hint unless said otherwise
inline astra_launch_info_t launch_info(int path, int block, int vpt, int lc, int64_t grid, int pace, int rows_per_block,
                                       int access_bytes = -1, int non_temporal = -1)
{
    const bool wide = (path == ASTRA_PATH_VECTOR || path == ASTRA_PATH_RAGGED || path == ASTRA_PATH_PHASED);
    astra_launch_info_t li;
    li.path = path;
    li.block = block;
    li.vectors_per_lane = vpt;
    li.log2_xcd_chunk = lc;
    li.grid = grid;
    li.pace = pace;
    li.rows_per_block = rows_per_block;
    li.access_bytes = access_bytes >= 0 ? access_bytes : (wide ? kVecBytes : 0);
    li.non_temporal = non_temporal >= 0 ? non_temporal : (wide ? 1 : 0);
    return li;
}

// calls f with the workgroup width of a flat kernel (64, 128 or 256 lanes) as a compile-time constant
template <class F>
inline void for_flat_block(int block, F&& f)
{
    if (block == 64) f(std::integral_constant<int, 64>{});
    else if (block == 128) f(std::integral_constant<int, 128>{});
    else f(std::integral_constant<int, 256>{});
}

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

// When the waves of the row kernel issue their requests (fused_add_rmsnorm_kernels.h, PACE), streaming grids (three
// rounds of resident workgroups or more; smaller grids further down).  "gap" = output store held until the residual
// store has completed, "x" = x arrived before r is requested, "w,x" = weight, then x, then r one after the other.
// The table below is what `bench.py --pacing` measures (T*H = 2^28 16-bit elements, every pace forced through the
// ablation entry point on the same 12 placements of x and r inside one allocation, one process), in two runs of the
// command: mean microseconds per launch of the default pace in either run, then the mean gain of the chosen pace over
// the default and on how many of the 12 placements it beat the default, again for either run.  The same code moves by
// 1-5 % with the placement alone, so a row length gets a pace of its own only if that pace beat the default on at
// least 23 of the 24 paired placements of the two runs and by at least 1 % on average in each; everything else takes
// the default.  Rows kept (H in 16-bit elements):
//   H =  1024   gap  330.0 / 329.7   w,x  +7.9 (11/12), +6.8 (12/12)
//   H =  1536   gap  338.2 / 338.0   w,x  +8.8 (12/12), +8.1 (12/12)
//   H =  2048   gap  330.3 / 331.0   w,x  +6.9 (11/12), +8.4 (12/12)
//   H =  2560   gap  330.2 / 330.7   x    +8.2 (12/12), +8.3 (12/12)
//   H =  3072   gap  334.5 / 335.1   x    +7.2 (12/12), +7.4 (12/12)
//   H =  8192   gap  329.4 / 330.2   w,x  +5.2 (12/12), +5.9 (12/12)
//   H = 10240   gap  341.9 / 342.4   w,x  +6.0 (12/12), +4.4 (11/12)     two vectors per lane
//   H = 14336   gap  343.9 / 344.6   w,x  +9.5 (12/12), +8.2 (12/12)     two vectors per lane
//   H = 16384   gap  343.9 / 344.8   x    +5.0 (12/12), +4.7 (11/12)     two vectors per lane
// Rows measured and left at the default (best alternative, either run): H = 512 x +4.5 (9/12), +4.6 (10/12); 4096 w,x
// +2.3 (10/12), +3.8 (12/12); 5120 none -0.9, -0.5; 6144 none +0.6 (9/12), +0.3 (8/12); 7168 x +3.5 (11/12), +3.4
// (11/12); 7680 x +2.9 (11/12), +3.3 (11/12); 11008 w,x +1.0 (8/12), +0.9 (8/12); 12288 w,x +1.6 (11/12), +0.7 (6/12);
// 20480 w,x +3.5 (11/12), +2.7 (11/12); 28672 x -0.5, +0.1; 32768 x +5.5 (10/12), +5.2 (11/12).  A forced pace can also
// lose a lot: "w,x" costs 31 us (10 %) at H = 5120, 26 us at H = 28672 and 10 us at H = 6144, "x" 8 us at H = 5120,
// "none" 9 us at H = 4096, which is why there is no blanket rule.  (floor at 8 TB/s: 268 us.)
// Default: "gap" against "none" is 3-9 us better for rows of 1536 to 4096 elements and level elsewhere.  The gap
// lengthens every workgroup's life by one store round trip, which the end of the grid pays once: about a microsecond
// whatever the size (H = 1024: 23.5 against 22.5 at T = 16384, 84.0 against 82.6 at T = 65536), so under kGapMinRounds
// rounds of resident workgroups the default is "none".
constexpr int kGapMinRounds = 32;

// The longest two-vector rows: one workgroup per compute unit at a time (kPaceOneResident).  What a compute unit has
// in flight is resident lanes x vectors per lane x 32 bytes: 64 KiB for every one-vector row (2048 lanes), but up to
// 128 KiB once a row takes two vectors per lane and two workgroups are resident, and the streaming rate is best at 56
// to 80 KiB.  Measured on MI355X (development harness, T = 8192, bf16, cold, two -> one resident workgroup, best pace
// of either): H = 13312 78.6 -> 79.0 % of the HBM peak, 14336 78.6 -> 79.5 %, 15360 77.5 -> 78.4 %, 16384 78.0 ->
// 79.6 %; too little in flight below that (H = 12288 78.7 -> 78.0 %, 10240 79.1 -> 73.6 %).  Through the library
// (`bench.py --pacing`, T*H = 2^28, 12 placements, two runs; the policy's choice against the best forced pace with two
// resident workgroups): H = 14336 331.0 / 331.0 us against "w,x" 333.3 / 335.1, H = 16384 334.3 / 334.6 against "x"
// 338.1 / 338.5, faster on 12 of 12 placements each time.  With one resident workgroup "w,x" is the best pace or level
// with it.  Rows of four vectors per lane (H = 20480, 24576) gain 3-4 % from the same at T = 4096 but nothing at
// T = 13107 (352.5 us against 348.6-350.6 for "w,x" with two resident), so they are left alone.  Hence: two-vector rows
// of 28 KiB or more, from 16 rows per compute unit on (what was measured).
constexpr int64_t kOneResidentMinRowBytes = 28 << 10;
constexpr int64_t kOneResidentMinRowsPerCu = 16;

inline int rmsnorm_stream_pace(int64_t hv, bool long_grid)
{
    // keys are row lengths in 16-byte vectors: H / 8 for the 16-bit storage types the table was measured with
    if (hv == 320 || hv == 384 || hv == 2048) return kPaceXBeforeR;
    if (hv == 128 || hv == 192 || hv == 256 || hv == 1024 || hv == 1280 || hv == 1792) return kPaceWeightFirst | kPaceXBeforeR;
    return long_grid ? kPaceStoreGap : kPaceNone;
}

// Grids of a few rounds.  Time is a staircase in n = ceil(T / 256), the most rows any of the 256 compute units
// gets, and what decides the best variant is how many bytes of x and r one compute unit has requested at once,
// n * (row bytes) * 2 (measured on MI355X for 16 row lengths from 1024 to 16384 16-bit elements, T in steps of
// 5 % of a round, two placements of x and r; microseconds per launch, cold):
//   * under 48 KiB per compute unit nothing is held back (the shortest dependent chain);
//   * from there up to three rounds of resident workgroups, "x" (x arrived before r is requested) is 10-18 %
//     faster where the compute units are just full (T = 1024, H = 4096: 6.6 against 7.7; T = 2048, H = 2048: 6.3
//     against 7.6; T = 768, H = 8192: 10.5 against 11.5) and within +-5 % elsewhere;
//   * rows that no longer fit at once (n above the resident workgroups per compute unit: 64 KiB requested) but
//     stay within 88 KiB per compute unit run 10-17 % faster in half-sized workgroups with two vectors per lane,
//     all resident at once (T = 1280, H = 4096: 7.8 against 9.1; T = 1024, H = 5120: 7.7 against 9.2; T = 1536,
//     H = 3072: 7.0 against 8.4; T = 2560, H = 2048: 7.8 against 8.9); past 88 KiB they are 3-9 % slower.
//     Workgroups of 5 and 10 waves hold one fewer per compute unit than their lane count allows (the step in the
//     measured times comes one row earlier), so H = 2560 and H = 5120 switch one row earlier;
//   * two-vector rows of 20 KiB or more that fill the compute units exactly (n = 2: two 640- to 1024-lane workgroups
//     each) are faster with four vectors per lane in half-sized workgroups, half as many waves with the same bytes
//     requested: T = 512: H = 14336 10.9 against 12.0, H = 12288 9.2 against 10.3, H = 16384 12.9 against 13.2;
//     T = 307: level to 5 %; 18 KiB rows (H = 9216) lose 0-5 % and n = 1 or n = 3 gain nothing, so only there;
//   * from three rounds on, the streaming policy above.
constexpr int kCus = 256;
constexpr int64_t kPaceMinBytesPerCu = 48 << 10;
constexpr int64_t kHalfBlockMaxBytesPerCu = 88 << 10;
constexpr int kStreamingRounds = 3;

inline int resident_row_blocks(int block)
{
    const int by_lanes = 2048 / block;
    return (block == 320 || block == 640) ? by_lanes - 1 : by_lanes;
}

// vectors per lane, lanes and pacing of the row kernel for T rows of hv vectors (row_bytes each)
inline bool rmsnorm_row_policy(int64_t T, int64_t hv, int64_t row_bytes, RowPlan* plan, int* pace)
{
    if (!rmsnorm_row_plan(hv, plan)) return false;
    const int64_t n = (T + kCus - 1) / kCus;
    const int64_t resident = resident_row_blocks(plan->block);
    // n * row_bytes * 2 without overflow: the comparisons only matter below 2^17
    const int64_t per_cu = n > (int64_t(1) << 20) ? std::numeric_limits<int64_t>::max() : n * row_bytes * 2;
    if (per_cu < kPaceMinBytesPerCu) {
        *pace = kPaceNone;
    } else if (plan->vpt == 1 && plan->block >= 2 * kWave && n > resident && per_cu <= kHalfBlockMaxBytesPerCu) {
        plan->vpt = 2;
        plan->block = round_up((int)((hv + 1) / 2), kWave);
        *pace = kPaceXBeforeR;
    } else if (plan->vpt == 2 && hv >= 1280 && n == 2) {
        plan->vpt = 4;
        plan->block = round_up((int)((hv + 3) / 4), kWave);
        *pace = kPaceXBeforeR;
    } else if (n < kStreamingRounds * resident) {
        *pace = kPaceXBeforeR;
    } else if (plan->vpt == 2 && row_bytes >= kOneResidentMinRowBytes && n >= kOneResidentMinRowsPerCu) {
        *pace = kPaceWeightFirst | kPaceXBeforeR | kPaceOneResident;
    } else {
        *pace = rmsnorm_stream_pace(hv, n >= kGapMinRounds * resident);
    }
    return true;
}

// Rows of at most kShortRowVecs vectors share a workgroup (fused_add_rmsnorm_short_row_kernel): lanes per row
constexpr int64_t kShortRowVecs = 32;
inline int short_row_group(int64_t hv) { return hv <= 8 ? 8 : hv <= 16 ? 16 : 32; }

// Rows of whole vectors that are no whole number of 128-byte lines (H * eb % 128 != 0) start in the middle of a line,
// so the waves of the fast kernel straddle nine lines instead of eight; the phased kernel counts its chunks from the
// line start and keeps every wave access on whole lines.  Measured on MI355X, T=16384, bf16, fast -> phased kernel:
// H=2056 75.1 -> 76.2 % of the HBM peak, H=4104 77.7 -> 79.4 %, H=4128 79.1 -> 79.7 %, H=5128 78.0 -> 79.1 %,
// H=8200 73.9 -> 78.3 %, H=8224 76.2 -> 77.5 %, H=11016 73.9 -> 77.5 %; H=1032 71.8 -> 71.3 %, hence the lower limit.
// Streaming grids only (32 rows per compute unit or more): shorter grids keep the fast kernel with its request pacing.
constexpr int64_t kLineGridMinRowBytes = 4096;
constexpr int64_t kLineGridMinRows = 32 * kCus;

// `short_rows`: the caller can launch the short-row kernel (the ablation variants, which restage the row kernel, cannot)
// `line_grid`: dense rows in place, any kernel allowed (the tuned dense operator): rows that are no whole number of
// 128-byte lines go to the phased kernel
inline astra_status_t plan_rmsnorm(int64_t T, int64_t H, int eb, int align, astra_launch_info_t* info,
                                   bool short_rows = true, bool weight16 = true, bool line_grid = false)
{
    // the fast path also needs the weight on the 16-byte grid; the phased path does not
    const bool aligned16 = (align == kAlign16) && weight16;
    const int64_t ne = kVecBytes / eb;  // elements per 16-byte vector
    int64_t n;
    // (the row length is bounded on its own as well: with T == 0 the product says nothing, and H * 4 bytes must not overflow)
    if (T < 0 || H <= 0 || H > std::numeric_limits<int64_t>::max() / 4 || mul_overflows(T, H, &n) ||
        n > std::numeric_limits<int64_t>::max() / 4)
        return ASTRA_ERR_SHAPE;
    *info = launch_info(ASTRA_PATH_NONE, 0, 0, 0, 0, 0, 0);
    if (T == 0) return ASTRA_OK;
    RowPlan rp;
    int pace = kPaceNone;
    const int short_group = short_row_group(H / ne);
    const int64_t short_rows_per_block = 256 / short_group;
    if (short_rows && aligned16 && H % ne == 0 && H / ne <= kShortRowVecs &&
        (T + short_rows_per_block - 1) / short_rows_per_block <= kMaxRowGrid) {
        // Workgroup width as for the flat kernels (a wave streams 4 KiB and needs no other wave: no barrier): single-wave
        // workgroups on streaming grids when the rows fill their lane groups (T*H = 2^28, bf16, 256 -> 64 lanes: H = 64,
        // 128 and 256 alike 81.0 -> 83.4 % of the HBM peak; H = 192 79.6 -> 80.2 %, H = 72, 9 of 16 lanes, 81.1 -> 79.6 %)
        int64_t rows_per_block = short_rows_per_block;
        if (H / ne == short_group && (T + rows_per_block - 1) / rows_per_block >= kFlatChunkMinBlocks &&
            (T + 64 / short_group - 1) / (64 / short_group) <= kMaxRowGrid)
            rows_per_block = 64 / short_group;
        const int block = (int)(rows_per_block * short_group);
        const int64_t blocks = (T + rows_per_block - 1) / rows_per_block;
        const int lc = fit_chunk_log2(blocks, kFlatChunkLog2, kFlatChunkMinBlocks * (256 / block));
        *info = launch_info(ASTRA_PATH_VECTOR, block, 1, lc, pad_grid(blocks, lc), kPaceNone, (int32_t)rows_per_block);
    } else if (line_grid && align == kAlign16 && H % ne == 0 && (H * eb) % kLineBytes != 0 && H * eb >= kLineGridMinRowBytes &&
               T >= kLineGridMinRows && T < kMaxRowGrid && rmsnorm_row_plan((H + kLineBytes / eb - 1 + ne - 1) / ne, &rp)) {
        const int lc = fit_chunk_log2(T, kRowChunkBytesLog2 - floor_log2(H * eb), kRowChunkMinRows);
        *info = launch_info(ASTRA_PATH_PHASED, rp.block, rp.vpt, lc, pad_grid(T, lc), 0, 0);
    } else if (aligned16 && H % ne == 0 && rmsnorm_row_policy(T, H / ne, H * eb, &rp, &pace)) {
        const int64_t rows = T < kMaxRowGrid ? T : kMaxRowGrid;
        const int lc = fit_chunk_log2(rows, kRowChunkBytesLog2 - floor_log2(H * eb), kRowChunkMinRows);
        if (T >= kMaxRowGrid) pace = kPaceNone;  // the row-loop kernel is not paced
        *info = launch_info(ASTRA_PATH_VECTOR, rp.block, rp.vpt, lc, T < kMaxRowGrid ? pad_grid(rows, lc) : rows, pace, 0);
    } else if (align != kAlignNone && H >= ne && rmsnorm_row_plan((H + kLineBytes / eb - 1 + ne - 1) / ne, &rp)) {
        // rows or pointers off the 16-byte grid, but x, r and the outputs in step with each other: lanes own the aligned
        // chunks of memory a row covers, counted from the start of the 128-byte line the row begins in: at most
        // ceil((128 / eb - 1 + H) / N) chunk slots (fused_add_rmsnorm_phased_row_kernel)
        const int64_t rows = T < kMaxRowGrid ? T : kMaxRowGrid;
        const int lc = fit_chunk_log2(rows, kRowChunkBytesLog2 - floor_log2(H * eb), kRowChunkMinRows);
        *info = launch_info(ASTRA_PATH_PHASED, rp.block, rp.vpt, lc, T < kMaxRowGrid ? pad_grid(rows, lc) : rows, 0, 0);
    } else if (H >= ne && rmsnorm_row_plan(H / ne, &rp)) {
        // rows that are no whole number of vectors, or pointers that are only element aligned: the row still lives in
        // registers, with 16-byte accesses at element alignment; lanes for the whole vectors (at least one), the tail
        // rides in the last lane (workgroups walk rows beyond the grid limit)
        const int64_t rows = T < kMaxRowGrid ? T : kMaxRowGrid;
        const int lc = fit_chunk_log2(rows, kRowChunkBytesLog2 - floor_log2(H * eb), kRowChunkMinRows);
        *info = launch_info(ASTRA_PATH_RAGGED, rp.block, rp.vpt, lc, T < kMaxRowGrid ? pad_grid(rows, lc) : rows, 0, 0);
    } else {
        *info = launch_info(ASTRA_PATH_GENERIC, 256, 0, 0, T < kMaxGenericGrid ? T : kMaxGenericGrid, 0, 0);
    }
    return ASTRA_OK;
}

// Lanes per workgroup of the flat kernels (silu_and_mul, merge_attn_states_lse fast paths) for `vecs` output vectors.
// Measured on MI355X by HIP-graph replay, cold, 16 bytes per lane throughout (narrower accesses never won):
//   * streaming grids (4096 or more 256-lane workgroups): single-wave workgroups are 1.5-3 % faster (silu T=4096
//     d=14336: 53.6 against 54.4 us; merge T=4096 32x128: 17.9 against 18.5; T=32768: 128.0 against 129.7) -- a wave
//     slot is handed on as soon as its own wave has finished instead of when all four of a workgroup have;
//   * fewer workgroups than compute units (33 to 255 of 256 lanes): 128 lanes spread the work over twice as many
//     compute units (silu T=16 d=12288: 2.06 against 2.14 us; T=32 d=5120: 2.06 against 2.13);
//   * everything else: 256 lanes (up to 32 workgroups: 1.79 against 1.95 us; 2048 workgroups: 5.9 against 6.1).
// Single-wave workgroups are bounded by the rate at which the chip starts workgroups, 4.7 per ns whatever their width
// (an empty kernel over 524288 workgroups of 64 lanes: 111.5 us; of 256 lanes, a quarter as many: 28.8 us), so a
// kernel that moves less than 1.5 KiB per wave must not use them; the flat kernels move 3 KiB per wave or more.
// Small flat problems (fewer than this many output vectors, about 1.5 MiB moved) use plain cached accesses, and
// silu_and_mul 8 bytes per lane: see silu_and_mul_small_kernel.  merge_attn_states_lse, same measurement: T=1 40x256
// 1.76 us against 2.04 non-temporal, T=16 32x128 1.94 against 2.04, and from T=64 32x128 (2^15 vectors) on 2.25
// non-temporal against 2.51 plain.
constexpr int64_t kSmallFlatVecs = int64_t(1) << 15;

inline int flat_block(int64_t vecs)
{
    const int64_t blocks256 = (vecs + 255) / 256;
    if (blocks256 >= kFlatChunkMinBlocks) return 64;
    if (blocks256 > 32 && blocks256 < kCus) return 128;
    return 256;
}

constexpr int64_t kSiluChunkMinRowVecs = 8;  // shortest rows (in vectors) for the output-chunk kernel of silu_and_mul

// `views`: the call is on row-strided views, whose kernels have no small-problem and no output-chunk form
inline astra_status_t plan_silu(int64_t T, int64_t d, int eb, int align, astra_launch_info_t* info, bool views = false)
{
    const bool aligned16 = (align == kAlign16);
    const int64_t ne = kVecBytes / eb;
    int64_t two_d, n;
    if (T < 0 || d <= 0 || mul_overflows(d, 2, &two_d) || mul_overflows(T, two_d, &n) ||
        n > std::numeric_limits<int64_t>::max() / 4)
        return ASTRA_ERR_SHAPE;
    *info = launch_info(ASTRA_PATH_NONE, 0, 0, 0, 0, 0, 0);
    if (T == 0) return ASTRA_OK;
    const int64_t dv = d / ne;
    // the input holds 2*T*dv vectors and is indexed with 32 bits
    if (aligned16 && d % ne == 0 && 2 * T * dv <= kMaxVecIndex) {  // rows under kSiluLaneDivBelow vectors: per-lane division
        if (!views && T * dv < kSmallFlatVecs) {  // half a vector per lane, plain accesses
            *info = launch_info(ASTRA_PATH_VECTOR, 256, 1, 0, (2 * T * dv + 255) / 256, 0, 0, kVecBytes / 2, 0);
            return ASTRA_OK;
        }
        const int block = flat_block(T * dv);
        const int64_t span = block * kSiluUnroll;
        const int64_t blocks = (T * dv + span - 1) / span;
        const int lc = fit_chunk_log2(blocks, kFlatChunkLog2, kFlatChunkMinBlocks * (256 / block));
        *info = launch_info(ASTRA_PATH_VECTOR, block, kSiluUnroll, lc, pad_grid(blocks, lc), 0, 0);
    } else if (!views && d >= kSiluChunkMinRowVecs * ne && T * d <= kMaxVecIndex) {
        // any other dense call with rows of at least eight vectors: the aligned chunks of memory the output covers, at
        // most one more than ceil(T * d / N) (silu_and_mul_phased_kernel: aligned stores, loads at element
        // alignment); flat output elements are indexed with 32 bits.  Shorter rows have a chunk across a row end (three
        // loads and a divergent branch) every few chunks, and the ragged kernel is faster there (HIP-graph replay, bf16,
        // ragged / chunked: T=1000 d=36 2.4 / 2.8-3.4 us, T=16 d=100 1.9-2.4 / 2.1-2.4, T=1000 d=68 2.5-3.2 / 2.4-3.1,
        // T=1000 d=132 2.8-3.6 / 2.4-3.2, d=260 3.2-3.8 / 2.5-3.2, T=40000 d=68 5.0-7.1 / 4.9-6.5)
        const int64_t chunks = (T * d + ne - 1) / ne + 1;
        const int block = flat_block(chunks);
        const int64_t blocks = (chunks + block - 1) / block;
        const int lc = fit_chunk_log2(blocks, kFlatChunkLog2, kFlatChunkMinBlocks * (256 / block));
        *info = launch_info(ASTRA_PATH_PHASED, block, 1, lc, pad_grid(blocks, lc), 0, 0);
    } else if (T * ((d + ne - 1) / ne) <= kMaxVecIndex) {  // no overflow: T * d is below 2^61
        *info = launch_info(ASTRA_PATH_RAGGED, 256, 1, 0, (T * ((d + ne - 1) / ne) + 255) / 256, 0, 0);
    } else {
        *info = launch_info(ASTRA_PATH_GENERIC, 256, 0, 0, T < kMaxGenericGrid ? T : kMaxGenericGrid, 0, 0);
    }
    return ASTRA_OK;
}

// `views`: the call is on strided views or a K-way merge, whose kernels have no plain-access and no output-chunk form
inline astra_status_t plan_merge(int64_t T, int64_t NH, int64_t D, int eb, int align, astra_launch_info_t* info,
                                 bool views = false)
{
    const bool aligned16 = (align == kAlign16);
    const int64_t ne = kVecBytes / eb;
    int64_t pairs, n;
    if (T < 0 || NH <= 0 || D <= 0 || mul_overflows(T, NH, &pairs) || mul_overflows(pairs, D, &n) ||
        n > std::numeric_limits<int64_t>::max() / 4)
        return ASTRA_ERR_SHAPE;
    *info = launch_info(ASTRA_PATH_NONE, 0, 0, 0, 0, 0, 0);
    if (T == 0) return ASTRA_OK;
    const int64_t dvec = D / ne;
    if (aligned16 && D % ne == 0 && pairs * dvec <= kMaxVecIndex) {
        const int block = flat_block(pairs * dvec);
        const int64_t span = block * kMergeUnroll;
        const int64_t blocks = (pairs * dvec + span - 1) / span;
        const int lc = fit_chunk_log2(blocks, kFlatChunkLog2, kFlatChunkMinBlocks * (256 / block));
        *info = launch_info(ASTRA_PATH_VECTOR, block, kMergeUnroll, lc, pad_grid(blocks, lc), 0, 0, kVecBytes,
                            !views && pairs * dvec < kSmallFlatVecs ? 0 : 1);
    } else if (!views && D >= ne && n < (int64_t(1) << 32)) {
        // head_dim or pointers off the 16-byte grid, dense tensors: one lane per aligned chunk of the flat output, at
        // most one more chunk than whole vectors (merge_attn_states_lse_phased_kernel: aligned stores, loads at
        // element alignment); workgroup width as for the fast kernel (T=16384 32x129, 256 -> 64 lanes: 78.4 -> 81.2 %
        // of the HBM peak, 32x132 80.8 -> 83.1 %, 32x128 one element off the grid 80.6 -> 83.3 %)
        const int64_t chunks = (n + ne - 1) / ne + 1;
        const int block = flat_block(chunks);
        const int64_t blocks = (chunks + block - 1) / block;
        const int lc = fit_chunk_log2(blocks, kFlatChunkLog2, kFlatChunkMinBlocks * (256 / block));
        *info = launch_info(ASTRA_PATH_PHASED, block, 1, lc, pad_grid(blocks, lc), 0, 0);
    } else if (pairs * ((D + ne - 1) / ne) <= kMaxVecIndex) {
        *info = launch_info(ASTRA_PATH_RAGGED, 256, 1, 0, (pairs * ((D + ne - 1) / ne) + 255) / 256, 0, 0);
    } else {
        *info = launch_info(ASTRA_PATH_GENERIC, 256, 0, 0, pairs < kMaxGenericGrid ? pairs : kMaxGenericGrid, 0, 0);
    }
    return ASTRA_OK;
}

}  // namespace astra
