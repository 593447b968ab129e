// C ABI of the astra library: argument validation and the kernel launches; the dispatch (shape x alignment x
// storage type -> kernel variant and launch geometry) is in launch_plan.h.  Everything before the first HIP
// call is plain host arithmetic, so every error path can be exercised without a GPU.
#include "astra.h"
#include "astra_ablation.h"
#include "astra_kway.h"
#include "astra_plan.h"
#include "astra_strided.h"

#include <hip/hip_runtime.h>

#include <cstdint>
#include <limits>
#include <type_traits>

#include "ablation_kernels.h"
#include "fused_add_rmsnorm_kernels.h"
#include "launch_plan.h"
#include "merge_attn_states_lse_kernels.h"
#include "silu_and_mul_kernels.h"
#include "stream_copy_kernel.h"

namespace {

using namespace astra;

astra_status_t after_launch() { return hipGetLastError() == hipSuccess ? ASTRA_OK : ASTRA_ERR_LAUNCH; }

// the `aligned16` argument of the astra_plan_* functions as an alignment class
int plan_align(int aligned16) { return aligned16 == 2 ? kAlignPhased : (aligned16 != 0 ? kAlign16 : kAlignNone); }

// ---- launches ---------------------------------------------------------------------------------------

// Launches the row kernel for one plan.  STRIDED = false: `input` / `residual` are updated in place and `y_out`, `r_out`,
// `views` are ignored; STRIDED = true: x = `input`, r = `residual` are read through `views` (strides in vectors) and
// the results go to y_out / r_out.  The ablation's reduction variant (LDS_TREE) is paced like the tuned kernel, so
// that the two differ in the reduction only.
template <int DT, int VPT, int MAXT, bool LDS_TREE = false, bool STRIDED = false>
void launch_rmsnorm_row(const astra_launch_info_t& li, void* input, void* residual, const void* weight, int64_t T,
                        int64_t H, float eps, hipStream_t stream, void* y_out = nullptr, void* r_out = nullptr,
                        RowViews views = RowViews{0, 0, 0, 0}, int store_scope = kStoreScopeNone)
{
    const uint32_t hv = (uint32_t)(H / Storage<DT>::kN);
    u32x4* const in = static_cast<u32x4*>(input);
    u32x4* const res = static_cast<u32x4*>(residual);
    const u32x4* const w = static_cast<const u32x4*>(weight);
    u32x4* const yo = static_cast<u32x4*>(y_out);
    u32x4* const ro = static_cast<u32x4*>(r_out);
    const dim3 grid((uint32_t)li.grid), block(li.block);
    const float inv_h = 1.0f / (float)H;
    const int lc = li.log2_xcd_chunk;
    if (li.grid < T) {  // more rows than the grid limit: workgroups walk several rows
        fused_add_rmsnorm_row_kernel<DT, VPT, MAXT, kNTLoad, kNTStore, LDS_TREE, true, kPaceNone, STRIDED>
            <<<grid, block, 0, stream>>>(in, res, w, T, hv, inv_h, eps, lc, yo, ro, views, store_scope);
        return;
    }
    switch (li.pace) {
        case kPaceStoreGap:
            fused_add_rmsnorm_row_kernel<DT, VPT, MAXT, kNTLoad, kNTStore, LDS_TREE, false, kPaceStoreGap, STRIDED>
                <<<grid, block, 0, stream>>>(in, res, w, T, hv, inv_h, eps, lc, yo, ro, views, store_scope);
            return;
        case kPaceWeightFirst | kPaceXBeforeR:
            fused_add_rmsnorm_row_kernel<DT, VPT, MAXT, kNTLoad, kNTStore, LDS_TREE, false, kPaceWeightFirst | kPaceXBeforeR, STRIDED>
                <<<grid, block, 0, stream>>>(in, res, w, T, hv, inv_h, eps, lc, yo, ro, views, store_scope);
            return;
        case kPaceXBeforeR:
            fused_add_rmsnorm_row_kernel<DT, VPT, MAXT, kNTLoad, kNTStore, LDS_TREE, false, kPaceXBeforeR, STRIDED>
                <<<grid, block, 0, stream>>>(in, res, w, T, hv, inv_h, eps, lc, yo, ro, views, store_scope);
            return;
        // one workgroup per compute unit at a time: planned for rows of two vectors per lane only
        case kPaceWeightFirst | kPaceXBeforeR | kPaceOneResident:
            if constexpr (VPT == 2) {
                fused_add_rmsnorm_row_kernel<DT, VPT, MAXT, kNTLoad, kNTStore, LDS_TREE, false,
                                             kPaceWeightFirst | kPaceXBeforeR | kPaceOneResident, STRIDED>
                    <<<grid, block, 0, stream>>>(in, res, w, T, hv, inv_h, eps, lc, yo, ro, views, store_scope);
                return;
            }
            break;
        default: break;
    }
    fused_add_rmsnorm_row_kernel<DT, VPT, MAXT, kNTLoad, kNTStore, LDS_TREE, false, kPaceNone, STRIDED>
        <<<grid, block, 0, stream>>>(in, res, w, T, hv, inv_h, eps, lc, yo, ro, views, store_scope);
}

// rows of at most 32 vectors, G lanes per row, li.block / G rows per workgroup (li.block is 256, or 64 on streaming
// grids); `views` (strides in vectors) only when STRIDED
template <int DT, bool STRIDED>
void launch_rmsnorm_short(const astra_launch_info_t& li, void* input, void* residual, const void* weight, int64_t T, int64_t H,
                          float eps, hipStream_t stream, void* y_out = nullptr, void* r_out = nullptr,
                          const RowViews& views = RowViews{0, 0, 0, 0})
{
    const uint32_t hv = (uint32_t)(H / Storage<DT>::kN);
    u32x4* const in = static_cast<u32x4*>(input);
    u32x4* const res = static_cast<u32x4*>(residual);
    const u32x4* const w = static_cast<const u32x4*>(weight);
    u32x4* const yo = static_cast<u32x4*>(y_out);
    u32x4* const ro = static_cast<u32x4*>(r_out);
    const dim3 grid((uint32_t)li.grid);
    const float inv_h = 1.0f / (float)H;
    auto go = [&](auto group, auto width) {
        constexpr int G = decltype(group)::value, B = decltype(width)::value;
        fused_add_rmsnorm_short_row_kernel<DT, G, kNTLoad, kNTStore, STRIDED, B>
            <<<grid, dim3(B), 0, stream>>>(in, res, w, T, hv, inv_h, eps, li.log2_xcd_chunk, yo, ro, views);
    };
    auto with_group = [&](auto group) {
        if (li.block == 64) go(group, std::integral_constant<int, 64>{});
        else go(group, std::integral_constant<int, 256>{});
    };
    switch (li.block / li.rows_per_block) {
        case 8: with_group(std::integral_constant<int, 8>{}); break;
        case 16: with_group(std::integral_constant<int, 16>{}); break;
        default: with_group(std::integral_constant<int, 32>{}); break;
    }
}

// `ev` holds the row strides in elements; in place: y_out = x, r_out = r
template <int DT>
void launch_rmsnorm_ragged(const astra_launch_info_t& li, void* y_out, void* r_out, const void* x, const void* r,
                           const void* weight, const RowViews& ev, int64_t T, int64_t H, float eps, hipStream_t stream)
{
    typedef typename Storage<DT>::elem_t E;
    const dim3 grid((uint32_t)li.grid), block(li.block);
    const float inv_h = 1.0f / (float)H;
    E* const y = static_cast<E*>(y_out);
    E* const ro = static_cast<E*>(r_out);
    const E* const xi = static_cast<const E*>(x);
    const E* const ri = static_cast<const E*>(r);
    const E* const w = static_cast<const E*>(weight);
    auto go = [&](auto vpt, auto with_tail) {
        fused_add_rmsnorm_ragged_row_kernel<DT, decltype(vpt)::value, decltype(with_tail)::value, kNTLoad, kNTStore>
            <<<grid, block, 0, stream>>>(y, ro, xi, ri, w, ev, T, H, inv_h, eps, li.log2_xcd_chunk);
    };
    auto with_vpt = [&](auto vpt) {
        if (li.path == ASTRA_PATH_PHASED) {  // all four views in step: aligned chunks
            if (li.grid < T)  // more rows than the grid limit: workgroups walk several rows
                fused_add_rmsnorm_phased_row_kernel<DT, decltype(vpt)::value, kNTLoad, kNTStore, true>
                    <<<grid, block, 0, stream>>>(y, ro, xi, ri, w, ev, T, H, inv_h, eps, li.log2_xcd_chunk);
            else
                fused_add_rmsnorm_phased_row_kernel<DT, decltype(vpt)::value, kNTLoad, kNTStore, false>
                    <<<grid, block, 0, stream>>>(y, ro, xi, ri, w, ev, T, H, inv_h, eps, li.log2_xcd_chunk);
            return;
        }
        if (H % Storage<DT>::kN != 0) go(vpt, std::true_type{});
        else go(vpt, std::false_type{});  // only the pointers or strides are unaligned: no tail code at all
    };
    switch (li.vectors_per_lane) {
        case 1: with_vpt(std::integral_constant<int, 1>{}); break;
        case 2: with_vpt(std::integral_constant<int, 2>{}); break;
        default: with_vpt(std::integral_constant<int, 4>{}); break;
    }
}

template <int DT>
void launch_rmsnorm(const astra_launch_info_t& li, void* input, void* residual, const void* weight, int64_t T, int64_t H,
                    float eps, int variant, hipStream_t stream)
{
    typedef typename Storage<DT>::elem_t E;
    if constexpr (DT != kF32) {  // the ablation variants exist for the 16-bit storage types only
        if (variant == ASTRA_VARIANT_SCALAR_LOADS) {
            // same decomposition as the tuned kernel (one workgroup per row, row in registers), 16-bit accesses
            const int block = H >= 1024 ? 1024 : round_up((int)H, kWave);
            fused_add_rmsnorm_scalar_kernel<DT, 16>
                <<<dim3((uint32_t)(T < kMaxRowGrid ? T : kMaxRowGrid)), dim3(block), 0, stream>>>(
                    static_cast<uint16_t*>(input), static_cast<uint16_t*>(residual), static_cast<const uint16_t*>(weight), T,
                    (uint32_t)H, 1.0f / (float)H, eps);
            return;
        }
        if (variant == ASTRA_VARIANT_LDS_TREE_REDUCTION) {
            switch (li.vectors_per_lane) {
                case 1: launch_rmsnorm_row<DT, 1, 1024, true>(li, input, residual, weight, T, H, eps, stream); break;
                case 2: launch_rmsnorm_row<DT, 2, 1024, true>(li, input, residual, weight, T, H, eps, stream); break;
                default: launch_rmsnorm_row<DT, 4, 1024, true>(li, input, residual, weight, T, H, eps, stream); break;
            }
            return;
        }
    }
    if (li.path == ASTRA_PATH_GENERIC) {
        fused_add_rmsnorm_generic_kernel<DT><<<dim3((uint32_t)li.grid), dim3(li.block), 0, stream>>>(
            static_cast<E*>(input), static_cast<E*>(residual), static_cast<const E*>(weight), T, H, 1.0f / (float)H, eps);
        return;
    }
    if (li.path == ASTRA_PATH_RAGGED || li.path == ASTRA_PATH_PHASED) {
        launch_rmsnorm_ragged<DT>(li, input, residual, input, residual, weight, RowViews{H, H, H, H}, T, H, eps, stream);
        return;
    }
    if (li.rows_per_block > 0) {
        launch_rmsnorm_short<DT, false>(li, input, residual, weight, T, H, eps, stream);
        return;
    }
    // (ablation: device-scope stores instead of plain non-temporal ones)
    const int scope = variant == ASTRA_VARIANT_STORE_DEVICE_SCOPE_WHOLE_LINES ? kStoreScopeWholeLineRows
                      : variant == ASTRA_VARIANT_STORE_DEVICE_SCOPE ? kStoreScopeAlways : kStoreScopeNone;
    const RowViews none{0, 0, 0, 0};
    switch (li.vectors_per_lane) {
        case 1: launch_rmsnorm_row<DT, 1, 1024>(li, input, residual, weight, T, H, eps, stream, nullptr, nullptr, none, scope); break;
        case 2: launch_rmsnorm_row<DT, 2, 1024>(li, input, residual, weight, T, H, eps, stream, nullptr, nullptr, none, scope); break;
        default: launch_rmsnorm_row<DT, 4, 1024>(li, input, residual, weight, T, H, eps, stream, nullptr, nullptr, none, scope); break;
    }
}

template <int DT>
void launch_silu(const astra_launch_info_t& li, void* out, const void* in, int64_t T, int64_t d, int variant,
                 hipStream_t stream)
{
    typedef typename Storage<DT>::elem_t E;
    if constexpr (DT != kF32) {
        if (variant == ASTRA_VARIANT_SCALAR_LOADS) {
            const uint32_t n = (uint32_t)(T * d);
            silu_and_mul_scalar_kernel<DT><<<dim3((uint32_t)(((uint64_t)n + 255u) / 256u)), dim3(256), 0, stream>>>(
                static_cast<uint16_t*>(out), static_cast<const uint16_t*>(in), n, (uint32_t)d, make_fastdiv((uint32_t)d));
            return;
        }
        if (variant == ASTRA_VARIANT_LIBM_EXP_DIVIDE) {
            const uint32_t dv = (uint32_t)(d / Storage<DT>::kN);
            for_flat_block(li.block, [&](auto bc) {
                constexpr int B = decltype(bc)::value;
                silu_and_mul_vec_kernel<DT, kSiluUnroll, kNTLoad, kNTStore, true, B><<<dim3((uint32_t)li.grid), dim3(B), 0, stream>>>(
                    static_cast<u32x4*>(out), static_cast<const u32x4*>(in), (uint32_t)(T * dv), dv, make_fastdiv(dv),
                    li.log2_xcd_chunk);
            });
            return;
        }
    }
    if (li.path == ASTRA_PATH_GENERIC) {
        silu_and_mul_generic_kernel<DT><<<dim3((uint32_t)li.grid), dim3(li.block), 0, stream>>>(
            static_cast<E*>(out), static_cast<const E*>(in), T, d);
        return;
    }
    if (li.path == ASTRA_PATH_PHASED) {  // the aligned chunks of the output, `phase` elements past the 16-byte grid
        constexpr int N = Storage<DT>::kN;
        const int phase = (int)((reinterpret_cast<uintptr_t>(out) & 15u) / sizeof(E));
        const uint32_t chunks = (uint32_t)((T * d + phase + N - 1) / N);
        for_flat_block(li.block, [&](auto bc) {
            constexpr int B = decltype(bc)::value;
            silu_and_mul_phased_kernel<DT, kNTLoad, kNTStore, B><<<dim3((uint32_t)li.grid), dim3(B), 0, stream>>>(
                static_cast<E*>(out), static_cast<const E*>(in), (uint32_t)T, (uint32_t)d, make_fastdiv((uint32_t)d), chunks,
                phase, li.log2_xcd_chunk);
        });
        return;
    }
    if (li.path == ASTRA_PATH_RAGGED) {
        const uint32_t dvr = (uint32_t)((d + Storage<DT>::kN - 1) / Storage<DT>::kN);
        silu_and_mul_ragged_kernel<DT, kNTLoad, kNTStore><<<dim3((uint32_t)li.grid), dim3(256), 0, stream>>>(
            static_cast<E*>(out), d, static_cast<const E*>(in), 2 * d, (uint32_t)(T * dvr), dvr, d, make_fastdiv(dvr));
        return;
    }
    const uint32_t dv = (uint32_t)(d / Storage<DT>::kN);
    if (li.access_bytes == kVecBytes / 2) {  // small problem: half a vector per lane, plain accesses
        silu_and_mul_small_kernel<DT><<<dim3((uint32_t)li.grid), dim3(256), 0, stream>>>(
            static_cast<u32x2*>(out), static_cast<const u32x2*>(in), (uint32_t)(2 * T * dv), 2 * dv, make_fastdiv(2 * dv));
        return;
    }
    for_flat_block(li.block, [&](auto bc) {
        constexpr int B = decltype(bc)::value;
        if (dv < kSiluLaneDivBelow)
            silu_and_mul_vec_kernel<DT, kSiluUnroll, kNTLoad, kNTStore, false, B, true>
                <<<dim3((uint32_t)li.grid), dim3(B), 0, stream>>>(static_cast<u32x4*>(out), static_cast<const u32x4*>(in),
                                                                  (uint32_t)(T * dv), dv, make_fastdiv(dv), li.log2_xcd_chunk);
        else
            silu_and_mul_vec_kernel<DT, kSiluUnroll, kNTLoad, kNTStore, false, B><<<dim3((uint32_t)li.grid), dim3(B), 0, stream>>>(
                static_cast<u32x4*>(out), static_cast<const u32x4*>(in), (uint32_t)(T * dv), dv, make_fastdiv(dv),
                li.log2_xcd_chunk);
    });
}

template <int DT>
void launch_merge(const astra_launch_info_t& li, void* v_out, float* lse_out, const void* v_a, const float* lse_a,
                  const void* v_b, const float* lse_b, int64_t pairs, int64_t D, int variant, hipStream_t stream)
{
    typedef typename Storage<DT>::elem_t E;
    if constexpr (DT != kF32) {
        if (variant == ASTRA_VARIANT_SCALAR_LOADS) {
            const uint32_t n = (uint32_t)(pairs * D);
            merge_attn_states_lse_scalar_kernel<DT><<<dim3((uint32_t)(((uint64_t)n + 255u) / 256u)), dim3(256), 0, stream>>>(
                static_cast<uint16_t*>(v_out), lse_out, static_cast<const uint16_t*>(v_a), lse_a,
                static_cast<const uint16_t*>(v_b), lse_b, n, (uint32_t)D, make_fastdiv((uint32_t)D));
            return;
        }
        if (variant == ASTRA_VARIANT_UNHOISTED_WEIGHTS) {
            const uint32_t dvec = (uint32_t)(D / Storage<DT>::kN);
            const int log2_dvec = (dvec & (dvec - 1)) == 0 ? __builtin_ctz(dvec) : -1;
            for_flat_block(li.block, [&](auto bc) {
                constexpr int B = decltype(bc)::value;
                merge_attn_states_lse_vec_kernel<DT, kMergeUnroll, kNTLoad, kNTStore, false, B>
                    <<<dim3((uint32_t)li.grid), dim3(B), 0, stream>>>(
                        static_cast<u32x4*>(v_out), lse_out, static_cast<const u32x4*>(v_a), lse_a,
                        static_cast<const u32x4*>(v_b), lse_b, (uint32_t)(pairs * dvec), dvec, log2_dvec, make_fastdiv(dvec),
                        li.log2_xcd_chunk);
            });
            return;
        }
    }
    if (li.path == ASTRA_PATH_GENERIC) {
        merge_attn_states_lse_generic_kernel<DT><<<dim3((uint32_t)li.grid), dim3(li.block), 0, stream>>>(
            static_cast<E*>(v_out), lse_out, static_cast<const E*>(v_a), lse_a, static_cast<const E*>(v_b), lse_b, pairs, D);
        return;
    }
    if (li.path == ASTRA_PATH_RAGGED) {
        const uint32_t dvr = (uint32_t)((D + Storage<DT>::kN - 1) / Storage<DT>::kN);
        merge_attn_states_lse_ragged_kernel<DT, kNTLoad, kNTStore><<<dim3((uint32_t)li.grid), dim3(256), 0, stream>>>(
            static_cast<E*>(v_out), lse_out, static_cast<const E*>(v_a), lse_a, static_cast<const E*>(v_b), lse_b,
            (uint32_t)(pairs * dvr), dvr, D, make_fastdiv(dvr));
        return;
    }
    if (li.path == ASTRA_PATH_PHASED) {  // the aligned chunks of the output
        constexpr int N = Storage<DT>::kN;
        const int phase = (int)((reinterpret_cast<uintptr_t>(v_out) / sizeof(E)) & (N - 1));
        const int64_t n = pairs * D;
        for_flat_block(li.block, [&](auto bc) {
            constexpr int B = decltype(bc)::value;
            merge_attn_states_lse_phased_kernel<DT, kNTLoad, kNTStore, B><<<dim3((uint32_t)li.grid), dim3(B), 0, stream>>>(
                static_cast<E*>(v_out), lse_out, static_cast<const E*>(v_a), lse_a, static_cast<const E*>(v_b), lse_b,
                (uint32_t)n, (uint32_t)D, make_fastdiv((uint32_t)D), (uint32_t)((n + phase + N - 1) / N), phase,
                li.log2_xcd_chunk);
        });
        return;
    }
    const uint32_t dvec = (uint32_t)(D / Storage<DT>::kN);
    int log2_dvec = -1;
    if ((dvec & (dvec - 1)) == 0) log2_dvec = __builtin_ctz(dvec);
    for_flat_block(li.block, [&](auto bc) {
        constexpr int B = decltype(bc)::value;
        auto go = [&](auto nt) {
            constexpr bool NT = decltype(nt)::value;
            merge_attn_states_lse_vec_kernel<DT, kMergeUnroll, kNTLoad && NT, kNTStore && NT, true, B>
                <<<dim3((uint32_t)li.grid), dim3(B), 0, stream>>>(static_cast<u32x4*>(v_out), lse_out,
                                                                  static_cast<const u32x4*>(v_a), lse_a,
                                                                  static_cast<const u32x4*>(v_b), lse_b, (uint32_t)(pairs * dvec),
                                                                  dvec, log2_dvec, make_fastdiv(dvec), li.log2_xcd_chunk);
        };
        if (li.non_temporal) go(std::true_type{});
        else go(std::false_type{});  // small problems: plain cached accesses
    });
}

// every part of the K-way input starts 16-byte aligned when the base is and head_dim is a whole number of
// vectors, which are the fast-path conditions already
template <int DT>
void launch_merge_kway(const astra_launch_info_t& li, void* v_out, float* lse_out, const void* v_parts,
                       const float* lse_parts, int64_t K, int64_t pairs, int64_t D, hipStream_t stream)
{
    if (li.path == ASTRA_PATH_RAGGED) {
        typedef typename Storage<DT>::elem_t E;
        const uint32_t dvr = (uint32_t)((D + Storage<DT>::kN - 1) / Storage<DT>::kN);
        merge_attn_states_lse_kway_ragged_kernel<DT, kKwayGroup, kNTLoad, kNTStore>
            <<<dim3((uint32_t)li.grid), dim3(256), 0, stream>>>(static_cast<E*>(v_out), lse_out, static_cast<const E*>(v_parts),
                                                                lse_parts, (uint32_t)K, (uint32_t)(pairs * dvr), pairs, dvr, D,
                                                                make_fastdiv(dvr));
        return;
    }
    const uint32_t dvec = (uint32_t)(D / Storage<DT>::kN);
    const int log2_dvec = (dvec & (dvec - 1)) == 0 ? __builtin_ctz(dvec) : -1;
    for_flat_block(li.block, [&](auto bc) {
        constexpr int B = decltype(bc)::value;
        merge_attn_states_lse_kway_vec_kernel<DT, kKwayGroup, kNTLoad, kNTStore, B><<<dim3((uint32_t)li.grid), dim3(B), 0, stream>>>(
            static_cast<u32x4*>(v_out), lse_out, static_cast<const u32x4*>(v_parts), lse_parts, (uint32_t)K,
            (uint32_t)(pairs * dvec), (uint32_t)pairs, dvec, log2_dvec, make_fastdiv(dvec), li.log2_xcd_chunk);
    });
}

// `ev` holds the row strides in elements
template <int DT>
void launch_rmsnorm_strided(const astra_launch_info_t& li, void* y_out, void* r_out, const void* x, const void* r,
                            const void* weight, const RowViews& ev, int64_t T, int64_t H, float eps, hipStream_t stream)
{
    if (li.path == ASTRA_PATH_GENERIC) {
        typedef typename Storage<DT>::elem_t E;
        fused_add_rmsnorm_strided_generic_kernel<DT><<<dim3((uint32_t)li.grid), dim3(256), 0, stream>>>(
            static_cast<E*>(y_out), static_cast<E*>(r_out), static_cast<const E*>(x), static_cast<const E*>(r),
            static_cast<const E*>(weight), ev, T, H, 1.0f / (float)H, eps);
        return;
    }
    if (li.path == ASTRA_PATH_RAGGED || li.path == ASTRA_PATH_PHASED) {
        launch_rmsnorm_ragged<DT>(li, y_out, r_out, x, r, weight, ev, T, H, eps, stream);
        return;
    }
    constexpr int N = Storage<DT>::kN;
    const RowViews vv{ev.y_stride / N, ev.r_out_stride / N, ev.x_stride / N, ev.r_stride / N};
    void* const xin = const_cast<void*>(x);  // read only when STRIDED
    void* const rin = const_cast<void*>(r);
    if (li.rows_per_block > 0) {
        launch_rmsnorm_short<DT, true>(li, xin, rin, weight, T, H, eps, stream, y_out, r_out, vv);
        return;
    }
    switch (li.vectors_per_lane) {
        case 1: launch_rmsnorm_row<DT, 1, 1024, false, true>(li, xin, rin, weight, T, H, eps, stream, y_out, r_out, vv); break;
        case 2: launch_rmsnorm_row<DT, 2, 1024, false, true>(li, xin, rin, weight, T, H, eps, stream, y_out, r_out, vv); break;
        default: launch_rmsnorm_row<DT, 4, 1024, false, true>(li, xin, rin, weight, T, H, eps, stream, y_out, r_out, vv); break;
    }
}

}  // namespace

// =======================================================================================================
// exported C ABI

extern "C" {

const char* astra_status_string(astra_status_t status)
{
    switch (status) {
        case ASTRA_OK: return "ok";
        case ASTRA_ERR_NULL: return "null pointer argument";
        case ASTRA_ERR_SHAPE: return "invalid shape";
        case ASTRA_ERR_DTYPE: return "unknown dtype";
        case ASTRA_ERR_EPS: return "eps is negative or NaN";
        case ASTRA_ERR_ALIGN: return "pointer not aligned to its element size";
        case ASTRA_ERR_ALIAS: return "output overlaps an input";
        case ASTRA_ERR_LAUNCH: return "kernel launch failed";
        case ASTRA_ERR_VARIANT: return "ablation variant not applicable to this operator or shape";
        default: break;
    }
    return "unknown status";
}

uint32_t astra_plan_xcd_chunked(uint32_t workgroup, int log2_chunk)
{
    if (log2_chunk < 0 || log2_chunk > kMaxChunkLog2) return workgroup;
    return xcd_chunked(workgroup, log2_chunk);
}

astra_status_t astra_plan_fused_add_rmsnorm(int64_t T, int64_t H, astra_dtype_t dtype, int aligned16,
                                            astra_launch_info_t* info)
{
    if (!info) return ASTRA_ERR_NULL;
    const astra_status_t st = plan_rmsnorm(T, H, elem_bytes((int)dtype), plan_align(aligned16), info, true, true, true);
    return st == ASTRA_OK && !valid_dtype((int)dtype) ? ASTRA_ERR_DTYPE : st;
}

astra_status_t astra_plan_silu_and_mul(int64_t T, int64_t d, astra_dtype_t dtype, int aligned16, astra_launch_info_t* info)
{
    if (!info) return ASTRA_ERR_NULL;
    const astra_status_t st = plan_silu(T, d, elem_bytes((int)dtype), plan_align(aligned16), info);
    return st == ASTRA_OK && !valid_dtype((int)dtype) ? ASTRA_ERR_DTYPE : st;
}

astra_status_t astra_plan_merge_attn_states_lse(int64_t T, int64_t num_heads, int64_t head_dim, astra_dtype_t dtype,
                                                int aligned16, astra_launch_info_t* info)
{
    if (!info) return ASTRA_ERR_NULL;
    const astra_status_t st = plan_merge(T, num_heads, head_dim, elem_bytes((int)dtype), plan_align(aligned16), info);
    return st == ASTRA_OK && !valid_dtype((int)dtype) ? ASTRA_ERR_DTYPE : st;
}

static astra_status_t run_fused_add_rmsnorm(void* input, void* residual, const void* weight, int64_t T, int64_t H,
                                            astra_dtype_t dtype, float eps, int variant, hipStream_t stream)
{
    if (!input || !residual || !weight) return ASTRA_ERR_NULL;
    astra_launch_info_t li;
    const int eb = elem_bytes((int)dtype);
    astra_status_t st = plan_rmsnorm(T, H, eb, align_class(input, residual), &li, variant == ASTRA_VARIANT_TUNED, aligned(weight, 16),
                                     variant == ASTRA_VARIANT_TUNED);
    if (st != ASTRA_OK) return st;
    if (!valid_dtype((int)dtype)) return ASTRA_ERR_DTYPE;
    if (!(eps >= 0.0f)) return ASTRA_ERR_EPS;
    if (!aligned(input, eb) || !aligned(residual, eb) || !aligned(weight, eb)) return ASTRA_ERR_ALIGN;
    const int64_t bytes = T * H * eb;
    if (overlaps(input, bytes, residual, bytes) || overlaps(input, bytes, weight, H * eb) ||
        overlaps(residual, bytes, weight, H * eb))
        return ASTRA_ERR_ALIAS;
    if (variant == ASTRA_VARIANT_ELEMENT_WISE) {
        li = launch_info(T > 0 ? ASTRA_PATH_GENERIC : ASTRA_PATH_NONE, 256, 0, 0, T < kMaxGenericGrid ? T : kMaxGenericGrid, 0, 0);
    } else if (variant >= ASTRA_VARIANT_PACE_NONE && variant <= ASTRA_VARIANT_PACE_WEIGHT_X_R) {
        // the tuned row kernel with a forced pace: only where the plan launches it with one row per workgroup
        if (T > 0 && (li.path != ASTRA_PATH_VECTOR || li.rows_per_block != 0 || li.grid < T)) return ASTRA_ERR_VARIANT;
        static const int forced[4] = {kPaceNone, kPaceStoreGap, kPaceXBeforeR, kPaceWeightFirst | kPaceXBeforeR};
        li.pace = forced[variant - ASTRA_VARIANT_PACE_NONE];
        variant = ASTRA_VARIANT_TUNED;
    } else if (variant == ASTRA_VARIANT_STORE_DEVICE_SCOPE_WHOLE_LINES || variant == ASTRA_VARIANT_STORE_DEVICE_SCOPE) {
        // the tuned row kernel, paced as the plan says, with device-scope stores: same shapes as the forced paces
        if (T > 0 && (li.path != ASTRA_PATH_VECTOR || li.rows_per_block != 0 || li.grid < T)) return ASTRA_ERR_VARIANT;
    } else if (variant != ASTRA_VARIANT_TUNED) {
        if (dtype == ASTRA_F32) return ASTRA_ERR_VARIANT;
        if (variant != ASTRA_VARIANT_SCALAR_LOADS && variant != ASTRA_VARIANT_LDS_TREE_REDUCTION) return ASTRA_ERR_VARIANT;
        if (T > 0 && li.path != ASTRA_PATH_VECTOR) return ASTRA_ERR_VARIANT;
        if (variant == ASTRA_VARIANT_SCALAR_LOADS && H > 16384) return ASTRA_ERR_VARIANT;
    }
    if (T == 0) return ASTRA_OK;
    for_dtype(dtype, [&](auto dt) { launch_rmsnorm<decltype(dt)::value>(li, input, residual, weight, T, H, eps, variant, stream); });
    return after_launch();
}

astra_status_t astra_fused_add_rmsnorm(void* input, void* residual, const void* weight, int64_t T, int64_t H,
                                       astra_dtype_t dtype, float eps, hipStream_t stream)
{
    return run_fused_add_rmsnorm(input, residual, weight, T, H, dtype, eps, ASTRA_VARIANT_TUNED, stream);
}

astra_status_t astra_ablation_fused_add_rmsnorm(void* input, void* residual, const void* weight, int64_t T, int64_t H,
                                                astra_dtype_t dtype, float eps, astra_variant_t variant,
                                                hipStream_t stream)
{
    return run_fused_add_rmsnorm(input, residual, weight, T, H, dtype, eps, (int)variant, stream);
}

static astra_status_t run_silu_and_mul(void* out, const void* input, int64_t T, int64_t d, astra_dtype_t dtype,
                                       int variant, hipStream_t stream)
{
    if (!out || !input) return ASTRA_ERR_NULL;
    astra_launch_info_t li;
    const int eb = elem_bytes((int)dtype);
    astra_status_t st = plan_silu(T, d, eb, align_class(out, input), &li);
    if (st != ASTRA_OK) return st;
    if (!valid_dtype((int)dtype)) return ASTRA_ERR_DTYPE;
    if (!aligned(out, eb) || !aligned(input, eb)) return ASTRA_ERR_ALIGN;
    if (overlaps(out, T * d * eb, input, T * d * 2 * eb)) return ASTRA_ERR_ALIAS;
    if (variant == ASTRA_VARIANT_ELEMENT_WISE) {
        li = launch_info(T > 0 ? ASTRA_PATH_GENERIC : ASTRA_PATH_NONE, 256, 0, 0, T < kMaxGenericGrid ? T : kMaxGenericGrid, 0, 0);
    } else if (variant != ASTRA_VARIANT_TUNED) {
        if (dtype == ASTRA_F32) return ASTRA_ERR_VARIANT;
        if (variant != ASTRA_VARIANT_SCALAR_LOADS && variant != ASTRA_VARIANT_LIBM_EXP_DIVIDE) return ASTRA_ERR_VARIANT;
        if (T > 0 && li.path != ASTRA_PATH_VECTOR) return ASTRA_ERR_VARIANT;
        if (variant == ASTRA_VARIANT_SCALAR_LOADS && T * d >= (int64_t(1) << 32)) return ASTRA_ERR_VARIANT;
    }
    if (T == 0) return ASTRA_OK;
    for_dtype(dtype, [&](auto dt) { launch_silu<decltype(dt)::value>(li, out, input, T, d, variant, stream); });
    return after_launch();
}

astra_status_t astra_silu_and_mul(void* out, const void* input, int64_t T, int64_t d, astra_dtype_t dtype,
                                  hipStream_t stream)
{
    return run_silu_and_mul(out, input, T, d, dtype, ASTRA_VARIANT_TUNED, stream);
}

astra_status_t astra_ablation_silu_and_mul(void* out, const void* input, int64_t T, int64_t d, astra_dtype_t dtype,
                                           astra_variant_t variant, hipStream_t stream)
{
    return run_silu_and_mul(out, input, T, d, dtype, (int)variant, stream);
}

static astra_status_t run_merge_attn_states_lse(void* v_out, float* lse_out, const void* v_a, const float* lse_a,
                                                const void* v_b, const float* lse_b, int64_t T, int64_t num_heads,
                                                int64_t head_dim, astra_dtype_t dtype, int variant, hipStream_t stream)
{
    if (!v_out || !lse_out || !v_a || !lse_a || !v_b || !lse_b) return ASTRA_ERR_NULL;
    astra_launch_info_t li;
    const int eb = elem_bytes((int)dtype);
    astra_status_t st =
        plan_merge(T, num_heads, head_dim, eb, align_class(v_out, v_a, v_b), &li);
    if (st != ASTRA_OK) return st;
    if (!valid_dtype((int)dtype)) return ASTRA_ERR_DTYPE;
    if (!aligned(v_out, eb) || !aligned(v_a, eb) || !aligned(v_b, eb) || !aligned(lse_out, 4) || !aligned(lse_a, 4) ||
        !aligned(lse_b, 4))
        return ASTRA_ERR_ALIGN;
    const int64_t pairs = T * num_heads;
    const int64_t vbytes = pairs * head_dim * eb, sbytes = pairs * 4;
    if ((v_out != v_a && overlaps(v_out, vbytes, v_a, vbytes)) || (v_out != v_b && overlaps(v_out, vbytes, v_b, vbytes)) ||
        overlaps(lse_out, sbytes, lse_a, sbytes) || overlaps(lse_out, sbytes, lse_b, sbytes) ||
        overlaps(v_out, vbytes, lse_a, sbytes) || overlaps(v_out, vbytes, lse_b, sbytes) ||
        overlaps(lse_out, sbytes, v_a, vbytes) || overlaps(lse_out, sbytes, v_b, vbytes) ||
        overlaps(lse_out, sbytes, v_out, vbytes))
        return ASTRA_ERR_ALIAS;
    if (variant == ASTRA_VARIANT_ELEMENT_WISE) {
        li = launch_info(T > 0 ? ASTRA_PATH_GENERIC : ASTRA_PATH_NONE, 256, 0, 0, pairs < kMaxGenericGrid ? pairs : kMaxGenericGrid, 0, 0);
    } else if (variant != ASTRA_VARIANT_TUNED) {
        if (dtype == ASTRA_F32) return ASTRA_ERR_VARIANT;
        if (variant != ASTRA_VARIANT_SCALAR_LOADS && variant != ASTRA_VARIANT_UNHOISTED_WEIGHTS) return ASTRA_ERR_VARIANT;
        if (T > 0 && li.path != ASTRA_PATH_VECTOR) return ASTRA_ERR_VARIANT;
        if (variant == ASTRA_VARIANT_SCALAR_LOADS && pairs * head_dim >= (int64_t(1) << 32)) return ASTRA_ERR_VARIANT;
    }
    if (T == 0) return ASTRA_OK;
    for_dtype(dtype, [&](auto dt) {
        launch_merge<decltype(dt)::value>(li, v_out, lse_out, v_a, lse_a, v_b, lse_b, pairs, head_dim, variant, stream);
    });
    return after_launch();
}

astra_status_t astra_merge_attn_states_lse(void* v_out, float* lse_out, const void* v_a, const float* lse_a,
                                           const void* v_b, const float* lse_b, int64_t T, int64_t num_heads,
                                           int64_t head_dim, astra_dtype_t dtype, hipStream_t stream)
{
    return run_merge_attn_states_lse(v_out, lse_out, v_a, lse_a, v_b, lse_b, T, num_heads, head_dim, dtype,
                                     ASTRA_VARIANT_TUNED, stream);
}

astra_status_t astra_ablation_merge_attn_states_lse(void* v_out, float* lse_out, const void* v_a, const float* lse_a,
                                                    const void* v_b, const float* lse_b, int64_t T, int64_t num_heads,
                                                    int64_t head_dim, astra_dtype_t dtype, astra_variant_t variant,
                                                    hipStream_t stream)
{
    return run_merge_attn_states_lse(v_out, lse_out, v_a, lse_a, v_b, lse_b, T, num_heads, head_dim, dtype, (int)variant,
                                     stream);
}

astra_status_t astra_merge_attn_states_lse_kway(void* v_out, float* lse_out, const void* v_parts,
                                                const float* lse_parts, int64_t K, int64_t T, int64_t num_heads,
                                                int64_t head_dim, astra_dtype_t dtype, hipStream_t stream)
{
    if (!v_out || !lse_out || !v_parts || !lse_parts) return ASTRA_ERR_NULL;
    astra_launch_info_t li;
    const int eb = elem_bytes((int)dtype);
    const int align = aligned(v_out, 16) && aligned(v_parts, 16) ? kAlign16 : kAlignNone;
    astra_status_t st = plan_merge(T, num_heads, head_dim, eb, align, &li, true);
    if (st != ASTRA_OK) return st;
    if (li.path == ASTRA_PATH_GENERIC) return ASTRA_ERR_SHAPE;  // more than 2^31 output vectors
    const int64_t pairs = T * num_heads;
    int64_t part_elems = pairs * head_dim, all_elems;
    if (K < 1 || K > 65536 || mul_overflows(part_elems, K, &all_elems) || all_elems > std::numeric_limits<int64_t>::max() / 4)
        return ASTRA_ERR_SHAPE;
    if (!valid_dtype((int)dtype)) return ASTRA_ERR_DTYPE;
    if (!aligned(v_out, eb) || !aligned(v_parts, eb) || !aligned(lse_out, 4) || !aligned(lse_parts, 4)) return ASTRA_ERR_ALIGN;
    const int64_t vbytes = part_elems * eb, sbytes = pairs * 4;
    if (overlaps(v_out, vbytes, v_parts, vbytes * K) || overlaps(v_out, vbytes, lse_parts, sbytes * K) ||
        overlaps(lse_out, sbytes, v_parts, vbytes * K) || overlaps(lse_out, sbytes, lse_parts, sbytes * K) ||
        overlaps(lse_out, sbytes, v_out, vbytes))
        return ASTRA_ERR_ALIAS;
    if (T == 0) return ASTRA_OK;
    for_dtype(dtype, [&](auto dt) {
        launch_merge_kway<decltype(dt)::value>(li, v_out, lse_out, v_parts, lse_parts, K, pairs, head_dim, stream);
    });
    return after_launch();
}

astra_status_t astra_fused_add_rmsnorm_strided(void* y_out, int64_t y_stride, void* r_out, int64_t r_out_stride,
                                               const void* x, int64_t x_stride, const void* r, int64_t r_stride,
                                               const void* weight, int64_t T, int64_t H, astra_dtype_t dtype, float eps,
                                               hipStream_t stream)
{
    if (!y_out || !r_out || !x || !r || !weight) return ASTRA_ERR_NULL;
    const int64_t strides[4] = {y_stride, r_out_stride, x_stride, r_stride};
    const void* const bases[4] = {y_out, r_out, x, r};
    const int eb = elem_bytes((int)dtype);
    // every view on the 16-byte grid, or at least all four in step with each other in every row
    int ac = align_class(y_out, r_out, x, r);
    for (int i = 0; i < 4; ++i) {
        if (ac == kAlign16 && strides[i] % (kVecBytes / eb) != 0) ac = kAlignPhased;
        if (strides[i] % (kVecBytes / eb) != strides[0] % (kVecBytes / eb)) ac = kAlignNone;  // (no difference of strides: it could overflow)
    }
    astra_launch_info_t li;
    astra_status_t st = plan_rmsnorm(T, H, eb, ac, &li, true, aligned(weight, 16));
    if (st != ASTRA_OK) return st;
    int64_t span[4];  // bounding extent of each view in bytes
    for (int i = 0; i < 4; ++i) {
        int64_t rows_bytes;
        if (strides[i] < H || mul_overflows(T > 0 ? T - 1 : 0, strides[i], &rows_bytes) ||
            rows_bytes > std::numeric_limits<int64_t>::max() / 8)
            return ASTRA_ERR_SHAPE;
        span[i] = T > 0 ? (rows_bytes + H) * eb : 0;
    }
    if (!valid_dtype((int)dtype)) return ASTRA_ERR_DTYPE;
    if (!(eps >= 0.0f)) return ASTRA_ERR_EPS;
    for (int i = 0; i < 4; ++i)
        if (!aligned(bases[i], eb)) return ASTRA_ERR_ALIGN;
    if (!aligned(weight, eb)) return ASTRA_ERR_ALIGN;
    const bool y_in_place = (y_out == x && y_stride == x_stride), r_in_place = (r_out == r && r_out_stride == r_stride);
    if ((!y_in_place && overlaps(y_out, span[0], x, span[2])) || (!r_in_place && overlaps(r_out, span[1], r, span[3])) ||
        overlaps(y_out, span[0], r, span[3]) || overlaps(r_out, span[1], x, span[2]) ||
        overlaps(y_out, span[0], r_out, span[1]) || overlaps(y_out, span[0], weight, H * eb) ||
        overlaps(r_out, span[1], weight, H * eb))
        return ASTRA_ERR_ALIAS;
    if (T == 0) return ASTRA_OK;
    const RowViews views{y_stride, r_out_stride, x_stride, r_stride};
    for_dtype(dtype, [&](auto dt) {
        launch_rmsnorm_strided<decltype(dt)::value>(li, y_out, r_out, x, r, weight, views, T, H, eps, stream);
    });
    return after_launch();
}

astra_status_t astra_silu_and_mul_strided(void* out, int64_t out_stride, const void* input, int64_t in_stride, int64_t T,
                                          int64_t d, astra_dtype_t dtype, hipStream_t stream)
{
    if (!out || !input) return ASTRA_ERR_NULL;
    const int eb = elem_bytes((int)dtype);
    const int64_t ne = kVecBytes / eb;
    const bool fast = aligned(out, 16) && aligned(input, 16) && out_stride % ne == 0 && in_stride % ne == 0;
    astra_launch_info_t li;
    astra_status_t st = plan_silu(T, d, eb, fast ? kAlign16 : kAlignNone, &li, true);
    if (st != ASTRA_OK) return st;
    if (li.path == ASTRA_PATH_GENERIC) return ASTRA_ERR_SHAPE;  // more than 2^31 output vectors
    int64_t out_rows, in_rows;
    if (out_stride < d || in_stride < 2 * d || mul_overflows(T > 0 ? T - 1 : 0, out_stride, &out_rows) ||
        mul_overflows(T > 0 ? T - 1 : 0, in_stride, &in_rows) || out_rows > std::numeric_limits<int64_t>::max() / 8 ||
        in_rows > std::numeric_limits<int64_t>::max() / 8)
        return ASTRA_ERR_SHAPE;
    if (!valid_dtype((int)dtype)) return ASTRA_ERR_DTYPE;
    if (!aligned(out, eb) || !aligned(input, eb)) return ASTRA_ERR_ALIGN;
    const int64_t out_span = T > 0 ? (out_rows + d) * eb : 0, in_span = T > 0 ? (in_rows + 2 * d) * eb : 0;
    if (overlaps(out, out_span, input, in_span)) return ASTRA_ERR_ALIAS;
    if (T == 0) return ASTRA_OK;
    for_dtype(dtype, [&](auto dtc) {
        constexpr int DT = decltype(dtc)::value;
        typedef typename Storage<DT>::elem_t E;
        if (li.path == ASTRA_PATH_RAGGED) {
            const uint32_t dvr = (uint32_t)((d + Storage<DT>::kN - 1) / Storage<DT>::kN);
            silu_and_mul_ragged_kernel<DT, kNTLoad, kNTStore><<<dim3((uint32_t)li.grid), dim3(256), 0, stream>>>(
                static_cast<E*>(out), out_stride, static_cast<const E*>(input), in_stride, (uint32_t)(T * dvr), dvr, d,
                make_fastdiv(dvr));
        } else {
            const uint32_t dv = (uint32_t)(d / Storage<DT>::kN);
            for_flat_block(li.block, [&](auto bc) {
                constexpr int B = decltype(bc)::value;
                silu_and_mul_strided_vec_kernel<DT, kNTLoad, kNTStore, B><<<dim3((uint32_t)li.grid), dim3(B), 0, stream>>>(
                    static_cast<u32x4*>(out), out_stride / Storage<DT>::kN, static_cast<const u32x4*>(input),
                    in_stride / Storage<DT>::kN, (uint32_t)(T * dv), dv, make_fastdiv(dv), li.log2_xcd_chunk);
            });
        }
    });
    return after_launch();
}

astra_status_t astra_merge_attn_states_lse_strided(void* v_out, int64_t out_token_stride, int64_t out_head_stride,
                                                   float* lse_out, const void* v_a, int64_t a_token_stride,
                                                   int64_t a_head_stride, const float* lse_a, const void* v_b,
                                                   int64_t b_token_stride, int64_t b_head_stride, const float* lse_b,
                                                   int64_t T, int64_t num_heads, int64_t head_dim, astra_dtype_t dtype,
                                                   hipStream_t stream)
{
    if (!v_out || !lse_out || !v_a || !lse_a || !v_b || !lse_b) return ASTRA_ERR_NULL;
    const int eb = elem_bytes((int)dtype);
    const int64_t ne = kVecBytes / eb;
    const int64_t ts[3] = {out_token_stride, a_token_stride, b_token_stride};
    const int64_t hs[3] = {out_head_stride, a_head_stride, b_head_stride};
    const void* const bases[3] = {v_out, v_a, v_b};
    bool fast = true;
    for (int i = 0; i < 3; ++i) fast = fast && aligned(bases[i], 16) && ts[i] % ne == 0 && hs[i] % ne == 0;
    astra_launch_info_t li;
    astra_status_t st = plan_merge(T, num_heads, head_dim, eb, fast ? kAlign16 : kAlignNone, &li, true);
    if (st != ASTRA_OK) return st;
    if (li.path == ASTRA_PATH_GENERIC) return ASTRA_ERR_SHAPE;  // more than 2^31 output vectors
    int64_t span[3];  // bounding extent of each value view in bytes
    for (int i = 0; i < 3; ++i) {
        int64_t heads_ext, tok_ext, total;
        if (hs[i] < head_dim || mul_overflows(num_heads - 1, hs[i], &heads_ext) ||
            __builtin_add_overflow(heads_ext, head_dim, &heads_ext) || ts[i] < heads_ext ||
            mul_overflows(T > 0 ? T - 1 : 0, ts[i], &tok_ext) || __builtin_add_overflow(tok_ext, heads_ext, &total) ||
            total > std::numeric_limits<int64_t>::max() / 8)
            return ASTRA_ERR_SHAPE;
        span[i] = T > 0 ? total * eb : 0;
    }
    if (!valid_dtype((int)dtype)) return ASTRA_ERR_DTYPE;
    for (int i = 0; i < 3; ++i)
        if (!aligned(bases[i], eb)) return ASTRA_ERR_ALIGN;
    if (!aligned(lse_out, 4) || !aligned(lse_a, 4) || !aligned(lse_b, 4)) return ASTRA_ERR_ALIGN;
    const int64_t pairs = T * num_heads, sbytes = pairs * 4;
    const bool out_is_a = (v_out == v_a && ts[0] == ts[1] && hs[0] == hs[1]);
    const bool out_is_b = (v_out == v_b && ts[0] == ts[2] && hs[0] == hs[2]);
    if ((!out_is_a && overlaps(v_out, span[0], v_a, span[1])) || (!out_is_b && overlaps(v_out, span[0], v_b, span[2])) ||
        overlaps(lse_out, sbytes, lse_a, sbytes) || overlaps(lse_out, sbytes, lse_b, sbytes) ||
        overlaps(v_out, span[0], lse_a, sbytes) || overlaps(v_out, span[0], lse_b, sbytes) ||
        overlaps(lse_out, sbytes, v_a, span[1]) || overlaps(lse_out, sbytes, v_b, span[2]) ||
        overlaps(lse_out, sbytes, v_out, span[0]))
        return ASTRA_ERR_ALIAS;
    if (T == 0) return ASTRA_OK;
    for_dtype(dtype, [&](auto dtc) {
        constexpr int DT = decltype(dtc)::value;
        constexpr int N = Storage<DT>::kN;
        typedef typename Storage<DT>::elem_t E;
        if (li.path == ASTRA_PATH_RAGGED) {
            const ValueStrides vs{ts[0], hs[0], ts[1], hs[1], ts[2], hs[2]};
            const uint32_t dvr = (uint32_t)((head_dim + N - 1) / N);
            merge_attn_states_lse_ragged_kernel<DT, kNTLoad, kNTStore, true><<<dim3((uint32_t)li.grid), dim3(256), 0, stream>>>(
                static_cast<E*>(v_out), lse_out, static_cast<const E*>(v_a), lse_a, static_cast<const E*>(v_b), lse_b,
                (uint32_t)(pairs * dvr), dvr, head_dim, make_fastdiv(dvr), vs, make_fastdiv((uint32_t)num_heads),
                (uint32_t)num_heads);
        } else {
            const ValueStrides vs{ts[0] / N, hs[0] / N, ts[1] / N, hs[1] / N, ts[2] / N, hs[2] / N};
            const uint32_t dvec = (uint32_t)(head_dim / N);
            for_flat_block(li.block, [&](auto bc) {
                constexpr int B = decltype(bc)::value;
                merge_attn_states_lse_strided_vec_kernel<DT, kNTLoad, kNTStore, B><<<dim3((uint32_t)li.grid), dim3(B), 0, stream>>>(
                    static_cast<u32x4*>(v_out), lse_out, static_cast<const u32x4*>(v_a), lse_a,
                    static_cast<const u32x4*>(v_b), lse_b, vs, (uint32_t)(pairs * dvec), dvec, make_fastdiv(dvec),
                    make_fastdiv((uint32_t)num_heads), (uint32_t)num_heads, li.log2_xcd_chunk);
            });
        }
    });
    return after_launch();
}

astra_status_t astra_device_memory_info(int device, int* memory_clock_khz, int* memory_bus_bits)
{
    if (!memory_clock_khz || !memory_bus_bits) return ASTRA_ERR_NULL;
    if (hipDeviceGetAttribute(memory_clock_khz, hipDeviceAttributeMemoryClockRate, device) != hipSuccess ||
        hipDeviceGetAttribute(memory_bus_bits, hipDeviceAttributeMemoryBusWidth, device) != hipSuccess) {
        (void)hipGetLastError();  // leave no sticky error behind for the next call
        return ASTRA_ERR_LAUNCH;
    }
    return ASTRA_OK;
}

astra_status_t astra_stream_copy(void* dst, const void* src, int64_t nbytes, hipStream_t stream)
{
    if (!dst || !src) return ASTRA_ERR_NULL;
    if (nbytes < 0 || nbytes % 16 != 0 || nbytes / 16 > kMaxVecIndex) return ASTRA_ERR_SHAPE;
    if (!aligned(dst, 16) || !aligned(src, 16)) return ASTRA_ERR_ALIGN;
    if (overlaps(dst, nbytes, src, nbytes)) return ASTRA_ERR_ALIAS;
    if (nbytes == 0) return ASTRA_OK;
    const int64_t nvec = nbytes / 16;
    const int64_t span = 256 * kCopyUnroll;
    const int64_t blocks = (nvec + span - 1) / span;
    const int lc = fit_chunk_log2(blocks, kFlatChunkLog2, kFlatChunkMinBlocks);
    stream_copy_kernel<kCopyUnroll, kNTLoad, kNTStore><<<dim3((uint32_t)pad_grid(blocks, lc)), dim3(256), 0, stream>>>(
        static_cast<u32x4*>(dst), static_cast<const u32x4*>(src), (uint32_t)nvec, lc);
    return after_launch();
}

astra_status_t astra_stream_probe(void* a, void* b, void* c, int64_t nbytes, astra_probe_t mode, hipStream_t stream)
{
    const int m = (int)mode;
    if (m < ASTRA_PROBE_COPY || m > ASTRA_PROBE_UPDATE2) return ASTRA_ERR_SHAPE;
    const bool use_a = (m != ASTRA_PROBE_WRITE1), use_b = (m == ASTRA_PROBE_READ2 || m == ASTRA_PROBE_READ2_WRITE1 || m == ASTRA_PROBE_UPDATE2);
    const bool use_c = (m == ASTRA_PROBE_COPY || m == ASTRA_PROBE_WRITE1 || m == ASTRA_PROBE_READ2_WRITE1);
    if ((use_a && !a) || (use_b && !b) || (use_c && !c)) return ASTRA_ERR_NULL;
    if (nbytes < 0 || nbytes % 16 != 0 || nbytes / 16 > kMaxVecIndex) return ASTRA_ERR_SHAPE;
    if ((use_a && !aligned(a, 16)) || (use_b && !aligned(b, 16)) || (use_c && !aligned(c, 16))) return ASTRA_ERR_ALIGN;
    if ((use_a && use_b && overlaps(a, nbytes, b, nbytes)) || (use_a && use_c && overlaps(a, nbytes, c, nbytes)) ||
        (use_b && use_c && overlaps(b, nbytes, c, nbytes)))
        return ASTRA_ERR_ALIAS;
    if (nbytes == 0) return ASTRA_OK;
    const int64_t nvec = nbytes / 16;
    // the operators' geometry, except for the write-only mode on streaming grids: one 1 KiB store per single-wave
    // workgroup runs at the rate the chip starts workgroups (4.7 per ns on MI355X: 58 % of the HBM peak), which says
    // nothing about memory, so that mode keeps four waves per workgroup (83-84 %)
    const int block = (m == ASTRA_PROBE_WRITE1 && flat_block(nvec) == 64) ? 256 : flat_block(nvec);
    const int64_t blocks = (nvec + block - 1) / block;
    const int lc = fit_chunk_log2(blocks, kFlatChunkLog2, kFlatChunkMinBlocks * (256 / block));
    const dim3 grid((uint32_t)pad_grid(blocks, lc));
    u32x4* const pa = static_cast<u32x4*>(a);
    u32x4* const pb = static_cast<u32x4*>(b);
    u32x4* const pc = static_cast<u32x4*>(c);
    for_flat_block(block, [&](auto bc) {
        constexpr int B = decltype(bc)::value;
        switch (m) {
            case ASTRA_PROBE_COPY: stream_probe_kernel<0, B><<<grid, dim3(B), 0, stream>>>(pa, pb, pc, (uint32_t)nvec, lc); break;
            case ASTRA_PROBE_READ2: stream_probe_kernel<1, B><<<grid, dim3(B), 0, stream>>>(pa, pb, pc, (uint32_t)nvec, lc); break;
            case ASTRA_PROBE_WRITE1: stream_probe_kernel<2, B><<<grid, dim3(B), 0, stream>>>(pa, pb, pc, (uint32_t)nvec, lc); break;
            case ASTRA_PROBE_READ2_WRITE1: stream_probe_kernel<3, B><<<grid, dim3(B), 0, stream>>>(pa, pb, pc, (uint32_t)nvec, lc); break;
            default: stream_probe_kernel<4, B><<<grid, dim3(B), 0, stream>>>(pa, pb, pc, (uint32_t)nvec, lc); break;
        }
    });
    return after_launch();
}

}  // extern "C"
