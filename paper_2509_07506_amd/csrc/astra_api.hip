// C ABI of the astra library: argument validation, dispatch (shape x alignment -> kernel variant and
// launch geometry) and the kernel launches.  Everything before the first HIP call is plain host
// arithmetic, so every error path can be exercised without a GPU.
#include "astra.h"
#include "astra_plan.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <limits>

#include "fused_add_rmsnorm_kernels.h"
#include "merge_attn_states_lse_kernels.h"
#include "silu_and_mul_kernels.h"
#include "stream_copy_kernel.h"

namespace {

using namespace astra;

// ---- tuning constants (measured on MI355X) ------------------------------------------------------
constexpr bool kStreamNT = true;   // non-temporal hint on the once-touched activation streams
constexpr int kSiluUnroll = 2;     // vector pairs in flight per lane, silu_and_mul
constexpr int kMergeUnroll = 2;    // vector pairs in flight per lane, merge
constexpr int kCopyUnroll = 4;

constexpr int64_t kMaxVecIndex = int64_t(1) << 31;  // 32-bit vector indices with head-room for the tail
constexpr int64_t kMaxGenericGrid = int64_t(1) << 20;
constexpr int64_t kMaxRowGrid = (int64_t(1) << 22) - 1;  // grid * 1024 work-items stays below 2^32
constexpr int kNumCUs = 256;

bool mul_overflows(int64_t a, int64_t b, int64_t* out) { return __builtin_mul_overflow(a, b, out); }

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// half-open byte ranges [p, p+n) and [q, q+m)
bool overlaps(const void* p, int64_t n, const void* q, int64_t m)
{
    const uintptr_t a = reinterpret_cast<uintptr_t>(p), b = reinterpret_cast<uintptr_t>(q);
    return n > 0 && m > 0 && a < b + (uintptr_t)m && b < a + (uintptr_t)n;
}

bool valid_dtype(int dt) { return dt == ASTRA_F16 || dt == ASTRA_BF16; }

astra_status_t after_launch() { return hipGetLastError() == hipSuccess ? ASTRA_OK : ASTRA_ERR_LAUNCH; }

int round_up(int v, int m) { return (v + m - 1) / m * m; }

// ---- fused_add_rmsnorm plan -----------------------------------------------------------------------
// The row lives in registers: hv = H/8 vectors spread over `block` lanes, `vpt` per lane.
// Few rows (decode): as many lanes per row as possible, so each lane has one dependent load-reduce-store
// chain and the row's bytes are requested at once.  Many rows (prefill): about four waves per row, so
// several rows share a CU and the cross-wave step stays short.
struct RowPlan {
    int vpt;
    int block;
};

bool rmsnorm_row_plan(int64_t T, int64_t hv, RowPlan* plan)
{
    static const int kVpt[4] = {1, 2, 4, 8};
    static const int kMaxBlock[4] = {1024, 1024, 1024, 512};
    const bool few_rows = T < 2 * kNumCUs;
    int best = -1, best_block = 0;
    double best_cost = 0.0;
    for (int i = 0; i < 4; ++i) {
        const int64_t need = (hv + kVpt[i] - 1) / kVpt[i];
        if (need > kMaxBlock[i]) continue;
        const int block = round_up((int)need, kWave);
        const double waste = double(block) * kVpt[i] / double(hv) - 1.0;  // idle lane-slots
        double cost;
        if (few_rows) cost = kVpt[i] + waste;                             // smallest vpt that fits
        else cost = waste * 4.0 + std::fabs(std::log2(double(block) / 256.0));
        if (best < 0 || cost < best_cost) {
            best = i;
            best_cost = cost;
            best_block = block;
        }
    }
    if (best < 0) return false;
    plan->vpt = kVpt[best];
    plan->block = best_block;
    return true;
}

astra_status_t plan_rmsnorm(int64_t T, int64_t H, bool aligned16, astra_launch_info_t* info)
{
    int64_t n;
    if (T < 0 || H <= 0 || mul_overflows(T, H, &n) || n > std::numeric_limits<int64_t>::max() / 2) return ASTRA_ERR_SHAPE;
    *info = astra_launch_info_t{ASTRA_PATH_NONE, 0, 0, 0, 0};
    if (T == 0) return ASTRA_OK;
    RowPlan rp;
    if (aligned16 && H % kVecElems == 0 && rmsnorm_row_plan(T, H / kVecElems, &rp)) {
        *info = astra_launch_info_t{ASTRA_PATH_VECTOR, rp.block, rp.vpt, 0, T < kMaxRowGrid ? T : kMaxRowGrid};
    } else {
        *info = astra_launch_info_t{ASTRA_PATH_GENERIC, 256, 0, 0, T < kMaxGenericGrid ? T : kMaxGenericGrid};
    }
    return ASTRA_OK;
}

astra_status_t plan_silu(int64_t T, int64_t d, bool aligned16, astra_launch_info_t* info)
{
    int64_t two_d, n;
    if (T < 0 || d <= 0 || mul_overflows(d, 2, &two_d) || mul_overflows(T, two_d, &n) ||
        n > std::numeric_limits<int64_t>::max() / 2)
        return ASTRA_ERR_SHAPE;
    *info = astra_launch_info_t{ASTRA_PATH_NONE, 0, 0, 0, 0};
    if (T == 0) return ASTRA_OK;
    const int64_t dv = d / kVecElems;
    // the input holds 2*T*dv vectors and is indexed with 32 bits
    if (aligned16 && d % kVecElems == 0 && dv >= 32 && 2 * T * dv <= kMaxVecIndex) {
        const int64_t span = 256 * kSiluUnroll;
        *info = astra_launch_info_t{ASTRA_PATH_VECTOR, 256, kSiluUnroll, 0, (T * dv + span - 1) / span};
    } else {
        *info = astra_launch_info_t{ASTRA_PATH_GENERIC, 256, 0, 0, T < kMaxGenericGrid ? T : kMaxGenericGrid};
    }
    return ASTRA_OK;
}

astra_status_t plan_merge(int64_t T, int64_t NH, int64_t D, bool aligned16, astra_launch_info_t* info)
{
    int64_t pairs, n;
    if (T < 0 || NH <= 0 || D <= 0 || mul_overflows(T, NH, &pairs) || mul_overflows(pairs, D, &n) ||
        n > std::numeric_limits<int64_t>::max() / 4)
        return ASTRA_ERR_SHAPE;
    *info = astra_launch_info_t{ASTRA_PATH_NONE, 0, 0, 0, 0};
    if (T == 0) return ASTRA_OK;
    const int64_t dvec = D / kVecElems;
    if (aligned16 && D % kVecElems == 0 && pairs * dvec <= kMaxVecIndex) {
        const int64_t span = 256 * kMergeUnroll;
        *info = astra_launch_info_t{ASTRA_PATH_VECTOR, 256, kMergeUnroll, 0, (pairs * dvec + span - 1) / span};
    } else {
        *info = astra_launch_info_t{ASTRA_PATH_GENERIC, 256, 0, 0, pairs < kMaxGenericGrid ? pairs : kMaxGenericGrid};
    }
    return ASTRA_OK;
}

// ---- launches ---------------------------------------------------------------------------------------

template <int DT, int VPT, int MAXT>
void launch_rmsnorm_row(const astra_launch_info_t& li, void* input, void* residual, const void* weight, int64_t T,
                        int64_t H, float eps, hipStream_t stream)
{
    fused_add_rmsnorm_row_kernel<DT, VPT, MAXT, kStreamNT><<<dim3((uint32_t)li.grid), dim3(li.block), 0, stream>>>(
        static_cast<u32x4*>(input), static_cast<u32x4*>(residual), static_cast<const u32x4*>(weight), T,
        (uint32_t)(H / kVecElems), 1.0f / (float)H, eps);
}

template <int DT>
void launch_rmsnorm(const astra_launch_info_t& li, void* input, void* residual, const void* weight, int64_t T, int64_t H,
                    float eps, hipStream_t stream)
{
    if (li.path == ASTRA_PATH_GENERIC) {
        fused_add_rmsnorm_generic_kernel<DT><<<dim3((uint32_t)li.grid), dim3(li.block), 0, stream>>>(
            static_cast<uint16_t*>(input), static_cast<uint16_t*>(residual), static_cast<const uint16_t*>(weight), T, H,
            1.0f / (float)H, eps);
        return;
    }
    switch (li.vectors_per_lane) {
        case 1: launch_rmsnorm_row<DT, 1, 1024>(li, input, residual, weight, T, H, eps, stream); break;
        case 2: launch_rmsnorm_row<DT, 2, 1024>(li, input, residual, weight, T, H, eps, stream); break;
        case 4: launch_rmsnorm_row<DT, 4, 1024>(li, input, residual, weight, T, H, eps, stream); break;
        default: launch_rmsnorm_row<DT, 8, 512>(li, input, residual, weight, T, H, eps, stream); break;
    }
}

template <int DT>
void launch_silu(const astra_launch_info_t& li, void* out, const void* in, int64_t T, int64_t d, hipStream_t stream)
{
    if (li.path == ASTRA_PATH_GENERIC) {
        silu_and_mul_generic_kernel<DT><<<dim3((uint32_t)li.grid), dim3(li.block), 0, stream>>>(
            static_cast<uint16_t*>(out), static_cast<const uint16_t*>(in), T, d);
        return;
    }
    const uint32_t dv = (uint32_t)(d / kVecElems);
    silu_and_mul_vec_kernel<DT, kSiluUnroll, kStreamNT><<<dim3((uint32_t)li.grid), dim3(256), 0, stream>>>(
        static_cast<u32x4*>(out), static_cast<const u32x4*>(in), (uint32_t)(T * dv), dv, make_fastdiv(dv));
}

template <int DT>
void launch_merge(const astra_launch_info_t& li, void* v_out, float* lse_out, const void* v_a, const float* lse_a,
                  const void* v_b, const float* lse_b, int64_t pairs, int64_t D, hipStream_t stream)
{
    if (li.path == ASTRA_PATH_GENERIC) {
        merge_attn_states_lse_generic_kernel<DT><<<dim3((uint32_t)li.grid), dim3(li.block), 0, stream>>>(
            static_cast<uint16_t*>(v_out), lse_out, static_cast<const uint16_t*>(v_a), lse_a,
            static_cast<const uint16_t*>(v_b), lse_b, pairs, D);
        return;
    }
    const uint32_t dvec = (uint32_t)(D / kVecElems);
    int log2_dvec = -1;
    if ((dvec & (dvec - 1)) == 0) log2_dvec = __builtin_ctz(dvec);
    merge_attn_states_lse_vec_kernel<DT, kMergeUnroll, kStreamNT><<<dim3((uint32_t)li.grid), dim3(256), 0, stream>>>(
        static_cast<u32x4*>(v_out), lse_out, static_cast<const u32x4*>(v_a), lse_a, static_cast<const u32x4*>(v_b), lse_b,
        (uint32_t)(pairs * dvec), dvec, log2_dvec, make_fastdiv(dvec));
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
    }
    return "unknown status";
}

astra_status_t astra_plan_fused_add_rmsnorm(int64_t T, int64_t H, int aligned16, astra_launch_info_t* info)
{
    if (!info) return ASTRA_ERR_NULL;
    return plan_rmsnorm(T, H, aligned16 != 0, info);
}

astra_status_t astra_plan_silu_and_mul(int64_t T, int64_t d, int aligned16, astra_launch_info_t* info)
{
    if (!info) return ASTRA_ERR_NULL;
    return plan_silu(T, d, aligned16 != 0, info);
}

astra_status_t astra_plan_merge_attn_states_lse(int64_t T, int64_t num_heads, int64_t head_dim, int aligned16,
                                                astra_launch_info_t* info)
{
    if (!info) return ASTRA_ERR_NULL;
    return plan_merge(T, num_heads, head_dim, aligned16 != 0, info);
}

astra_status_t astra_fused_add_rmsnorm(void* input, void* residual, const void* weight, int64_t T, int64_t H,
                                       astra_dtype_t dtype, float eps, hipStream_t stream)
{
    if (!input || !residual || !weight) return ASTRA_ERR_NULL;
    astra_launch_info_t li;
    const bool a16 = aligned(input, 16) && aligned(residual, 16) && aligned(weight, 16);
    astra_status_t st = plan_rmsnorm(T, H, a16, &li);
    if (st != ASTRA_OK) return st;
    if (!valid_dtype((int)dtype)) return ASTRA_ERR_DTYPE;
    if (!(eps >= 0.0f)) return ASTRA_ERR_EPS;
    if (!aligned(input, 2) || !aligned(residual, 2) || !aligned(weight, 2)) return ASTRA_ERR_ALIGN;
    const int64_t bytes = T * H * 2;
    if (overlaps(input, bytes, residual, bytes) || overlaps(input, bytes, weight, H * 2) ||
        overlaps(residual, bytes, weight, H * 2))
        return ASTRA_ERR_ALIAS;
    if (T == 0) return ASTRA_OK;
    if (dtype == ASTRA_BF16) launch_rmsnorm<kBF16>(li, input, residual, weight, T, H, eps, stream);
    else launch_rmsnorm<kF16>(li, input, residual, weight, T, H, eps, stream);
    return after_launch();
}

astra_status_t astra_silu_and_mul(void* out, const void* input, int64_t T, int64_t d, astra_dtype_t dtype,
                                  hipStream_t stream)
{
    if (!out || !input) return ASTRA_ERR_NULL;
    astra_launch_info_t li;
    astra_status_t st = plan_silu(T, d, aligned(out, 16) && aligned(input, 16), &li);
    if (st != ASTRA_OK) return st;
    if (!valid_dtype((int)dtype)) return ASTRA_ERR_DTYPE;
    if (!aligned(out, 2) || !aligned(input, 2)) return ASTRA_ERR_ALIGN;
    if (overlaps(out, T * d * 2, input, T * d * 4)) return ASTRA_ERR_ALIAS;
    if (T == 0) return ASTRA_OK;
    if (dtype == ASTRA_BF16) launch_silu<kBF16>(li, out, input, T, d, stream);
    else launch_silu<kF16>(li, out, input, T, d, stream);
    return after_launch();
}

astra_status_t astra_merge_attn_states_lse(void* v_out, float* lse_out, const void* v_a, const float* lse_a,
                                           const void* v_b, const float* lse_b, int64_t T, int64_t num_heads,
                                           int64_t head_dim, astra_dtype_t dtype, hipStream_t stream)
{
    if (!v_out || !lse_out || !v_a || !lse_a || !v_b || !lse_b) return ASTRA_ERR_NULL;
    astra_launch_info_t li;
    astra_status_t st =
        plan_merge(T, num_heads, head_dim, aligned(v_out, 16) && aligned(v_a, 16) && aligned(v_b, 16), &li);
    if (st != ASTRA_OK) return st;
    if (!valid_dtype((int)dtype)) return ASTRA_ERR_DTYPE;
    if (!aligned(v_out, 2) || !aligned(v_a, 2) || !aligned(v_b, 2) || !aligned(lse_out, 4) || !aligned(lse_a, 4) ||
        !aligned(lse_b, 4))
        return ASTRA_ERR_ALIGN;
    const int64_t pairs = T * num_heads;
    const int64_t vbytes = pairs * head_dim * 2, sbytes = pairs * 4;
    if ((v_out != v_a && overlaps(v_out, vbytes, v_a, vbytes)) || (v_out != v_b && overlaps(v_out, vbytes, v_b, vbytes)) ||
        overlaps(lse_out, sbytes, lse_a, sbytes) || overlaps(lse_out, sbytes, lse_b, sbytes) ||
        overlaps(v_out, vbytes, lse_a, sbytes) || overlaps(v_out, vbytes, lse_b, sbytes) ||
        overlaps(lse_out, sbytes, v_a, vbytes) || overlaps(lse_out, sbytes, v_b, vbytes) ||
        overlaps(lse_out, sbytes, v_out, vbytes))
        return ASTRA_ERR_ALIAS;
    if (T == 0) return ASTRA_OK;
    if (dtype == ASTRA_BF16) launch_merge<kBF16>(li, v_out, lse_out, v_a, lse_a, v_b, lse_b, pairs, head_dim, stream);
    else launch_merge<kF16>(li, v_out, lse_out, v_a, lse_a, v_b, lse_b, pairs, head_dim, stream);
    return after_launch();
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
    stream_copy_kernel<kCopyUnroll, kStreamNT><<<dim3((uint32_t)((nvec + span - 1) / span)), dim3(256), 0, stream>>>(
        static_cast<u32x4*>(dst), static_cast<const u32x4*>(src), (uint32_t)nvec);
    return after_launch();
}

}  // extern "C"
