// Stand-alone check of the C ABI from a plain C++ host program: no Python, no PyTorch.  Device memory and the
// stream come from the HIP runtime directly (hipMalloc / hipStreamCreate), the operators from libastra_hip.so,
// the expectations from the CPU oracle library (test infrastructure).  Bars as everywhere: residual of
// fused_add_rmsnorm bit-exact; other 16-bit outputs within rtol 1.6e-2 / atol 1e-2 (bf16), 2e-3 / 1e-3 (fp16);
// binary32 storage within 2e-5 / 1e-6; lse within 1e-4.
//
// Build (done by __graft_entry__.build()):
//   hipcc -O2 -std=c++17 -I include tests/c_abi/check_abi.cpp -o tests/c_abi/check_abi
//         -L paper_2509_07506_amd -lastra_hip -L oracle -loracle -Wl,-rpath,... (both directories)
// Exit status 0 and a final line "c_abi: all checks passed" on success.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "astra.h"
#include "astra_kway.h"
#include "astra_plan.h"
#include "astra_strided.h"

extern "C" {
// oracle/astra_oracle.c
float oracle_bf16_to_f32(uint16_t h);
float oracle_f16_to_f32(uint16_t h);
uint16_t oracle_f32_to_bf16(float f);
uint16_t oracle_f32_to_f16(float f);
void oracle_fused_add_rmsnorm(uint16_t* input, uint16_t* residual, const uint16_t* weight, int64_t T, int64_t H, int dtype,
                              float eps);
void oracle_fused_add_rmsnorm_f32(const float* x, const float* r, const float* w, int64_t T, int64_t H, float eps,
                                  float* s_out, float* y_out);
void oracle_silu_and_mul(uint16_t* out, const uint16_t* in, int64_t T, int64_t d, int dtype);
void oracle_silu_and_mul_f32(float* out, const float* in, int64_t T, int64_t d);
void oracle_merge_attn_states_lse(uint16_t* v_out, float* lse_out, const uint16_t* v_a, const float* lse_a,
                                  const uint16_t* v_b, const float* lse_b, int64_t T, int64_t NH, int64_t D, int dtype);
void oracle_merge_attn_states_lse_f32(float* v_out, float* lse_out, const float* v_a, const float* lse_a, const float* v_b,
                                      const float* lse_b, int64_t T, int64_t NH, int64_t D);
void oracle_merge_attn_states_lse_kway(uint16_t* v_out, float* lse_out, const uint16_t* v_parts, const float* lse_parts,
                                       int64_t K, int64_t P, int64_t D, int dtype);
}

namespace {

int g_failures = 0;

#define HIP_OK(call)                                                                                 \
    do {                                                                                             \
        hipError_t e_ = (call);                                                                      \
        if (e_ != hipSuccess) {                                                                      \
            std::fprintf(stderr, "c_abi: %s failed: %s\n", #call, hipGetErrorString(e_));            \
            std::exit(2);                                                                            \
        }                                                                                            \
    } while (0)

void expect(bool ok, const char* what)
{
    if (!ok) {
        ++g_failures;
        std::printf("c_abi: FAILED %s\n", what);
    }
    std::fflush(stdout);
}

// splitmix64 -> roughly normal values (sum of four uniforms, variance 1)
struct Rng {
    uint64_t s;
    uint64_t next()
    {
        uint64_t z = (s += 0x9E3779B97F4A7C15ull);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    float uniform() { return (float)(next() >> 40) * (1.0f / 16777216.0f); }
    float normalish() { return (uniform() + uniform() + uniform() + uniform() - 2.0f) * 1.7320508f; }
};

float widen(uint16_t h, int dt) { return dt == ASTRA_BF16 ? oracle_bf16_to_f32(h) : oracle_f16_to_f32(h); }
uint16_t narrow(float f, int dt) { return dt == ASTRA_BF16 ? oracle_f32_to_bf16(f) : oracle_f32_to_f16(f); }

struct Tol {
    double rtol, atol;
};
Tol tol_of(int dt) { return dt == ASTRA_BF16 ? Tol{1.6e-2, 1e-2} : dt == ASTRA_F16 ? Tol{2e-3, 1e-3} : Tol{2e-5, 1e-6}; }

bool close(double got, double ref, Tol t)
{
    if (std::isnan(got) || std::isnan(ref)) return std::isnan(got) && std::isnan(ref);
    if (std::isinf(got) || std::isinf(ref)) return got == ref;
    return std::fabs(got - ref) <= t.atol + t.rtol * std::fabs(ref);
}

template <class E>
double value_of(E e, int dt);
template <>
double value_of<uint16_t>(uint16_t e, int dt) { return widen(e, dt); }
template <>
double value_of<float>(float e, int) { return e; }

template <class E>
size_t count_far(const std::vector<E>& got, const std::vector<E>& ref, int dt)
{
    size_t bad = 0;
    for (size_t i = 0; i < got.size(); ++i)
        if (std::memcmp(&got[i], &ref[i], sizeof(E)) != 0 && !close(value_of(got[i], dt), value_of(ref[i], dt), tol_of(dt))) ++bad;
    return bad;
}

size_t count_far_lse(const std::vector<float>& got, const std::vector<float>& ref)
{
    size_t bad = 0;
    for (size_t i = 0; i < got.size(); ++i)
        if (!close(got[i], ref[i], Tol{0.0, 1e-4})) ++bad;
    return bad;
}

template <class E>
E make_elem(float f, int dt);
template <>
uint16_t make_elem<uint16_t>(float f, int dt) { return narrow(f, dt); }
template <>
float make_elem<float>(float f, int) { return f; }

template <class E>
struct DevBuf {
    E* p = nullptr;
    size_t n = 0;
    explicit DevBuf(size_t n_) : n(n_) { HIP_OK(hipMalloc((void**)&p, (n ? n : 1) * sizeof(E))); }
    ~DevBuf() { (void)hipFree(p); }
    void upload(const std::vector<E>& h, hipStream_t s) { HIP_OK(hipMemcpyAsync(p, h.data(), n * sizeof(E), hipMemcpyHostToDevice, s)); }
    std::vector<E> download(hipStream_t s)
    {
        std::vector<E> h(n);
        HIP_OK(hipMemcpyAsync(h.data(), p, n * sizeof(E), hipMemcpyDeviceToHost, s));
        HIP_OK(hipStreamSynchronize(s));
        return h;
    }
};

template <class E>
void check_rmsnorm(int dt, int64_t T, int64_t H, float eps, hipStream_t s)
{
    Rng g{uint64_t(1000 + dt * 97 + T * 31 + H)};
    std::vector<E> x(T * H), r(T * H), w(H);
    for (auto& v : x) v = make_elem<E>(g.normalish(), dt);
    for (auto& v : r) v = make_elem<E>(2.0f * g.normalish(), dt);
    for (auto& v : w) v = make_elem<E>(1.0f + 0.3f * g.normalish(), dt);
    DevBuf<E> dx(x.size()), dr(r.size()), dw(w.size());
    dx.upload(x, s);
    dr.upload(r, s);
    dw.upload(w, s);
    astra_status_t st = astra_fused_add_rmsnorm(dx.p, dr.p, dw.p, T, H, (astra_dtype_t)dt, eps, s);
    std::vector<E> y = dx.download(s), res = dr.download(s);
    std::vector<E> y_ref, res_ref;
    if constexpr (sizeof(E) == 2) {
        y_ref = x;
        res_ref = r;
        oracle_fused_add_rmsnorm((uint16_t*)y_ref.data(), (uint16_t*)res_ref.data(), (const uint16_t*)w.data(), T, H, dt, eps);
    } else {
        y_ref.resize(x.size());
        res_ref.resize(x.size());
        oracle_fused_add_rmsnorm_f32((const float*)x.data(), (const float*)r.data(), (const float*)w.data(), T, H, eps,
                                     (float*)res_ref.data(), (float*)y_ref.data());
    }
    char what[160];
    std::snprintf(what, sizeof what, "fused_add_rmsnorm dtype=%d T=%lld H=%lld", dt, (long long)T, (long long)H);
    const bool ok = st == ASTRA_OK && std::memcmp(res.data(), res_ref.data(), res.size() * sizeof(E)) == 0 &&
                    count_far(y, y_ref, dt) == 0;
    expect(ok, what);
    if (ok) std::printf("c_abi: ok %s (residual bit-exact)\n", what);
}

template <class E>
void check_silu(int dt, int64_t T, int64_t d, hipStream_t s)
{
    Rng g{uint64_t(2000 + dt * 97 + T * 31 + d)};
    std::vector<E> in(T * 2 * d);
    for (auto& v : in) {
        float f = g.normalish();
        if (g.uniform() < 1e-3f) f *= 20.0f;
        v = make_elem<E>(f, dt);
    }
    DevBuf<E> din(in.size()), dout(T * d);
    din.upload(in, s);
    astra_status_t st = astra_silu_and_mul(dout.p, din.p, T, d, (astra_dtype_t)dt, s);
    std::vector<E> out = dout.download(s), ref(T * d);
    if constexpr (sizeof(E) == 2) oracle_silu_and_mul((uint16_t*)ref.data(), (const uint16_t*)in.data(), T, d, dt);
    else oracle_silu_and_mul_f32((float*)ref.data(), (const float*)in.data(), T, d);
    char what[160];
    std::snprintf(what, sizeof what, "silu_and_mul dtype=%d T=%lld d=%lld", dt, (long long)T, (long long)d);
    const bool ok = st == ASTRA_OK && count_far(out, ref, dt) == 0;
    expect(ok, what);
    if (ok) std::printf("c_abi: ok %s\n", what);
}

std::vector<float> make_scores(Rng& g, size_t n)
{
    std::vector<float> s(n);
    for (auto& v : s) v = g.uniform() < 0.05f ? -INFINITY : -5.0f + 20.0f * g.uniform();
    return s;
}

template <class E>
void check_merge(int dt, int64_t T, int64_t NH, int64_t D, hipStream_t s)
{
    Rng g{uint64_t(3000 + dt * 97 + T * 31 + NH * 7 + D)};
    const size_t P = T * NH;
    std::vector<E> va(P * D), vb(P * D);
    for (auto& v : va) v = make_elem<E>(g.normalish(), dt);
    for (auto& v : vb) v = make_elem<E>(g.normalish(), dt);
    std::vector<float> la = make_scores(g, P), lb = make_scores(g, P);
    DevBuf<E> dva(va.size()), dvb(vb.size()), dvo(va.size());
    DevBuf<float> dla(P), dlb(P), dlo(P);
    dva.upload(va, s);
    dvb.upload(vb, s);
    dla.upload(la, s);
    dlb.upload(lb, s);
    astra_status_t st = astra_merge_attn_states_lse(dvo.p, dlo.p, dva.p, dla.p, dvb.p, dlb.p, T, NH, D, (astra_dtype_t)dt, s);
    std::vector<E> vo = dvo.download(s), vo_ref(va.size());
    std::vector<float> lo = dlo.download(s), lo_ref(P);
    if constexpr (sizeof(E) == 2)
        oracle_merge_attn_states_lse((uint16_t*)vo_ref.data(), lo_ref.data(), (const uint16_t*)va.data(), la.data(),
                                     (const uint16_t*)vb.data(), lb.data(), T, NH, D, dt);
    else
        oracle_merge_attn_states_lse_f32((float*)vo_ref.data(), lo_ref.data(), (const float*)va.data(), la.data(),
                                         (const float*)vb.data(), lb.data(), T, NH, D);
    char what[160];
    std::snprintf(what, sizeof what, "merge_attn_states_lse dtype=%d T=%lld NH=%lld D=%lld", dt, (long long)T, (long long)NH,
                  (long long)D);
    bool ok = st == ASTRA_OK && count_far(vo, vo_ref, dt) == 0 && count_far_lse(lo, lo_ref) == 0;
    expect(ok, what);
    if (ok) std::printf("c_abi: ok %s\n", what);

    if constexpr (sizeof(E) == 2) {
        // the same two states through the K-way entry point (K = 2, parts stacked)
        std::vector<uint16_t> parts(2 * P * D);
        std::memcpy(parts.data(), va.data(), P * D * 2);
        std::memcpy(parts.data() + P * D, vb.data(), P * D * 2);
        std::vector<float> lparts(2 * P);
        std::memcpy(lparts.data(), la.data(), P * 4);
        std::memcpy(lparts.data() + P, lb.data(), P * 4);
        DevBuf<uint16_t> dparts(parts.size());
        DevBuf<float> dlparts(lparts.size());
        dparts.upload(parts, s);
        dlparts.upload(lparts, s);
        st = astra_merge_attn_states_lse_kway(dvo.p, dlo.p, dparts.p, dlparts.p, 2, T, NH, D, (astra_dtype_t)dt, s);
        std::vector<uint16_t> kv = dvo.download(s), kv_ref(P * D);
        std::vector<float> kl = dlo.download(s), kl_ref(P);
        oracle_merge_attn_states_lse_kway(kv_ref.data(), kl_ref.data(), parts.data(), lparts.data(), 2, (int64_t)P, D, dt);
        std::snprintf(what, sizeof what, "merge_attn_states_lse_kway K=2 dtype=%d T=%lld NH=%lld D=%lld", dt, (long long)T,
                      (long long)NH, (long long)D);
        ok = st == ASTRA_OK && count_far(kv, kv_ref, dt) == 0 && count_far_lse(kl, kl_ref) == 0;
        expect(ok, what);
        if (ok) std::printf("c_abi: ok %s\n", what);
    }
}

// the strided entry points on padded views (rows / heads further apart than their length), 16-bit storage
void check_strided(int dt, hipStream_t s)
{
    // silu_and_mul: T rows of 2d, input row stride 2d + 16, output row stride d + 8
    {
        const int64_t T = 37, d = 1408, is = 2 * d + 16, os = d + 8;
        Rng g{uint64_t(4000 + dt)};
        std::vector<uint16_t> dense(T * 2 * d), in(T * is, narrow(7.0f, dt));
        for (auto& v : dense) v = narrow(g.normalish(), dt);
        for (int64_t t = 0; t < T; ++t) std::memcpy(&in[t * is], &dense[t * 2 * d], 2 * d * 2);
        DevBuf<uint16_t> din(in.size()), dout(T * os);
        std::vector<uint16_t> out_init(T * os, narrow(9.0f, dt));
        din.upload(in, s);
        dout.upload(out_init, s);
        astra_status_t st = astra_silu_and_mul_strided(dout.p, os, din.p, is, T, d, (astra_dtype_t)dt, s);
        std::vector<uint16_t> out = dout.download(s), ref(T * d), got(T * d);
        oracle_silu_and_mul(ref.data(), dense.data(), T, d, dt);
        bool gaps = true;
        for (int64_t t = 0; t < T; ++t) {
            std::memcpy(&got[t * d], &out[t * os], d * 2);
            for (int64_t j = d; j < os; ++j) gaps = gaps && out[t * os + j] == narrow(9.0f, dt);
        }
        char what[120];
        std::snprintf(what, sizeof what, "silu_and_mul_strided dtype=%d", dt);
        const bool ok = st == ASTRA_OK && gaps && count_far(got, ref, dt) == 0;
        expect(ok, what);
        if (ok) std::printf("c_abi: ok %s (gaps untouched)\n", what);
    }
    // merge: heads of 128 values inside 192-wide head slots for v_a, dense v_b, 136-wide slots for the output
    {
        const int64_t T = 21, NH = 8, D = 128, ha = 192, ho = 136;
        const size_t P = T * NH;
        Rng g{uint64_t(5000 + dt)};
        std::vector<uint16_t> va(P * D), vb(P * D), wa(P * ha, narrow(7.0f, dt));
        for (auto& v : va) v = narrow(g.normalish(), dt);
        for (auto& v : vb) v = narrow(g.normalish(), dt);
        for (size_t p = 0; p < P; ++p) std::memcpy(&wa[p * ha], &va[p * D], D * 2);
        std::vector<float> la = make_scores(g, P), lb = make_scores(g, P);
        DevBuf<uint16_t> dwa(wa.size()), dvb(vb.size()), dvo(P * ho);
        DevBuf<float> dla(P), dlb(P), dlo(P);
        std::vector<uint16_t> out_init(P * ho, narrow(9.0f, dt));
        dwa.upload(wa, s);
        dvb.upload(vb, s);
        dvo.upload(out_init, s);
        dla.upload(la, s);
        dlb.upload(lb, s);
        astra_status_t st = astra_merge_attn_states_lse_strided(dvo.p, NH * ho, ho, dlo.p, dwa.p, NH * ha, ha, dla.p, dvb.p, NH * D,
                                                                D, dlb.p, T, NH, D, (astra_dtype_t)dt, s);
        std::vector<uint16_t> out = dvo.download(s), got(P * D), ref(P * D);
        std::vector<float> lo = dlo.download(s), lo_ref(P);
        oracle_merge_attn_states_lse(ref.data(), lo_ref.data(), va.data(), la.data(), vb.data(), lb.data(), T, NH, D, dt);
        bool gaps = true;
        for (size_t p = 0; p < P; ++p) {
            std::memcpy(&got[p * D], &out[p * ho], D * 2);
            for (int64_t j = D; j < ho; ++j) gaps = gaps && out[p * ho + j] == narrow(9.0f, dt);
        }
        char what[120];
        std::snprintf(what, sizeof what, "merge_attn_states_lse_strided dtype=%d", dt);
        const bool ok = st == ASTRA_OK && gaps && count_far(got, ref, dt) == 0 && count_far_lse(lo, lo_ref) == 0;
        expect(ok, what);
        if (ok) std::printf("c_abi: ok %s (gaps untouched)\n", what);
    }
    // fused_add_rmsnorm out of place on dense views equals the in-place oracle
    {
        const int64_t T = 19, H = 4096;
        Rng g{uint64_t(6000 + dt)};
        std::vector<uint16_t> x(T * H), r(T * H), w(H);
        for (auto& v : x) v = narrow(g.normalish(), dt);
        for (auto& v : r) v = narrow(2.0f * g.normalish(), dt);
        for (auto& v : w) v = narrow(1.0f + 0.3f * g.normalish(), dt);
        DevBuf<uint16_t> dx(x.size()), dr(r.size()), dw(w.size()), dy(x.size()), dro(r.size());
        dx.upload(x, s);
        dr.upload(r, s);
        dw.upload(w, s);
        astra_status_t st = astra_fused_add_rmsnorm_strided(dy.p, H, dro.p, H, dx.p, H, dr.p, H, dw.p, T, H, (astra_dtype_t)dt, 1e-6f, s);
        std::vector<uint16_t> y = dy.download(s), res = dro.download(s), x_after = dx.download(s), y_ref = x, res_ref = r;
        oracle_fused_add_rmsnorm(y_ref.data(), res_ref.data(), w.data(), T, H, dt, 1e-6f);
        char what[120];
        std::snprintf(what, sizeof what, "fused_add_rmsnorm_strided dtype=%d", dt);
        const bool ok = st == ASTRA_OK && res == res_ref && x_after == x && count_far(y, y_ref, dt) == 0;
        expect(ok, what);
        if (ok) std::printf("c_abi: ok %s (inputs untouched, residual bit-exact)\n", what);
    }
}

void check_host_queries()
{
    astra_launch_info_t li;
    expect(astra_plan_fused_add_rmsnorm(32768, 8192, ASTRA_BF16, 1, &li) == ASTRA_OK && li.path == ASTRA_PATH_VECTOR &&
               li.block == 1024 && li.grid == 32768,
           "plan of the headline rmsnorm shape");
    expect(astra_plan_silu_and_mul(3, 100, ASTRA_F16, 1, &li) == ASTRA_OK && li.path == ASTRA_PATH_PHASED, "plan of an odd silu shape");
    expect(astra_plan_silu_and_mul(3, 5, ASTRA_F16, 1, &li) == ASTRA_OK && li.path == ASTRA_PATH_RAGGED, "plan of a silu shape with short rows");
    expect(astra_plan_merge_attn_states_lse(0, 4, 64, ASTRA_F16, 1, &li) == ASTRA_OK && li.path == ASTRA_PATH_NONE, "plan of an empty merge");
    int clk = 0, bits = 0;
    expect(astra_device_memory_info(0, &clk, &bits) == ASTRA_OK && clk > 0 && bits > 0, "device memory info");
    std::printf("c_abi: ok host queries (memory clock %d kHz, bus %d bits)\n", clk, bits);
}

void check_errors(hipStream_t s)
{
    DevBuf<uint16_t> a(4096), b(4096), c(4096);
    expect(astra_fused_add_rmsnorm(nullptr, b.p, c.p, 1, 8, ASTRA_F16, 1e-6f, s) == ASTRA_ERR_NULL, "null pointer status");
    expect(astra_fused_add_rmsnorm(a.p, b.p, c.p, -1, 8, ASTRA_F16, 1e-6f, s) == ASTRA_ERR_SHAPE, "shape status");
    expect(astra_fused_add_rmsnorm(a.p, b.p, c.p, 1, 8, (astra_dtype_t)9, 1e-6f, s) == ASTRA_ERR_DTYPE, "dtype status");
    expect(astra_fused_add_rmsnorm(a.p, b.p, c.p, 1, 8, ASTRA_F16, -1.0f, s) == ASTRA_ERR_EPS, "eps status");
    expect(astra_fused_add_rmsnorm((char*)a.p + 1, b.p, c.p, 1, 8, ASTRA_F16, 1e-6f, s) == ASTRA_ERR_ALIGN, "alignment status");
    expect(astra_fused_add_rmsnorm(a.p, a.p + 4, c.p, 1, 8, ASTRA_F16, 1e-6f, s) == ASTRA_ERR_ALIAS, "alias status");
    expect(astra_silu_and_mul(a.p, a.p + 8, 2, 8, ASTRA_BF16, s) == ASTRA_ERR_ALIAS, "silu alias status");
    expect(astra_fused_add_rmsnorm(a.p, b.p, c.p, 0, 8, ASTRA_F16, 1e-6f, s) == ASTRA_OK, "T == 0 is a no-op");
    expect(std::strcmp(astra_status_string(ASTRA_OK), "ok") == 0, "status string");
    HIP_OK(hipStreamSynchronize(s));
    std::printf("c_abi: ok error statuses\n");
}

}  // namespace

int main()
{
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) {
        std::fprintf(stderr, "c_abi: no HIP device\n");
        return 2;
    }
    HIP_OK(hipSetDevice(0));
    hipStream_t s;
    HIP_OK(hipStreamCreate(&s));  // a stream of the default priority that is not the null stream

    check_errors(s);
    check_host_queries();
    for (int dt : {ASTRA_F16, ASTRA_BF16}) {
        check_strided(dt, s);
        check_rmsnorm<uint16_t>(dt, 5, 4096, 1e-6f, s);
        check_rmsnorm<uint16_t>(dt, 300, 8192, 1e-5f, s);
        check_rmsnorm<uint16_t>(dt, 17, 5120, 1e-5f, s);
        check_rmsnorm<uint16_t>(dt, 3, 100, 1e-5f, s);      // element-wise path
        check_rmsnorm<uint16_t>(dt, 1100, 2048, 1e-5f, s);   // XCD-aware launch order
        check_silu<uint16_t>(dt, 7, 1408, s);
        check_silu<uint16_t>(dt, 130, 11008, s);
        check_silu<uint16_t>(dt, 3, 100, s);
        check_merge<uint16_t>(dt, 33, 40, 128, s);
        check_merge<uint16_t>(dt, 5, 7, 36, s);
    }
    check_rmsnorm<float>(ASTRA_F32, 40, 8192, 1e-5f, s);
    check_rmsnorm<float>(ASTRA_F32, 3, 6, 1e-5f, s);
    check_silu<float>(ASTRA_F32, 9, 1412, s);
    check_merge<float>(ASTRA_F32, 33, 8, 64, s);

    HIP_OK(hipStreamSynchronize(s));
    HIP_OK(hipStreamDestroy(s));
    if (g_failures) {
        std::printf("c_abi: %d check(s) FAILED\n", g_failures);
        return 1;
    }
    std::printf("c_abi: all checks passed\n");
    return 0;
}
