"""Memory- and UB-safety of the host side of the C-ABI library (argument validation, launch planning, the
workgroup-to-work map): the API source is compiled by hipcc with AddressSanitizer and UndefinedBehaviorSanitizer on
the HOST side only, linked with a driver, and run on the CPU.  The driver stays on paths that return before any
kernel launch (failed validation, T == 0, the plan functions), with ordinary and extreme shapes: T, H, strides near
2^62, K = 65536, pointers near the top of the address space."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = r"""
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include "astra.h"
#include "astra_ablation.h"
#include "astra_kway.h"
#include "astra_plan.h"
#include "astra_strided.h"

static int fails = 0;
#define EXPECT(cond) do { if (!(cond)) { std::printf("FAILED %s:%d %s\n", __FILE__, __LINE__, #cond); ++fails; } } while (0)
static void* P(uint64_t a) { return reinterpret_cast<void*>(a); }

int main()
{
    const int64_t big[] = {0, 1, 7, 8, 9, 4096, 4099, 5121, 32768, 32775, 65536, (int64_t(1) << 21) - 1, int64_t(1) << 21,
                           (int64_t(1) << 31) - 1, int64_t(1) << 31, (int64_t(1) << 32) + 3, int64_t(1) << 40, (int64_t(1) << 61) - 1,
                           int64_t(1) << 61, (int64_t(1) << 62) - 1, int64_t(1) << 62, INT64_MAX, -1, INT64_MIN};
    const int nb = (int)(sizeof big / sizeof big[0]);
    astra_launch_info_t li;
    // ---- plan functions over every pair of sizes, storage type and alignment class
    for (int a = 0; a < nb; ++a)
        for (int b = 0; b < nb; ++b)
            for (int dt = -1; dt <= 3; ++dt)
                for (int al = 0; al <= 2; ++al) {
                    const int64_t T = big[a], H = big[b];
                    astra_status_t st = astra_plan_fused_add_rmsnorm(T, H, (astra_dtype_t)dt, al, &li);
                    if (st == ASTRA_OK && T > 0) {
                        EXPECT(li.path >= ASTRA_PATH_VECTOR && li.path <= ASTRA_PATH_PHASED && li.grid >= 1 && li.block >= 64 && li.block <= 1024);
                        EXPECT(li.log2_xcd_chunk >= 0 && li.log2_xcd_chunk <= 8 && li.grid % (int64_t(8) << li.log2_xcd_chunk) == 0 || li.log2_xcd_chunk == 0 || li.grid < T);
                        EXPECT(li.grid <= (int64_t(1) << 21) + 2048);
                    }
                    st = astra_plan_silu_and_mul(T, H, (astra_dtype_t)dt, al, &li);
                    if (st == ASTRA_OK && T > 0) EXPECT(li.grid >= 1 && li.grid < (int64_t(1) << 32) && (li.block == 64 || li.block == 128 || li.block == 256));
                    for (int64_t D : {int64_t(1), int64_t(7), int64_t(128), int64_t(129), int64_t(1) << 33}) {
                        st = astra_plan_merge_attn_states_lse(T, H, D, (astra_dtype_t)dt, al, &li);
                        if (st == ASTRA_OK && T > 0) EXPECT(li.grid >= 1 && li.grid < (int64_t(1) << 32));
                    }
                }
    EXPECT(astra_plan_fused_add_rmsnorm(1, 8, ASTRA_BF16, 1, nullptr) == ASTRA_ERR_NULL);
    // ---- the workgroup-to-work map is a permutation of [0, G) for G a multiple of 8 * 2^lc
    for (int lc = -2; lc <= 10; ++lc) {
        const uint32_t G = (lc >= 0 && lc <= 8) ? 3u * (8u << lc) : 64u;
        std::vector<char> seen(G, 0);
        for (uint32_t wg = 0; wg < G; ++wg) {
            const uint32_t u = astra_plan_xcd_chunked(wg, lc);
            EXPECT(u < G);
            if (u < G) { EXPECT(!seen[u]); seen[u] = 1; }
        }
    }
    (void)astra_plan_xcd_chunked(0xffffffffu, 8);
    (void)astra_plan_xcd_chunked(0xffffffffu, 0);
    // ---- entry points: every call below fails validation or has T == 0, so no kernel is launched.  Pointers are never
    // dereferenced on the host; they are spread over the address space, including its top.
    const uint64_t bases[] = {0x10000, 0x7fff00000000ull, 0xffffffffffff0000ull, 0xfffffffffffffff0ull};
    for (uint64_t base : bases)
        for (int a = 0; a < nb; ++a)
            for (int b = 0; b < nb; ++b) {
                const int64_t T = big[a], H = big[b];
                const bool huge = T > 0 && H > 0 && (T >= 0x200 || H >= 0x200);  // tensors 256 bytes apart: these overlap or wrap and must be refused, not launched
                void *x = P(base), *r = P(base + 0x100), *w = P(base + 0x200), *o = P(base + 0x300);
                if (T <= 0 || H <= 0 || huge) {
                    for (int dt = 0; dt <= 3; ++dt) {
                        astra_status_t st = astra_fused_add_rmsnorm(x, r, w, T, H, (astra_dtype_t)dt, 1e-6f, nullptr);
                        EXPECT(st != ASTRA_ERR_LAUNCH && (T == 0 || st != ASTRA_OK || H <= 0));
                        st = astra_silu_and_mul(o, x, T, H, (astra_dtype_t)dt, nullptr);
                        EXPECT(st != ASTRA_ERR_LAUNCH);
                        st = astra_merge_attn_states_lse(o, (float*)P(base + 0xc0), x, (const float*)P(base + 0x40), r, (const float*)P(base + 0x80), T, H, 128, (astra_dtype_t)dt, nullptr);
                        EXPECT(st != ASTRA_ERR_LAUNCH);
                        st = astra_merge_attn_states_lse(o, (float*)P(base + 0xc0), x, (const float*)P(base + 0x40), r, (const float*)P(base + 0x80), 3, T, H, (astra_dtype_t)dt, nullptr);
                        EXPECT(st != ASTRA_ERR_LAUNCH && (st != ASTRA_OK));
                        for (int64_t K : {int64_t(0), int64_t(1), int64_t(65536), int64_t(65537), INT64_MAX}) {
                            st = astra_merge_attn_states_lse_kway(o, (float*)P(base + 0xc0), x, (const float*)P(base + 0x40), K, T, H, 64, (astra_dtype_t)dt, nullptr);
                            EXPECT(st != ASTRA_ERR_LAUNCH);
                        }
                        for (int v = -1; v <= 10; ++v) {
                            st = astra_ablation_fused_add_rmsnorm(x, r, w, T, H, (astra_dtype_t)dt, 1e-6f, (astra_variant_t)v, nullptr);
                            EXPECT(st != ASTRA_ERR_LAUNCH);
                            st = astra_ablation_silu_and_mul(o, x, T, H, (astra_dtype_t)dt, (astra_variant_t)v, nullptr);
                            EXPECT(st != ASTRA_ERR_LAUNCH);
                            st = astra_ablation_merge_attn_states_lse(o, (float*)P(base + 0xc0), x, (const float*)P(base + 0x40), r, (const float*)P(base + 0x80), T, H, 128, (astra_dtype_t)dt, (astra_variant_t)v, nullptr);
                            EXPECT(st != ASTRA_ERR_LAUNCH);
                        }
                        // strided forms with strides from the same list
                        for (int c = 0; c < nb; c += 3) {
                            const int64_t S = big[c];
                            st = astra_fused_add_rmsnorm_strided(o, S, P(base + 0x380), S, x, S, r, big[(c + 5) % nb], w, T, H, (astra_dtype_t)dt, 1e-6f, nullptr);
                            EXPECT(st != ASTRA_ERR_LAUNCH);
                            st = astra_silu_and_mul_strided(o, S, x, big[(c + 7) % nb], T, H, (astra_dtype_t)dt, nullptr);
                            EXPECT(st != ASTRA_ERR_LAUNCH);
                            st = astra_merge_attn_states_lse_strided(o, S, big[(c + 2) % nb], (float*)P(base + 0xc0), x, S, S, (const float*)P(base + 0x40), r, big[(c + 9) % nb], S,
                                                                     (const float*)P(base + 0x80), T, H, 64, (astra_dtype_t)dt, nullptr);
                            EXPECT(st != ASTRA_ERR_LAUNCH);
                        }
                    }
                }
                astra_status_t st = astra_stream_copy(o, x, T, nullptr);
                EXPECT(st != ASTRA_ERR_LAUNCH || T > 0);
                if (T <= 0 || T % 16 != 0 || T > 0x4000) {
                    st = astra_stream_copy(o, x, T, nullptr);
                    EXPECT(st != ASTRA_ERR_LAUNCH);
                    for (int m = -1; m <= 5; ++m)  // (mode 2 touches one buffer only, so a size that is valid for it would be launched)
                        if (m != ASTRA_PROBE_WRITE1 || T <= 0 || T % 16 != 0) EXPECT(astra_stream_probe(x, r, o, T, (astra_probe_t)m, nullptr) != ASTRA_ERR_LAUNCH);
                }
            }
    for (int s = -2; s <= 12; ++s) EXPECT(astra_status_string((astra_status_t)s) != nullptr);
    int clk = 0, width = 0;
    EXPECT(astra_device_memory_info(0, nullptr, &width) == ASTRA_ERR_NULL && astra_device_memory_info(0, &clk, nullptr) == ASTRA_ERR_NULL);
    std::printf(fails ? "driver saw %d failed expectations\n" : "ok\n", fails);
    return fails ? 1 : 0;
}
"""


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="needs hipcc")
def test_api_layer_is_clean_under_asan_and_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    drv = tmp_path / "driver.cpp"
    drv.write_text(DRIVER)
    exe = tmp_path / "api_san"
    host = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fno-gpu-rdc",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    for f in host:                      # sanitizers on the host side only: each flag directly after -Xarch_host
        cmd += ["-Xarch_host", f]
    cmd += ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2509_07506_amd", "csrc"), "-o", str(exe), str(drv),
            os.path.join(ROOT, "paper_2509_07506_amd", "csrc", "astra_api.hip")]
    b = subprocess.run(cmd, capture_output=True, text=True)
    assert b.returncode == 0, b.stdout + b.stderr
    nm = subprocess.run(["nm", str(exe)], capture_output=True, text=True).stdout
    assert "__asan_init" in nm and "__ubsan_handle" in nm, "the host code was not instrumented"
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), (r.stdout + r.stderr)[-4000:]
