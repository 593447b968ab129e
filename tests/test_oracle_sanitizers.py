"""Memory- and UB-safety of the C oracle: it is compiled together with a small driver under
AddressSanitizer and UndefinedBehaviorSanitizer (host only) and run over ordinary and degenerate sizes."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = r"""
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
void oracle_set_threads(int);
void oracle_fused_add_rmsnorm(uint16_t*, uint16_t*, const uint16_t*, int64_t, int64_t, int, float);
void oracle_silu_and_mul(uint16_t*, const uint16_t*, int64_t, int64_t, int);
void oracle_merge_attn_states_lse(uint16_t*, float*, const uint16_t*, const float*, const uint16_t*, const float*, int64_t, int64_t, int64_t, int);
void oracle_merge_attn_states_lse_kway(uint16_t*, float*, const uint16_t*, const float*, int64_t, int64_t, int64_t, int);
uint16_t oracle_f32_to_f16(float); uint16_t oracle_f32_to_bf16(float); float oracle_f16_to_f32(uint16_t); float oracle_bf16_to_f32(uint16_t);
static uint32_t rs = 12345u;
static uint16_t rnd16(void) { rs = rs * 1664525u + 1013904223u; return (uint16_t)(rs >> 11); }
static uint16_t* buf16(size_t n) { uint16_t* p = malloc(n * 2 + 2); for (size_t i = 0; i < n; ++i) p[i] = rnd16(); return p; }
static float* buff(size_t n) { float* p = malloc(n * 4 + 4); for (size_t i = 0; i < n; ++i) p[i] = (rnd16() % 7 == 0) ? -INFINITY : (float)(rnd16() % 2000) / 100.f - 5.f; return p; }
int main(void) {
    const int64_t Ts[] = {0, 1, 3}, Hs[] = {1, 7, 8, 129};
    for (int dt = 0; dt < 2; ++dt) for (int th = 1; th <= 3; th += 2) {
        oracle_set_threads(th);
        for (int a = 0; a < 3; ++a) for (int b = 0; b < 4; ++b) {
            int64_t T = Ts[a], H = Hs[b];
            uint16_t *x = buf16(T * H), *r = buf16(T * H), *w = buf16(H);
            oracle_fused_add_rmsnorm(x, r, w, T, H, dt, 1e-6f);
            uint16_t *in = buf16(T * 2 * H), *out = buf16(T * H);
            oracle_silu_and_mul(out, in, T, H, dt);
            int64_t NH = 3;
            uint16_t *va = buf16(T * NH * H), *vb = buf16(T * NH * H), *vo = buf16(T * NH * H);
            float *la = buff(T * NH), *lb = buff(T * NH), *lo = buff(T * NH);
            oracle_merge_attn_states_lse(vo, lo, va, la, vb, lb, T, NH, H, dt);
            for (int64_t K = 1; K <= 5; K += 2) {
                uint16_t* vp = buf16(K * T * NH * H); float* lp = buff(K * T * NH);
                oracle_merge_attn_states_lse_kway(vo, lo, vp, lp, K, T * NH, H, dt);
                free(vp); free(lp);
            }
            free(x); free(r); free(w); free(in); free(out); free(va); free(vb); free(vo); free(la); free(lb); free(lo);
        }
    }
    /* every 16-bit pattern through both conversions, and a sweep of float patterns through the narrowing */
    volatile float sink = 0; volatile uint16_t s16 = 0;
    for (uint32_t h = 0; h < 65536; ++h) { sink += oracle_f16_to_f32((uint16_t)h) == 0.f; sink += oracle_bf16_to_f32((uint16_t)h) == 0.f; }
    for (uint64_t u = 0; u < (1ull << 32); u += 65521) { union { uint32_t u; float f; } c; c.u = (uint32_t)u; s16 ^= oracle_f32_to_f16(c.f); s16 ^= oracle_f32_to_bf16(c.f); }
    printf("ok\n");
    return 0;
}
"""


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    drv = tmp_path / "driver.c"
    drv.write_text(DRIVER)
    exe = tmp_path / "oracle_san"
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-o", str(exe), str(drv),
           os.path.join(ROOT, "oracle", "astra_oracle.c"), "-lm"]
    subprocess.run(cmd, check=True)
    # verify_asan_link_order=0: the environment may preload another library ahead of the sanitizer runtime
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env)
    assert r.returncode == 0 and r.stdout.strip() == "ok", r.stdout + r.stderr
