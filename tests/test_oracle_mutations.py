"""Do the pins bite?  Each case plants one plausible mistake in a copy of the C oracle (a dropped term,
a wrong sign, swapped operands, a wrong rounding), builds it, and runs the oracle's pin tests against
that build in a subprocess.  Every mutant must make at least one pin fail.  CPU only."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "astra_oracle.c")

MUTANTS = [
    ("rmsnorm_drop_eps", "1.0f / sqrtf(ms + eps)", "1.0f / sqrtf(ms)", "test_oracle_rmsnorm.py"),
    ("rmsnorm_eps_outside_sqrt", "1.0f / sqrtf(ms + eps)", "1.0f / (sqrtf(ms) + eps)", "test_oracle_rmsnorm.py"),
    ("rmsnorm_sum_not_mean", "float ms = sumsq / (float)H;", "float ms = sumsq;", "test_oracle_rmsnorm.py"),
    ("rmsnorm_one_plus_weight", "y[j] = (s[j] * inv) * w[j];", "y[j] = (s[j] * inv) * (1.0f + w[j]);", "test_oracle_rmsnorm.py"),
    ("rmsnorm_subtract_residual", "s[j] = x[j] + r[j];", "s[j] = x[j] - r[j];", "test_oracle_rmsnorm.py"),
    ("rmsnorm_squares_of_x_only", "sumsq += s[j] * s[j];", "sumsq += x[j] * x[j];", "test_oracle_rmsnorm.py"),
    ("rmsnorm_roles_swapped", "ri[j] = narrow(s[j], dtype);\n                xi[j] = narrow(y[j], dtype);",
     "xi[j] = narrow(s[j], dtype);\n                ri[j] = narrow(y[j], dtype);", "test_oracle_rmsnorm.py"),
    ("rmsnorm_stats_from_rounded_weight_order", "y[j] = (s[j] * inv) * w[j];", "y[j] = (x[j] * inv) * w[j];", "test_oracle_rmsnorm.py"),
    ("silu_wrong_sign", "return z / (1.0f + expf(-z));", "return z / (1.0f + expf(z));", "test_oracle_silu.py"),
    ("silu_sigmoid_only", "return z / (1.0f + expf(-z));", "return 1.0f / (1.0f + expf(-z));", "test_oracle_silu.py"),
    ("silu_halves_swapped", "float x = widen(row[j], dtype);\n            float g = widen(row[d + j], dtype);",
     "float g = widen(row[j], dtype);\n            float x = widen(row[d + j], dtype);", "test_oracle_silu.py"),
    ("silu_f32_halves_swapped", "oracle_silu_f32(in[t * 2 * d + j]) * in[t * 2 * d + d + j]",
     "oracle_silu_f32(in[t * 2 * d + d + j]) * in[t * 2 * d + j]", "test_oracle_silu.py"),
    ("merge_min_instead_of_max", "float m = fmaxf(sa, sb);", "float m = fminf(sa, sb);", "test_oracle_merge.py"),
    ("merge_weights_swapped", "*a = wa / den;\n        *b = wb / den;", "*a = wb / den;\n        *b = wa / den;", "test_oracle_merge.py"),
    ("merge_lse_drops_max", "*s_out = m + logf(den);", "*s_out = logf(den);", "test_oracle_merge.py"),
    ("merge_unnormalised", "*a = wa / den;", "*a = wa;", "test_oracle_merge.py"),
    ("merge_no_empty_guard", "if (m == -INFINITY) {\n        *a = 0.0f;", "if (0) {\n        *a = 0.0f;", "test_oracle_merge.py"),
    ("kway_no_empty_guard", "if (m == -INFINITY) {\n            lse_out[p] = -INFINITY;", "if (0) {\n            lse_out[p] = -INFINITY;", "test_oracle_merge_kway.py"),
    ("kway_sum_not_max", "for (int64_t k = 0; k < K; ++k) m = fmaxf(m, lse_parts[k * P + p]);", "for (int64_t k = 0; k < K; ++k) m = fmaxf(m, 100.0f + lse_parts[k * P + p]);", "test_oracle_merge_kway.py"),
    ("kway_unnormalised", "float a = expf(lse_parts[k * P + p] - m) / den;", "float a = expf(lse_parts[k * P + p] - m);", "test_oracle_merge_kway.py"),
    ("kway_part_stride_wrong", "acc += a * widen(v_parts[(k * P + p) * D + j], dtype);", "acc += a * widen(v_parts[(p * K + k) * D + j], dtype);", "test_oracle_merge_kway.py"),
    ("kway_lse_drops_max", "lse_out[p] = m + logf(den);", "lse_out[p] = logf(den);", "test_oracle_merge_kway.py"),
    ("merge_empty_side_leaks", "if (a == 0.0f) return b * vb;", "if (0) return b * vb;", "test_oracle_merge.py"),
    ("merge_both_empty_leaks", "if (a == 0.0f && b == 0.0f) return 0.0f;", "", "test_oracle_merge.py"),
    ("kway_empty_part_leaks", "if (a != 0.0f) acc += a * widen(", "acc += a * widen(", "test_oracle_merge_kway.py"),
    ("kway_f32_unnormalised", "float wgt = expf(lse_parts[k * P + p] - top) / total;", "float wgt = expf(lse_parts[k * P + p] - top);", "test_oracle_merge_kway.py"),
    ("kway_f32_empty_part_leaks", "if (wgt != 0.0f) sum += wgt * v_parts[", "sum += wgt * v_parts[", "test_oracle_merge_kway.py"),
    ("kway_f32_no_empty_guard", "if (top == -INFINITY) { /* every partition empty */", "if (0) {", "test_oracle_merge_kway.py"),
    ("merge_log_of_sum_of_scores", "float wb = expf(sb - m);", "float wb = expf(sb + m);", "test_oracle_merge.py"),
    ("bf16_truncates", "return (uint16_t)(sign | shr_rne(mag, 16));", "return (uint16_t)(sign | (mag >> 16));", "test_oracle_convert.py"),
    ("f16_flushes_subnormals", "if (e < 101u) return (uint16_t)sign;", "if (e < 113u) return (uint16_t)sign;", "test_oracle_convert.py"),
    ("f16_ties_away", "if (rem > half || (rem == half && (q & 1u))) q += 1u;", "if (rem >= half) q += 1u;", "test_oracle_convert.py"),
    ("f16_nan_becomes_inf", "if (mag > 0x7f800000u) return (uint16_t)(sign | 0x7e00u);", "", "test_oracle_convert.py"),
    ("f16_widen_drops_subnormals", "float v = (float)m * 5.9604644775390625e-08f; /* 2^-24 */", "float v = 0.0f * (float)m;", "test_oracle_convert.py"),
]


def _build(src_text, out):
    c = out + ".c"
    with open(c, "w") as f:
        f.write(src_text)
    subprocess.run(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC", "-shared", "-o", out, c,
                    "-lm"], check=True)


def _run_pins(lib, test_file):
    env = dict(os.environ, ASTRA_ORACLE_LIB=lib)
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                           os.path.join(ROOT, "tests", test_file)], env=env, cwd=ROOT, capture_output=True, text=True)


def test_unmodified_copy_passes_through_the_hook(tmp_path):
    """the hook itself must not be what makes the mutants fail"""
    lib = str(tmp_path / "clean.so")
    _build(open(SRC).read(), lib)
    r = _run_pins(lib, "test_oracle_merge.py")
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name,old,new,test_file", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_mutant(tmp_path, name, old, new, test_file):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for {name} not found exactly once"
    lib = str(tmp_path / f"{name}.so")
    _build(text.replace(old, new), lib)
    r = _run_pins(lib, test_file)
    assert r.returncode != 0, f"no pin noticed the planted mistake '{name}'"
    assert "failed" in r.stdout or "error" in r.stdout.lower()
