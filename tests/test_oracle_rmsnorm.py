"""Pins for the fused_add_rmsnorm oracle (paper Table 1, Kernel 2):
y = (x+r) / sqrt(||x+r||^2 / D + eps) (.) w.

Nothing here calls the oracle to produce its own expected value: every expectation is a closed form,
an invariant of the formula, or numpy float64 evaluating the textbook definition.
"""
import numpy as np
import pytest

from oracle import reference_f64
from tests.util import TOL, assert_bits_equal, assert_close
import workloads


def _rand(shape, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float32)


def test_unit_rms_before_weighting(oracle):
    """y / w has RMS sqrt(ms / (ms + eps)); with eps << ms that is 1."""
    T, H = 5, 1000
    x, r = _rand((T, H), 0), _rand((T, H), 1, 2.0)
    w = (1.0 + 0.3 * _rand((H,), 2)).astype(np.float32)
    eps = 1e-6
    s, y = oracle.fused_add_rmsnorm_f32(x, r, w, eps)
    u = y.astype(np.float64) / w.astype(np.float64)
    rms = np.sqrt(np.mean(u * u, axis=1))
    ms = np.mean(s.astype(np.float64) ** 2, axis=1)
    np.testing.assert_allclose(rms, np.sqrt(ms / (ms + eps)), rtol=2e-6)
    np.testing.assert_allclose(rms, 1.0, rtol=2e-6)
    # with w = 1 exactly, y itself has unit RMS
    _, y1 = oracle.fused_add_rmsnorm_f32(x, r, np.ones(H, np.float32), eps)
    np.testing.assert_allclose(np.sqrt(np.mean(y1.astype(np.float64) ** 2, axis=1)), 1.0, rtol=2e-6)


def test_unit_rms_after_storage_rounding(oracle):
    for dt, tol in (("bf16", 3e-3), ("f16", 4e-4)):
        T, H = 4, 4096
        x = workloads.to_bits(_rand((T, H), 3), dt)
        r = workloads.to_bits(_rand((T, H), 4), dt)
        w = workloads.to_bits(np.ones(H, np.float32), dt)
        yb, _ = oracle.fused_add_rmsnorm(x, r, w, 1e-6, dt)
        y = reference_f64.widen(yb, dt)
        np.testing.assert_allclose(np.sqrt(np.mean(y * y, axis=1)), 1.0, rtol=tol)


def test_constant_row_closed_form(oracle):
    """s_j = c for all j  =>  y_j = c / sqrt(c^2 + eps) * w_j."""
    H = 257
    w = (1.0 + 0.3 * _rand((H,), 5)).astype(np.float32)
    for c, eps in [(3.0, 1e-6), (-0.5, 1e-5), (1e-3, 1e-6), (0.0, 1e-6), (100.0, 0.25)]:
        x = np.full((1, H), 0.25 * c, np.float32)
        r = np.full((1, H), 0.75 * c, np.float32)
        _, y = oracle.fused_add_rmsnorm_f32(x, r, w, eps)
        expect = c / np.sqrt(np.float64(c) ** 2 + np.float64(np.float32(eps))) * w.astype(np.float64)
        np.testing.assert_allclose(y[0], expect, rtol=2e-6, atol=0)   # binary32 sequential sum of 257 terms


def test_all_zero_row_is_zero_not_nan(oracle):
    H = 64
    z = np.zeros((1, H), np.float32)
    _, y = oracle.fused_add_rmsnorm_f32(z, z, np.ones(H, np.float32), 1e-6)
    assert np.all(y == 0.0)


def test_power_of_two_scale_invariance(oracle):
    """eps = 0: scaling x and r by 2^k is exact in binary32, so y is bit-identical and s scales by 2^k."""
    T, H = 3, 512
    x, r = _rand((T, H), 6), _rand((T, H), 7)
    w = (1.0 + 0.3 * _rand((H,), 8)).astype(np.float32)
    s0, y0 = oracle.fused_add_rmsnorm_f32(x, r, w, 0.0)
    for k in (-20, -3, 5, 30):
        f = np.float32(2.0 ** k)
        s1, y1 = oracle.fused_add_rmsnorm_f32(x * f, r * f, w, 0.0)
        assert np.array_equal(y1.view(np.uint32), y0.view(np.uint32))
        assert np.array_equal(s1.view(np.uint32), (s0 * f).view(np.uint32))


def test_zero_residual_is_textbook_rmsnorm(oracle):
    """r = 0: x / sqrt(mean(x^2) + eps) * w, evaluated here in float64 from the definition."""
    T, H = 7, 1536
    x = _rand((T, H), 9, 3.0)
    w = (1.0 + 0.3 * _rand((H,), 10)).astype(np.float32)
    eps = 1e-5
    s, y = oracle.fused_add_rmsnorm_f32(x, np.zeros_like(x), w, eps)
    assert np.array_equal(s.view(np.uint32), x.view(np.uint32))
    xd = x.astype(np.float64)
    expect = xd / np.sqrt(np.mean(xd * xd, axis=1, keepdims=True) + np.float64(np.float32(eps))) * w.astype(np.float64)
    np.testing.assert_allclose(y, expect, rtol=2e-6, atol=1e-9)


def test_hidden_size_one(oracle):
    """H = 1: y = s / sqrt(s^2 + eps) * w."""
    for xv, rv, wv, eps in [(0.5, 0.25, 2.0, 1e-6), (-3.0, 1.0, 0.5, 1e-2), (1e-4, 0.0, 1.0, 1e-6)]:
        _, y = oracle.fused_add_rmsnorm_f32(np.array([[xv]], np.float32), np.array([[rv]], np.float32),
                                            np.array([wv], np.float32), eps)
        s = np.float64(np.float32(xv) + np.float32(rv))
        np.testing.assert_allclose(y[0, 0], s / np.sqrt(s * s + np.float64(np.float32(eps))) * wv, rtol=3e-7)


def test_eps_is_inside_the_square_root(oracle):
    """With eps comparable to the mean square the two placements differ by a lot; the formula has
    sqrt(ms + eps)."""
    H = 16
    x = np.full((1, H), 1.0, np.float32)
    _, y = oracle.fused_add_rmsnorm_f32(x, np.zeros_like(x), np.ones(H, np.float32), 3.0)
    np.testing.assert_allclose(y[0], 1.0 / np.sqrt(1.0 + 3.0), rtol=3e-7)     # inside: 0.5 ; outside would be 0.25


def test_rows_are_independent_and_weight_is_per_column(oracle):
    T, H = 4, 96
    x, r = _rand((T, H), 11), _rand((T, H), 12)
    w = np.arange(1, H + 1, dtype=np.float32)
    _, y = oracle.fused_add_rmsnorm_f32(x, r, w, 1e-6)
    for t in range(T):
        _, yt = oracle.fused_add_rmsnorm_f32(x[t:t + 1], r[t:t + 1], w, 1e-6)
        assert np.array_equal(yt[0].view(np.uint32), y[t].view(np.uint32))
    _, y1 = oracle.fused_add_rmsnorm_f32(x, r, np.ones(H, np.float32), 1e-6)
    np.testing.assert_allclose(y, y1.astype(np.float64) * w, rtol=2e-7)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_stored_residual_is_one_float32_add_one_rounding(oracle, dt):
    """residual <- RNE(float32(x) + float32(r)): expectation built from numpy float32 addition and the
    library casts (numpy float16 / torch bfloat16), none of which is oracle code.  Includes exact ties
    (which must go to the even pattern) and fp16-subnormal sums."""
    T, H = 6, 2048
    xb = workloads.to_bits(_rand((T, H), 13), dt)
    rb = workloads.to_bits(_rand((T, H), 14, 2.0), dt)
    # tiny operands (fp16 subnormal results) in row 1, an exact tie in row 0
    rb[1, :64] = workloads.to_bits(np.full(64, 2.0 ** -16, np.float32) * np.arange(64, dtype=np.float32), dt)
    xb[1, :64] = workloads.to_bits(np.full(64, 2.0 ** -17, np.float32), dt)
    xb[0, 0] = workloads.to_bits(np.array([1.0], np.float32), dt)[0]
    half_ulp = 2.0 ** -8 if dt == "bf16" else 2.0 ** -11
    rb[0, 0] = workloads.to_bits(np.array([half_ulp], np.float32), dt)[0]      # 1 + half ulp: tie, rounds to 1.0
    xb[0, 1] = workloads.to_bits(np.array([1.0 + 2 * half_ulp], np.float32), dt)[0]
    rb[0, 1] = rb[0, 0]                                                         # odd + half ulp: tie, rounds up
    wb = workloads.to_bits(np.ones(H, np.float32), dt)
    _, res = oracle.fused_add_rmsnorm(xb, rb, wb, 1e-6, dt)
    xf = reference_f64.widen(xb, dt).astype(np.float32)
    rf = reference_f64.widen(rb, dt).astype(np.float32)
    expect = workloads.to_bits(xf + rf, dt)
    assert_bits_equal(res, expect, "residual")
    one = workloads.to_bits(np.array([1.0, 1.0 + 4 * half_ulp], np.float32), dt)
    assert res[0, 0] == one[0] and res[0, 1] == one[1]


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_stored_residual_is_the_correctly_rounded_exact_sum(oracle, dt):
    """For 16-bit operands the float32 sum followed by one rounding equals the exact sum rounded once
    (float32 has at least 2p+2 bits for p = 8 and p = 11, so the double rounding is innocuous).  The
    exact sum is formed in float64 (exact for these magnitudes) and rounded by a nearest-even search over
    all representable values -- no float32 and no library cast involved."""
    T, H = 4, 4096
    xb = workloads.to_bits(_rand((T, H), 21), dt)
    rb = workloads.to_bits(_rand((T, H), 22, 2.0), dt)
    wb = workloads.to_bits(np.ones(H, np.float32), dt)
    _, res = oracle.fused_add_rmsnorm(xb, rb, wb, 1e-6, dt)
    exact = reference_f64.widen(xb, dt) + reference_f64.widen(rb, dt)
    all16 = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    with np.errstate(invalid="ignore"):
        table = reference_f64.widen(all16, dt)
    pos = all16[(all16 < 0x8000) & np.isfinite(table)]
    vals = table[pos]
    mag = np.abs(exact).ravel()
    hi = np.clip(np.searchsorted(vals, mag, side="left"), 1, len(vals) - 1)
    lo = hi - 1
    dlo, dhi = mag - vals[lo], vals[hi] - mag
    pick_hi = (dhi < dlo) | ((dhi == dlo) & (pos[hi] % 2 == 0))
    expect = np.where(pick_hi, pos[hi], pos[lo]).astype(np.uint16)
    expect = np.where(np.signbit(exact).ravel(), expect | np.uint16(0x8000), expect).reshape(T, H)
    zero = (expect & 0x7FFF) == 0
    assert np.array_equal(res[~zero], expect[~zero]) and np.all((res[zero] & 0x7FFF) == 0)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_storage_form_agrees_with_float64_definition(oracle, dt):
    """The binary32 oracle stays within a small multiple of the storage ulp of the float64 definition
    (far inside the operator's tolerance), on the benchmark's distributions."""
    T, H = 9, 5120
    rng = np.random.default_rng(15)
    x, r, w = workloads.rmsnorm_inputs(T, H, dt, rng, r_std=2.0)
    yb, rb = oracle.fused_add_rmsnorm(x, r, w, 1e-5, dt)
    y64, s64 = reference_f64.fused_add_rmsnorm(x, r, w, 1e-5, dt)
    ulp = 2.0 ** -8 if dt == "bf16" else 2.0 ** -11
    assert_close(reference_f64.widen(yb, dt), y64, rtol=1.01 * ulp, atol=1e-7, what="y")
    assert_close(reference_f64.widen(rb, dt), s64, rtol=1.01 * ulp, atol=1e-7, what="residual")
    rt, at = TOL[dt]
    assert_close(reference_f64.widen(yb, dt), y64, rt, at, "y (operator tolerance)")


def test_in_place_roles(oracle):
    """input receives y, residual receives x + r."""
    dt = "bf16"
    H = 128
    x = workloads.to_bits(np.full((1, H), 1.0, np.float32), dt)
    r = workloads.to_bits(np.full((1, H), 2.0, np.float32), dt)
    w = workloads.to_bits(np.full(H, 0.5, np.float32), dt)
    y, res = oracle.fused_add_rmsnorm(x, r, w, 0.0, dt)
    assert np.all(reference_f64.widen(res, dt) == 3.0)
    assert np.all(reference_f64.widen(y, dt) == 0.5)


def test_threads_do_not_change_bits(oracle):
    dt = "f16"
    x, r, w = workloads.rmsnorm_inputs(33, 1024, dt, np.random.default_rng(16))
    oracle.set_threads(1)
    y1, r1 = oracle.fused_add_rmsnorm(x, r, w, 1e-6, dt)
    oracle.set_threads(4)
    y4, r4 = oracle.fused_add_rmsnorm(x, r, w, 1e-6, dt)
    oracle.set_threads(1)
    assert np.array_equal(y1, y4) and np.array_equal(r1, r4)
