"""Pins for the silu_and_mul oracle (paper Table 1, Kernel 3): out = SiLU(x) (.) g, SiLU(z) = z / (1 + e^-z).

Expectations are closed forms and identities of the logistic function evaluated with numpy/scipy in
float64, never the oracle's own output.
"""
import json
import os

import numpy as np
import pytest
from scipy.special import expit, lambertw

from oracle import reference_f64
from tests.util import TOL, assert_close
import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "closed_forms.json")


def _silu32(oracle, z):
    z = np.asarray(z, np.float32).reshape(-1, 1)
    a = np.concatenate([z, np.ones_like(z)], axis=1)
    return oracle.silu_and_mul_f32(a)[:, 0]


def test_silu_zero_is_zero(oracle):
    assert oracle.silu_f32(0.0) == 0.0
    for dt in ("bf16", "f16"):
        g = workloads.to_bits(np.array([3.5, -7.0, 1e3, 0.0], np.float32), dt)
        a = np.concatenate([np.zeros(4, np.uint16), g]).reshape(1, 8)
        out = oracle.silu_and_mul(a, dt)
        assert np.all((out & 0x7FFF) == 0)       # +-0


def test_odd_part_identity(oracle):
    """silu(x) - silu(-x) = x."""
    x = np.linspace(-30, 30, 4001).astype(np.float32)
    d = _silu32(oracle, x).astype(np.float64) - _silu32(oracle, -x).astype(np.float64)
    np.testing.assert_allclose(d, x, rtol=3e-7, atol=1e-7)


def test_tanh_and_expit_forms(oracle):
    """silu(x) = x/2 (1 + tanh(x/2)) = x * expit(x), both through library routines the oracle does not use."""
    x = np.concatenate([np.linspace(-20, 20, 8001), np.random.default_rng(0).standard_normal(4000) * 3]).astype(np.float32)
    got = _silu32(oracle, x).astype(np.float64)
    xd = x.astype(np.float64)
    np.testing.assert_allclose(got, xd * expit(xd), rtol=3e-7, atol=1e-12)
    np.testing.assert_allclose(got, 0.5 * xd * (1.0 + np.tanh(0.5 * xd)), rtol=3e-7, atol=2e-7)


def test_asymptotes(oracle):
    # x >= 20: 1 + e^-x == 1 in binary32, so silu(x) == x exactly
    for x in (20.0, 33.5, 100.0, 6e4):
        assert oracle.silu_f32(x) == np.float32(x)
    # x <= -89: expf(-x) overflows to inf, x / inf = -0
    for x in (-89.0, -100.0, -2000.0):
        v = np.float32(oracle.silu_f32(x))
        assert v == 0.0 and np.signbit(v)
    # moderately negative: x * e^x
    for x in (-20.0, -40.0, -60.0):
        np.testing.assert_allclose(oracle.silu_f32(x), x * np.exp(np.float64(x)), rtol=3e-7)


def test_minimum_location_and_value(oracle):
    """d/dz silu = 0 at z* = -(1 + W(1/e)), where silu(z*) = -W(1/e) (W = Lambert W).  Golden file
    keeps the two constants; scipy recomputes them here."""
    with open(GOLDEN) as f:
        gold = json.load(f)["silu_minimum"]
    w = float(np.real(lambertw(np.exp(-1.0))))
    assert abs(gold["argmin"] - (-(1.0 + w))) < 1e-12 and abs(gold["min"] - (-w)) < 1e-12
    grid = np.linspace(-1.4, -1.15, 250001).astype(np.float32)
    v = _silu32(oracle, grid)
    i = int(np.argmin(v))
    assert abs(float(grid[i]) - gold["argmin"]) < 2e-3     # flat minimum: value pins tighter than location
    assert abs(float(v[i]) - gold["min"]) < 1e-7
    assert np.all(v >= np.float32(gold["min"]) - np.float32(1e-7))


def test_gate_roles_and_linearity(oracle):
    """out = silu(first half) * second half; g = 1 gives silu(x); doubling g doubles out bit-exactly."""
    rng = np.random.default_rng(1)
    x = rng.standard_normal((3, 40)).astype(np.float32) * 3
    g = rng.standard_normal((3, 40)).astype(np.float32)
    a = np.concatenate([x, g], axis=1)
    out = oracle.silu_and_mul_f32(a)
    xd, gd = x.astype(np.float64), g.astype(np.float64)
    np.testing.assert_allclose(out, xd * expit(xd) * gd, rtol=4e-7, atol=1e-12)
    # swapping halves is a different function: the test would fail under the other convention
    swapped = gd * expit(gd) * xd
    assert np.max(np.abs(out - swapped)) > 0.1
    out2 = oracle.silu_and_mul_f32(np.concatenate([x, 2 * g], axis=1))
    assert np.array_equal(out2.view(np.uint32), (2 * out).view(np.uint32))
    out0 = oracle.silu_and_mul_f32(np.concatenate([x, 0 * g], axis=1))
    assert np.all(out0 == 0.0)


def test_row_layout_T_by_2d(oracle):
    """row t of in is [x_t | g_t]; out[t, j] depends on in[t, j] and in[t, d + j] only."""
    T, d = 5, 24
    rng = np.random.default_rng(2)
    a = rng.standard_normal((T, 2 * d)).astype(np.float32)
    out = oracle.silu_and_mul_f32(a)
    for t in (0, 3, 4):
        for j in (0, 7, 23):
            x, g = np.float64(a[t, j]), np.float64(a[t, d + j])
            np.testing.assert_allclose(out[t, j], x * expit(x) * g, rtol=4e-7, atol=1e-12)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_storage_form_single_rounding(oracle, dt):
    """Storage form = library-cast(binary32 product) and agrees with the float64 definition to one
    storage ulp, including the x20 outliers of the benchmark distribution."""
    rng = np.random.default_rng(3)
    a = workloads.silu_inputs(64, 1408, dt, rng)
    a[0, :4] = workloads.to_bits(np.array([-100.0, -95.0, 90.0, 0.0], np.float32), dt)
    out = oracle.silu_and_mul(a, dt)
    ref = reference_f64.silu_and_mul(a, dt)
    ulp = 2.0 ** -8 if dt == "bf16" else 2.0 ** -11
    assert_close(reference_f64.widen(out, dt), ref, rtol=1.01 * ulp, atol=6.1e-8, what="out")
    rt, at = TOL[dt]
    assert_close(reference_f64.widen(out, dt), ref, rt, at, "out (operator tolerance)")
    # all-binary32 form followed by the library cast gives the same bits
    f32 = oracle.silu_and_mul_f32(reference_f64.widen(a, dt).astype(np.float32))
    assert np.array_equal(workloads.to_bits(f32, dt), out)
