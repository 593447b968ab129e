"""Comparison helpers shared by the CPU and GPU tests (no operator arithmetic here)."""
import numpy as np

# tolerances fixed by the benchmark statement: (rtol, atol) per storage type, and the lse bound.  The
# binary32 storage type is not part of the benchmark; its bound comes from the arithmetic (u = 2^-24 = 6e-8):
#   fused_add_rmsnorm  the order of the row sum, about sqrt(H) * u relative on the mean square, half of it on the
#                      scale (3e-6 at H = 8192), the hardware rsq (1 ulp), two products: under 5e-6;
#   silu_and_mul       e^-x as 2^(-x log2 e): rounding the exponent argument costs |x| * log2(e) * u relative
#                      (9e-6 at |x| = 100, the largest outlier), exp2 and rcp 1 ulp each, two products: under 1.2e-5;
#   merge              the same on e^(S - max) with |S - max| <= 20 (2e-6), rcp, log2, one multiply and one fused
#                      multiply-add per element: under 5e-6 relative to the larger term.
# rtol 2e-5 covers the largest of these with less than a factor of two to spare; atol 1e-6 is for results near
# zero (a blend of two terms of opposite sign, silu of a very negative x).
TOL = {"bf16": (1.6e-2, 1e-2), "f16": (2e-3, 1e-3), "f32": (2e-5, 1e-6)}
LSE_ATOL = 1e-4


def close_mask(got, ref, rtol, atol):
    """|got - ref| <= atol + rtol*|ref| elementwise; equal infinities match; NaN matches only NaN."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    with np.errstate(invalid="ignore"):
        ok = np.abs(got - ref) <= atol + rtol * np.abs(ref)
    inf = np.isinf(got) | np.isinf(ref)
    ok = np.where(inf, got == ref, ok)
    nan = np.isnan(got) | np.isnan(ref)
    ok = np.where(nan, np.isnan(got) & np.isnan(ref), ok)
    return ok


def assert_close(got, ref, rtol, atol, what=""):
    ok = close_mask(got, ref, rtol, atol)
    if not ok.all():
        bad = np.argwhere(~ok)
        i = tuple(bad[0])
        raise AssertionError(f"{what}: {len(bad)} of {ok.size} elements out of tolerance (rtol={rtol}, atol={atol}); "
                             f"first at {i}: got {np.asarray(got)[i]!r}, ref {np.asarray(ref)[i]!r}")


def assert_bits_equal(got, ref, what=""):
    got = np.asarray(got)
    ref = np.asarray(ref)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    if not np.array_equal(got, ref):
        bad = np.argwhere(got != ref)
        i = tuple(bad[0])
        raise AssertionError(f"{what}: {len(bad)} of {got.size} bit patterns differ; first at {i}: "
                             f"got 0x{int(got[i]):04x}, ref 0x{int(ref[i]):04x}")
