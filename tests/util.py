"""Comparison helpers shared by the CPU and GPU tests (no operator arithmetic here)."""
import numpy as np

# tolerances fixed by the benchmark statement: (rtol, atol) per storage type, and the lse bound.  The
# binary32 storage type is not part of the benchmark; its bound comes from the arithmetic: the order of the
# row sum (about sqrt(H) * 2^-24 relative on the mean square) and the hardware exp2 / rcp / rsq (about one
# ulp each, with |x| * log2(e) * 2^-24 relative on e^x from rounding the exponent argument, |x| <= 100).
TOL = {"bf16": (1.6e-2, 1e-2), "f16": (2e-3, 1e-3), "f32": (1e-4, 1e-6)}
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
