"""Pins for the oracle's hand-written 16-bit conversions.

They are the basis of the bit-exact residual requirement, so they are checked against two library
casts that share nothing with them (numpy's float16, torch's bfloat16) and against a brute-force
nearest-neighbour search done in float64.
"""
import numpy as np
import pytest
import torch

ALL16 = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)


def _same_float_bits(a, b):
    a = np.asarray(a, np.float32)
    b = np.asarray(b, np.float32)
    nan = np.isnan(a) | np.isnan(b)
    return np.array_equal(a.view(np.uint32)[~nan], b.view(np.uint32)[~nan]) and np.array_equal(np.isnan(a), np.isnan(b))


def _probe_f32(seed=0, n=1 << 22):
    """float32 probes: random bit patterns, every fp16/bf16 tie and its two float32 neighbours, edge values."""
    rng = np.random.default_rng(seed)
    rnd = rng.integers(0, 1 << 32, size=n, dtype=np.uint64).astype(np.uint32).view(np.float32)
    # values in the ranges where fp16 is normal / subnormal / overflowing
    mid = (rng.standard_normal(n // 4) * np.exp(rng.uniform(-20, 12, n // 4))).astype(np.float32)
    edge = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 65504.0, 65519.996, 65520.0, 65536.0, -65520.0,
                     2.0 ** -14, 2.0 ** -24, 2.0 ** -25, np.nextafter(np.float32(2.0 ** -25), np.float32(1)),
                     2.0 ** -26, 3 * 2.0 ** -25, 5 * 2.0 ** -25, 3.3895314e38, 3.4028235e38, 1e-45, 1.17549435e-38],
                    np.float32)
    return np.concatenate([rnd, mid, edge])


def _ties(dtype_bits_to_f32, drop_bits):
    """all exact ties of the 16-bit format inside float32, with their float32 neighbours"""
    f = dtype_bits_to_f32(ALL16)
    u = f.view(np.uint32)
    finite = np.isfinite(f)
    tie = (u[finite] | np.uint32(1 << (drop_bits - 1)))
    out = np.concatenate([tie, tie + np.uint32(1), tie - np.uint32(1)]).view(np.float32)
    return out


def test_f16_widen_all_patterns(oracle):
    got = oracle.widen(ALL16, "f16")
    ref = ALL16.view(np.float16).astype(np.float32)
    assert _same_float_bits(got, ref)


def test_bf16_widen_all_patterns(oracle):
    got = oracle.widen(ALL16, "bf16")
    ref = torch.from_numpy(ALL16.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    assert _same_float_bits(got, ref)


def test_f16_narrow_matches_numpy(oracle):
    x = np.concatenate([_probe_f32(), _ties(lambda b: b.view(np.float16).astype(np.float32), 13)])
    # fp16 subnormal ties: odd multiples of 2^-25
    k = np.arange(1, 2049, 2, dtype=np.float32) * np.float32(2.0 ** -25)
    x = np.concatenate([x, k, -k, np.nextafter(k, np.float32(1)), np.nextafter(k, np.float32(0))])
    got = oracle.narrow(x, "f16")
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    nan = np.isnan(x)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.all((got[nan] & 0x7C00) == 0x7C00) and np.all((got[nan] & 0x03FF) != 0)


def test_bf16_narrow_matches_torch(oracle):
    x = np.concatenate([_probe_f32(1), _ties(lambda b: (b.astype(np.uint32) << np.uint32(16)).view(np.float32), 16)])
    got = oracle.narrow(x, "bf16")
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    nan = np.isnan(x)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.all((got[nan] & 0x7F80) == 0x7F80) and np.all((got[nan] & 0x007F) != 0)


@pytest.mark.parametrize("dtype,drop", [("bf16", 16), ("f16", 13)])
def test_narrow_is_nearest_even_by_search(oracle, dtype, drop):
    """Independent of any library cast: among all representable neighbours pick the nearest in exact
    (float64) arithmetic, ties to the even pattern; overflow beyond max + half ulp is inf."""
    if dtype == "bf16":
        with np.errstate(invalid="ignore"):                    # the table includes signalling NaN patterns
            table = (ALL16.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    else:
        table = ALL16.view(np.float16).astype(np.float64)
    pos = ALL16[(ALL16 < 0x8000) & np.isfinite(table)]         # non-negative finite patterns, ascending in value
    vals = table[pos]
    assert np.all(np.diff(vals) > 0)
    rng = np.random.default_rng(7)
    x = np.abs(np.concatenate([_probe_f32(3, 1 << 18), _ties(
        (lambda b: (b.astype(np.uint32) << np.uint32(16)).view(np.float32)) if dtype == "bf16" else
        (lambda b: b.view(np.float16).astype(np.float32)), drop)]))
    x = x[np.isfinite(x)]
    x = x[rng.permutation(x.size)[: 1 << 19]]
    xd = x.astype(np.float64)
    hi = np.searchsorted(vals, xd, side="left")                # first value >= x
    hi = np.clip(hi, 1, len(vals) - 1)
    lo = hi - 1
    dlo = xd - vals[lo]
    dhi = vals[hi] - xd
    pick_hi = (dhi < dlo) | ((dhi == dlo) & (pos[hi] % 2 == 0))
    expect = np.where(pick_hi, pos[hi], pos[lo]).astype(np.uint16)
    # overflow: beyond the largest finite value the next "grid point" is 2^(emax+1)
    vmax = vals[-1]
    ulp = vals[-1] - vals[-2]
    inf_pat = np.uint16(0x7F80 if dtype == "bf16" else 0x7C00)
    expect = np.where(xd >= vmax + ulp / 2, inf_pat, expect)
    expect = np.where((xd > vmax) & (xd < vmax + ulp / 2), pos[-1], expect)
    got = oracle.narrow(x, dtype)
    assert np.array_equal(got, expect)
    # sign symmetry
    assert np.array_equal(oracle.narrow(-x, dtype), got | np.uint16(0x8000))


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_round_trip_every_pattern(oracle, dtype):
    f = oracle.widen(ALL16, dtype)
    back = oracle.narrow(f, dtype)
    nan = np.isnan(f)
    assert np.array_equal(back[~nan], ALL16[~nan])


def test_workload_cast_agrees_with_oracle(oracle):
    """The input generator's library casts and the oracle's conversions name the same values."""
    import workloads

    x = _probe_f32(11, 1 << 16)
    x = x[np.isfinite(x)]
    for dt in ("bf16", "f16"):
        with np.errstate(over="ignore"):
            assert np.array_equal(workloads.to_bits(x, dt), oracle.narrow(x, dt))
