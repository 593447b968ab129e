"""The seeded synthetic inputs: determinism, shapes, and the distribution recipe."""
import numpy as np

from oracle import reference_f64
import workloads


def test_case_table_covers_every_benchmark_config():
    names = set(workloads.CASES)
    assert "c0_rmsnorm_T16_H4096_bf16" in names
    assert "c1_silu_T4096_d14336_bf16" in names
    assert "c2_merge_T4096_NH32_D128_bf16" in names
    for T in (1, 8, 64, 512, 8192, 32768):
        for dt in ("bf16", "f16"):
            assert f"c3_rmsnorm_T{T}_H8192_{dt}" in names
    for T in (1, 3, 257, 4099):
        for n in (f"c4_rmsnorm_T{T}_H5120_f16", f"c4_rmsnorm_T{T}_H7168_f16", f"c4_silu_T{T}_d11008_f16",
                  f"c4_silu_T{T}_d1408_f16", f"c4_merge_T{T}_NH40_D64_f16", f"c4_merge_T{T}_NH40_D256_f16"):
            assert n in names
    assert len({(c.config, c.case) for c in workloads.CASES.values()}) == len(names)


def test_deterministic():
    c = workloads.case("c4_merge_T257_NH40_D64_f16")
    a = c.generate()
    b = c.generate()
    for u, v in zip(a, b):
        assert np.array_equal(u.view(np.uint8), v.view(np.uint8))


def test_rmsnorm_recipe():
    c = workloads.case("c3_rmsnorm_T64_H8192_bf16")
    x, r, w = c.generate()
    assert x.shape == (64, 8192) and r.shape == (64, 8192) and w.shape == (8192,) and x.dtype == np.uint16
    xf, rf, wf = (reference_f64.widen(t, "bf16") for t in (x, r, w))
    assert abs(xf.std() - 1.0) < 0.01 and abs(rf.std() - 2.0) < 0.02
    assert abs(wf.mean() - 1.0) < 0.02 and abs(wf.var() - 0.1) < 0.01
    assert c.algorithmic_bytes() == 4 * 64 * 8192 * 2 + 8192 * 2


def test_silu_recipe():
    c = workloads.case("c4_silu_T257_d1408_f16")
    (a,) = c.generate()
    assert a.shape == (257, 2816)
    f = reference_f64.widen(a, "f16")
    frac_big = np.mean(np.abs(f) > 6.0)                 # P(|z|>6) ~ 2e-9 without outliers; 20 z exceeds 6 w.p. 0.76
    assert 4e-4 < frac_big < 1.2e-3
    assert c.algorithmic_bytes() == 3 * 257 * 1408 * 2


def test_merge_recipe():
    c = workloads.case("c4_merge_T4099_NH40_D64_f16")
    va, la, vb, lb = c.generate()
    assert va.shape == (4099, 40, 64) and la.shape == (4099, 40) and la.dtype == np.float32
    for s in (la, lb):
        e = np.isneginf(s)
        assert 0.007 < e.mean() < 0.013
        assert s[~e].min() >= -5.0 and s[~e].max() < 15.0
    assert (np.isneginf(la) & np.isneginf(lb)).sum() > 0
    assert c.algorithmic_bytes() == 3 * 4099 * 40 * 64 * 2 + 3 * 4099 * 40 * 4
