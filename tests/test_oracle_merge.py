"""Pins for the merge_attn_states_lse oracle (paper Table 1, Kernel 1):
V_out = (e^Sa Va + e^Sb Vb) / (e^Sa + e^Sb),  S_out = log(e^Sa + e^Sb).

The main pin is the operator's meaning: merging the partial softmax-attention results of two key sets
gives the attention over their union.  That is computed here by brute force in float64.
"""
import json
import os

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from oracle import reference_f64
from tests.util import LSE_ATOL, TOL, assert_close
import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "closed_forms.json")


def _attention(q, K, V):
    """softmax(q K^T) V and logsumexp(q K^T), float64, one query."""
    s = K @ q
    return softmax(s) @ V, logsumexp(s)


@pytest.mark.parametrize("D", [1, 4, 8])
def test_merge_equals_attention_over_union(oracle, D):
    rng = np.random.default_rng(D)
    for na in range(1, 6):
        for nb in range(1, 6):
            q = rng.standard_normal(D) * 2
            KA, VA = rng.standard_normal((na, D)), rng.standard_normal((na, D))
            KB, VB = rng.standard_normal((nb, D)), rng.standard_normal((nb, D))
            va, sa = _attention(q, KA, VA)
            vb, sb = _attention(q, KB, VB)
            vu, su = _attention(q, np.concatenate([KA, KB]), np.concatenate([VA, VB]))
            vo, lo = oracle.merge_attn_states_lse_f32(va.astype(np.float32).reshape(1, 1, D), np.float32(sa).reshape(1, 1),
                                                      vb.astype(np.float32).reshape(1, 1, D), np.float32(sb).reshape(1, 1))
            np.testing.assert_allclose(vo[0, 0], vu, rtol=0, atol=2e-6)
            np.testing.assert_allclose(lo[0, 0], su, rtol=0, atol=2e-6)


def test_merge_equals_attention_large_score_gap(oracle):
    """scores far apart and far from zero: the naive e^S would overflow binary32 (S up to 200)."""
    rng = np.random.default_rng(99)
    D = 4
    q = rng.standard_normal(D)
    KA, VA = rng.standard_normal((3, D)) * 60 + 40, rng.standard_normal((3, D))
    KB, VB = rng.standard_normal((2, D)) * 60 - 40, rng.standard_normal((2, D))
    va, sa = _attention(q, KA, VA)
    vb, sb = _attention(q, KB, VB)
    vu, su = _attention(q, np.concatenate([KA, KB]), np.concatenate([VA, VB]))
    vo, lo = oracle.merge_attn_states_lse_f32(va.astype(np.float32).reshape(1, 1, D), np.float32(sa).reshape(1, 1),
                                              vb.astype(np.float32).reshape(1, 1, D), np.float32(sb).reshape(1, 1))
    assert np.all(np.isfinite(vo)) and np.isfinite(lo[0, 0])
    np.testing.assert_allclose(vo[0, 0], vu, rtol=0, atol=2e-6)
    np.testing.assert_allclose(lo[0, 0], su, rtol=1e-6)


def _rand_case(T, NH, D, seed, dt=None):
    rng = np.random.default_rng(seed)
    if dt is None:
        va = rng.standard_normal((T, NH, D)).astype(np.float32)
        vb = rng.standard_normal((T, NH, D)).astype(np.float32)
        la = rng.uniform(-5, 15, (T, NH)).astype(np.float32)
        lb = rng.uniform(-5, 15, (T, NH)).astype(np.float32)
        return va, la, vb, lb
    return workloads.merge_inputs(T, NH, D, dt, rng, empty_p=0.2)


def test_symmetry_bit_exact(oracle):
    va, la, vb, lb = _rand_case(7, 5, 16, 0)
    v1, l1 = oracle.merge_attn_states_lse_f32(va, la, vb, lb)
    v2, l2 = oracle.merge_attn_states_lse_f32(vb, lb, va, la)
    assert np.array_equal(v1.view(np.uint32), v2.view(np.uint32))
    assert np.array_equal(l1.view(np.uint32), l2.view(np.uint32))
    for dt in ("bf16", "f16"):
        a, sa, b, sb = _rand_case(9, 4, 24, 1, dt)
        o1, s1 = oracle.merge_attn_states_lse(a, sa, b, sb, dt)
        o2, s2 = oracle.merge_attn_states_lse(b, sb, a, sa, dt)
        assert np.array_equal(o1, o2) and np.array_equal(s1.view(np.uint32), s2.view(np.uint32))


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_one_sided_empty_returns_the_other_bit_exactly(oracle, dt):
    a, sa, b, sb = _rand_case(6, 3, 32, 2, dt)
    sa = np.where(np.isneginf(sa), np.float32(1.5), sa)       # keep side a non-empty
    sb_empty = np.full_like(sb, -np.inf)
    vo, lo = oracle.merge_attn_states_lse(a, sa, b, sb_empty, dt)
    assert np.array_equal(vo, a) and np.array_equal(lo.view(np.uint32), sa.view(np.uint32))
    vo, lo = oracle.merge_attn_states_lse(b, sb_empty, a, sa, dt)
    assert np.array_equal(vo, a) and np.array_equal(lo.view(np.uint32), sa.view(np.uint32))


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_garbage_in_an_empty_partition_is_never_looked_at(oracle, dt):
    """The merged result is attention over the union of the key sets; a partition with no keys (score -inf) has
    no value vector, so whatever its buffer holds -- NaN, inf, anything -- must not reach the output, and the
    other side comes back bit for bit (including a negative zero)."""
    a, sa, b, sb = _rand_case(6, 3, 32, 12, dt)
    sa = np.where(np.isneginf(sa), np.float32(0.25), sa)
    a[0, 0, :4] = workloads.to_bits(np.array([-0.0, 0.0, -1.0, 3.0], np.float32), dt)
    sb_empty = np.full_like(sb, -np.inf)
    for junk in (np.nan, np.inf, -np.inf):
        g = b.copy()
        g[...] = workloads.to_bits(np.array([junk], np.float32), dt)[0]
        for vo, lo in (oracle.merge_attn_states_lse(a, sa, g, sb_empty, dt), oracle.merge_attn_states_lse(g, sb_empty, a, sa, dt)):
            assert np.array_equal(vo, a) and np.array_equal(lo.view(np.uint32), sa.view(np.uint32))
    # the all-binary32 and the float64 forms
    af = reference_f64.widen(a, dt).astype(np.float32)
    gf = np.full_like(af, np.nan)
    vo, lo = oracle.merge_attn_states_lse_f32(af, sa, gf, sb_empty)
    assert np.array_equal(vo.view(np.uint32), af.view(np.uint32))
    vo, lo = oracle.merge_attn_states_lse_f32(gf, sb_empty, af, sa)
    assert np.array_equal(vo.view(np.uint32), af.view(np.uint32))
    v64, _ = reference_f64.merge_attn_states_lse(a, sa, workloads.to_bits(gf, dt), sb_empty, dt)
    assert np.array_equal(v64, reference_f64.widen(a, dt))
    # both sides empty, both full of garbage: still 0 and -inf
    vo, lo = oracle.merge_attn_states_lse(workloads.to_bits(gf, dt), sb_empty, workloads.to_bits(gf, dt), sb_empty, dt)
    assert np.all((vo & 0x7FFF) == 0) and np.all(np.isneginf(lo))
    # a weight that underflows to exactly zero (scores more than 104 apart) leaves its side out as well
    far = (sa - np.float32(200.0)).astype(np.float32)
    vo, _ = oracle.merge_attn_states_lse(a, sa, workloads.to_bits(gf, dt), far, dt)
    assert np.array_equal(vo, a)


def test_both_empty_gives_zero_and_minus_inf(oracle):
    dt = "bf16"
    a, _, b, _ = _rand_case(2, 2, 8, 3, dt)
    e = np.full((2, 2), -np.inf, np.float32)
    vo, lo = oracle.merge_attn_states_lse(a, e, b, e, dt)
    assert np.all((vo & 0x7FFF) == 0) and np.all(np.isneginf(lo))
    aw, bw, s = oracle.merge_weights_f32(-np.inf, -np.inf)
    assert aw == 0.0 and bw == 0.0 and s == -np.inf


def test_equal_scores_average_and_ln2(oracle):
    with open(GOLDEN) as f:
        ln2 = json.load(f)["merge_equal_scores"]["ln2"]
    assert abs(ln2 - np.log(2.0)) < 1e-15
    va, la, vb, _ = _rand_case(4, 3, 8, 4)
    vo, lo = oracle.merge_attn_states_lse_f32(va, la, vb, la)
    assert np.array_equal(vo.view(np.uint32), (0.5 * va + 0.5 * vb).view(np.uint32))
    np.testing.assert_allclose(lo, la.astype(np.float64) + ln2, rtol=0, atol=1e-6)


def test_shift_invariance(oracle):
    va, la, vb, lb = _rand_case(5, 4, 8, 5)
    v0, l0 = oracle.merge_attn_states_lse_f32(va, la, vb, lb)
    for c in (8.0, -16.0, 64.0):                               # exact shifts for these magnitudes? not always: compare with tolerance
        v1, l1 = oracle.merge_attn_states_lse_f32(va, la + np.float32(c), vb, lb + np.float32(c))
        np.testing.assert_allclose(v1, v0, rtol=0, atol=2e-5)
        np.testing.assert_allclose(l1, l0.astype(np.float64) + c, rtol=0, atol=2e-5)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_convexity_after_rounding(oracle, dt):
    """a, b >= 0 and a + b = 1: V_out lies between v_a and v_b; rounding is monotone and the end points
    are representable, so it holds for the stored result too."""
    a, sa, b, sb = _rand_case(16, 4, 64, 6, dt)
    vo, lo = oracle.merge_attn_states_lse(a, sa, b, sb, dt)
    fa, fb, fo = (reference_f64.widen(t, dt) for t in (a, b, vo))
    live = ~(np.isneginf(sa) & np.isneginf(sb))[..., None]
    lo_b, hi_b = np.minimum(fa, fb), np.maximum(fa, fb)
    assert np.all(((fo >= lo_b) & (fo <= hi_b)) | ~live)
    m = np.maximum(sa, sb).astype(np.float64)
    liv = live[..., 0]
    assert np.all(lo[liv] >= m[liv] - 1e-6) and np.all(lo[liv] <= m[liv] + np.log(2.0) + 1e-6)


def test_associativity_three_way(oracle):
    rng = np.random.default_rng(7)
    T, NH, D = 6, 3, 8
    v = [rng.standard_normal((T, NH, D)).astype(np.float32) for _ in range(3)]
    s = [rng.uniform(-5, 15, (T, NH)).astype(np.float32) for _ in range(3)]
    ab = oracle.merge_attn_states_lse_f32(v[0], s[0], v[1], s[1])
    left = oracle.merge_attn_states_lse_f32(ab[0], ab[1], v[2], s[2])
    bc = oracle.merge_attn_states_lse_f32(v[1], s[1], v[2], s[2])
    right = oracle.merge_attn_states_lse_f32(v[0], s[0], bc[0], bc[1])
    np.testing.assert_allclose(left[0], right[0], rtol=0, atol=3e-6)
    np.testing.assert_allclose(left[1], right[1], rtol=0, atol=3e-6)
    # and both equal the three-way softmax-weighted mean in float64
    S = np.stack(s).astype(np.float64)
    W = softmax(S, axis=0)
    np.testing.assert_allclose(left[0], np.einsum("kth,kthd->thd", W, np.stack(v).astype(np.float64)), rtol=0, atol=3e-6)
    np.testing.assert_allclose(left[1], logsumexp(S, axis=0), rtol=0, atol=3e-6)


def test_dominance(oracle):
    """Sa - Sb > 104: e^(Sb - Sa) underflows binary32 entirely, so V_out = v_a bit-exactly."""
    va, _, vb, _ = _rand_case(3, 2, 8, 8)
    la = np.full((3, 2), 60.0, np.float32)
    lb = np.full((3, 2), -45.0, np.float32)
    vo, lo = oracle.merge_attn_states_lse_f32(va, la, vb, lb)
    assert np.array_equal(vo.view(np.uint32), va.view(np.uint32)) and np.all(lo == 60.0)


def test_weights_closed_form(oracle):
    """a = sigmoid(Sa - Sb), b = sigmoid(Sb - Sa), S_out = logaddexp(Sa, Sb) via library routines."""
    from scipy.special import expit

    rng = np.random.default_rng(9)
    for sa, sb in rng.uniform(-5, 15, (200, 2)).astype(np.float32):
        a, b, s = oracle.merge_weights_f32(sa, sb)
        d = np.float64(sa) - np.float64(sb)
        assert abs(a - expit(d)) < 2e-7 and abs(b - expit(-d)) < 2e-7
        assert abs(s - np.logaddexp(np.float64(sa), np.float64(sb))) < 2e-6


def test_layout_lse_is_token_major(oracle):
    """lse[t, h] pairs with v[t, h, :]: a single dominant (t, h) on side b flips exactly that vector."""
    T, NH, D = 3, 4, 8
    va = np.zeros((T, NH, D), np.float32)
    vb = np.ones((T, NH, D), np.float32)
    la = np.zeros((T, NH), np.float32)
    lb = np.full((T, NH), -200.0, np.float32)
    lb[2, 1] = 200.0
    vo, _ = oracle.merge_attn_states_lse_f32(va, la, vb, lb)
    expect = np.zeros((T, NH, D), np.float32)
    expect[2, 1, :] = 1.0
    assert np.array_equal(vo, expect)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_storage_form_agrees_with_float64_definition(oracle, dt):
    a, sa, b, sb = workloads.merge_inputs(64, 8, 128, dt, np.random.default_rng(10), empty_p=0.1)
    vo, lo = oracle.merge_attn_states_lse(a, sa, b, sb, dt)
    v64, l64 = reference_f64.merge_attn_states_lse(a, sa, b, sb, dt)
    ulp = 2.0 ** -8 if dt == "bf16" else 2.0 ** -11
    assert_close(reference_f64.widen(vo, dt), v64, rtol=1.01 * ulp, atol=1e-6, what="v_out")
    assert_close(lo, l64, rtol=0, atol=2e-6, what="lse_out")
    rt, at = TOL[dt]
    assert_close(reference_f64.widen(vo, dt), v64, rt, at, "v_out (operator tolerance)")
    assert_close(lo, l64, 0, LSE_ATOL, "lse_out (operator tolerance)")
    assert np.isneginf(sa).any() and np.isneginf(sb).any() and (np.isneginf(sa) & np.isneginf(sb)).any()
