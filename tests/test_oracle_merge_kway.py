"""Pins for the K-way merge oracle: the K-term form of the paper's Table 1, Kernel 1.  The paper defines
K = 2 only; the K-way operator is pinned by what it must mean (attention over the union of K key sets),
by its reduction to the two-way operator, and by associativity."""
import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from oracle import reference_f64
from tests.util import LSE_ATOL, TOL, assert_close
import workloads


def _attention(q, K, V):
    s = K @ q
    return softmax(s) @ V, logsumexp(s)


def _f16_exact(a):
    """values that survive the fp16 storage exactly (so the storage form can be compared tightly)"""
    return a.astype(np.float16).astype(np.float64)


@pytest.mark.parametrize("K", [1, 2, 3, 5, 8])
def test_kway_merge_equals_attention_over_the_union(oracle, K):
    rng = np.random.default_rng(K)
    D = 8
    for trial in range(6):
        q = rng.standard_normal(D) * 2
        sizes = rng.integers(1, 6, K)
        Ks = [rng.standard_normal((n, D)) for n in sizes]
        Vs = [rng.standard_normal((n, D)) for n in sizes]
        parts = [_attention(q, k, v) for k, v in zip(Ks, Vs)]
        vu, su = _attention(q, np.concatenate(Ks), np.concatenate(Vs))
        v_parts = np.stack([p[0] for p in parts]).reshape(K, 1, 1, D)
        s_parts = np.array([p[1] for p in parts], np.float32).reshape(K, 1, 1)
        vb = workloads.to_bits(v_parts.astype(np.float32), "f16")
        vo, lo = oracle.merge_attn_states_lse_kway(vb, s_parts, "f16")
        # expectation from the fp16-rounded partial outputs (the operator's actual inputs), in float64
        vq = reference_f64.widen(vb, "f16")[:, 0, 0, :]
        w = softmax(s_parts[:, 0, 0].astype(np.float64))
        np.testing.assert_allclose(reference_f64.widen(vo, "f16")[0, 0], w @ vq, rtol=1e-3, atol=1e-3)
        np.testing.assert_allclose(w @ vq, vu, rtol=0, atol=3e-3)          # and that is the union attention
        np.testing.assert_allclose(lo[0, 0], su, rtol=0, atol=2e-6)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_k2_is_the_two_way_operator_bit_exactly(oracle, dt):
    va, la, vb, lb = workloads.merge_inputs(17, 5, 64, dt, np.random.default_rng(1), empty_p=0.2)
    v2, l2 = oracle.merge_attn_states_lse(va, la, vb, lb, dt)
    vk, lk = oracle.merge_attn_states_lse_kway(np.stack([va, vb]), np.stack([la, lb]), dt)
    assert np.array_equal(vk & 0x7FFF, v2 & 0x7FFF) and np.array_equal(lk.view(np.uint32), l2.view(np.uint32))


def test_k1_is_the_identity(oracle):
    va, la, _, _ = workloads.merge_inputs(5, 3, 16, "bf16", np.random.default_rng(2), empty_p=0.0)
    vo, lo = oracle.merge_attn_states_lse_kway(va[None], la[None], "bf16")
    assert np.array_equal(vo, va) and np.array_equal(lo, la)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_matches_float64_definition_and_chained_two_way_merges(oracle, dt):
    rng = np.random.default_rng(3)
    K, T, NH, D = 6, 9, 4, 32
    parts = [workloads.merge_inputs(T, NH, D, dt, rng, empty_p=0.25)[:2] for _ in range(K)]
    v = np.stack([p[0] for p in parts])
    s = np.stack([p[1] for p in parts])
    s[:, 0, 0] = -np.inf                                   # one pair with every partition empty
    vo, lo = oracle.merge_attn_states_lse_kway(v, s, dt)
    v64, l64 = reference_f64.merge_attn_states_lse_kway(v, s, dt)
    rt, at = TOL[dt]
    ulp = 2.0 ** -8 if dt == "bf16" else 2.0 ** -11
    assert_close(reference_f64.widen(vo, dt), v64, 1.01 * ulp, 2e-6, "v_out vs float64")
    assert_close(lo, l64, 0, 3e-6, "lse_out vs float64")
    assert np.all((vo[0, 0] & 0x7FFF) == 0) and np.isneginf(lo[0, 0])
    # chain of two-way merges (each step rounds to the storage type, so compare with the operator tolerance)
    cv, cl = v[0], s[0]
    for k in range(1, K):
        cv, cl = oracle.merge_attn_states_lse(cv, cl, v[k], s[k], dt)
    assert_close(reference_f64.widen(cv, dt), v64, rt, at, "chained two-way vs K-way")
    assert_close(cl, l64, 0, LSE_ATOL, "chained lse")


def test_permutation_of_partitions(oracle):
    rng = np.random.default_rng(4)
    K, T, NH, D = 5, 4, 3, 16
    v = np.stack([workloads.merge_inputs(T, NH, D, "f16", rng)[0] for _ in range(K)])
    s = rng.uniform(-5, 15, (K, T, NH)).astype(np.float32)
    v0, l0 = oracle.merge_attn_states_lse_kway(v, s, "f16")
    perm = rng.permutation(K)
    v1, l1 = oracle.merge_attn_states_lse_kway(v[perm], s[perm], "f16")
    assert_close(reference_f64.widen(v1, "f16"), reference_f64.widen(v0, "f16"), 2e-3, 1e-3, "permuted")
    np.testing.assert_allclose(l1, l0, rtol=0, atol=2e-6)


def test_dominant_partition_wins_exactly(oracle):
    rng = np.random.default_rng(5)
    K, T, NH, D = 4, 2, 2, 8
    v = np.stack([workloads.merge_inputs(T, NH, D, "bf16", rng)[0] for _ in range(K)])
    s = np.full((K, T, NH), -100.0, np.float32)
    s[2] = 30.0
    vo, lo = oracle.merge_attn_states_lse_kway(v, s, "bf16")
    assert np.array_equal(vo, v[2]) and np.all(lo == 30.0)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_garbage_in_empty_partitions_is_never_looked_at(oracle, dt):
    """partitions with score -inf hold no keys: whatever their value buffers contain stays out of the result"""
    rng = np.random.default_rng(6)
    K, T, NH, D = 5, 3, 2, 16
    parts = [workloads.merge_inputs(T, NH, D, dt, rng, empty_p=0.0)[:2] for _ in range(K)]
    v = np.stack([p[0] for p in parts])
    s = np.stack([p[1] for p in parts])
    s[1] = -np.inf
    s[3] = -np.inf
    clean_v, clean_l = oracle.merge_attn_states_lse_kway(v, s, dt)
    for junk in (np.nan, np.inf, -np.inf):
        g = v.copy()
        g[1] = workloads.to_bits(np.array([junk], np.float32), dt)[0]
        g[3] = workloads.to_bits(np.array([junk], np.float32), dt)[0]
        vo, lo = oracle.merge_attn_states_lse_kway(g, s, dt)
        assert np.array_equal(vo, clean_v) and np.array_equal(lo.view(np.uint32), clean_l.view(np.uint32))
        v64, _ = reference_f64.merge_attn_states_lse_kway(g, s, dt)
        assert np.all(np.isfinite(v64))
    # a single live partition comes back bit for bit
    s1 = np.full_like(s, -np.inf)
    s1[2] = s[2]
    g = np.full_like(v, workloads.to_bits(np.array([np.nan], np.float32), dt)[0])
    g[2] = v[2]
    vo, lo = oracle.merge_attn_states_lse_kway(g, s1, dt)
    assert np.array_equal(vo & 0x7FFF, v[2] & 0x7FFF) and np.array_equal(lo.view(np.uint32), s[2].view(np.uint32))


def test_binary32_form_is_the_same_operator(oracle):
    """the all-binary32 K-way oracle: attention over the union of K key sets (float64 brute force), K = 2 equal to the
    all-binary32 two-way oracle bit for bit, and equal to the 16-bit oracle on values the 16-bit type holds exactly"""
    rng = np.random.default_rng(7)
    D = 8
    for K in (1, 2, 3, 6):
        for trial in range(4):
            q = rng.standard_normal(D) * 2
            sizes = rng.integers(1, 6, K)
            Ks = [rng.standard_normal((n, D)) for n in sizes]
            Vs = [rng.standard_normal((n, D)) for n in sizes]
            parts = [_attention(q, k, v) for k, v in zip(Ks, Vs)]
            vu, su = _attention(q, np.concatenate(Ks), np.concatenate(Vs))
            v_parts = np.stack([p[0] for p in parts]).reshape(K, 1, 1, D).astype(np.float32)
            s_parts = np.array([p[1] for p in parts], np.float32).reshape(K, 1, 1)
            vo, lo = oracle.merge_attn_states_lse_kway_f32(v_parts, s_parts)
            np.testing.assert_allclose(vo[0, 0], vu, rtol=0, atol=3e-6)
            np.testing.assert_allclose(lo[0, 0], su, rtol=0, atol=3e-6)
    va, la, vb, lb = workloads.merge_inputs(11, 3, 24, "f32", np.random.default_rng(8), empty_p=0.2)
    v2, l2 = oracle.merge_attn_states_lse_f32(va, la, vb, lb)
    vk, lk = oracle.merge_attn_states_lse_kway_f32(np.stack([va, vb]), np.stack([la, lb]))
    assert np.array_equal(np.abs(vk).view(np.uint32), np.abs(v2).view(np.uint32)) and np.array_equal(lk.view(np.uint32), l2.view(np.uint32))
    # against the 16-bit form: same arithmetic before the final rounding
    v16, s16 = np.stack([workloads.merge_inputs(5, 2, 16, "bf16", rng, empty_p=0.2)[0] for _ in range(4)]), rng.uniform(-5, 15, (4, 5, 2)).astype(np.float32)
    s16[1, 0, 0] = -np.inf
    vo16, lo16 = oracle.merge_attn_states_lse_kway(v16, s16, "bf16")
    vo32, lo32 = oracle.merge_attn_states_lse_kway_f32(reference_f64.widen(v16, "bf16").astype(np.float32), s16)
    assert np.array_equal(workloads.to_bits(vo32, "bf16") & 0x7FFF, vo16 & 0x7FFF) and np.array_equal(lo32.view(np.uint32), lo16.view(np.uint32))
    # garbage in empty partitions
    g = np.stack([va, np.full_like(va, np.nan)])
    vo, lo = oracle.merge_attn_states_lse_kway_f32(g, np.stack([la, np.full_like(la, -np.inf)]))
    live = ~np.isneginf(la)
    assert np.array_equal(vo[live].view(np.uint32), va[live].view(np.uint32)) and np.all(vo[~live] == 0)
