"""K-way merge (include/astra_kway.h) against its oracle: same bars as the two-way operator."""
import os

import numpy as np
import pytest
import torch

import oracle as O
from oracle import reference_f64
import workloads
from tests.gpu_util import assert_lse_close, assert_storage_close, assert_storage_close_to_real, canaries_intact, padded, to_bits, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def A():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2509_07506_amd as astra

    astra.load_library()
    O.build()
    O.set_threads(min(16, len(os.sched_getaffinity(0))))
    return astra


def _inputs(K, T, NH, D, dt, seed, empty_p=0.1):
    rng = np.random.default_rng([41, K, T, NH, D, seed])
    parts = [workloads.merge_inputs(T, NH, D, dt, rng, empty_p=empty_p)[:2] for _ in range(K)]
    return np.stack([p[0] for p in parts]), np.stack([p[1] for p in parts])


def _run(A, v, s, dt):
    vd = to_dev(v, dt)
    sd = torch.from_numpy(s).cuda()
    K, T, NH, D = v.shape
    vo = torch.empty((T, NH, D), dtype=vd.dtype, device="cuda")
    lo = torch.empty((T, NH), dtype=torch.float32, device="cuda")
    A.merge_attn_states_lse_kway(vo, lo, vd, sd)
    torch.cuda.synchronize()
    return to_bits(vo), lo.cpu().numpy()


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("K,T,NH,D", [(1, 5, 3, 64), (2, 33, 8, 128), (3, 257, 40, 64), (4, 64, 32, 128), (8, 129, 8, 256), (16, 7, 5, 72),
                                      (5, 3, 2, 8), (3, 4, 3, 100), (7, 2, 2, 4), (2, 1, 1, 1024), (32, 16, 4, 128),
                                      (3, 2100, 32, 128),      # streaming grid: single-wave workgroups, XCD-aware order
                                      (2, 20, 32, 128),        # fewer 256-lane workgroups than compute units: 128 lanes
                                      (4, 70, 9, 129), (5, 33, 7, 13), (3, 9, 4, 7), (6, 300, 5, 132)])    # ragged path
def test_kway_matches_oracle(A, K, T, NH, D, dt):
    print(f"[kway] K={K} T={T} NH={NH} D={D} {dt}", flush=True)
    v, s = _inputs(K, T, NH, D, dt, 0)
    two_pairs = T * NH >= 2
    if two_pairs:
        s[:, 0, 0] = -np.inf                                # every partition empty for one pair
    s[1:, -1, -1] = -np.inf                                 # a single live partition for another
    s[0, -1, -1] = 3.25
    vo, lo = _run(A, v, s, dt)
    vo_ref, lo_ref = O.merge_attn_states_lse_kway(v, s, dt)
    assert_storage_close(vo, vo_ref, dt, "v_out")
    assert_lse_close(lo, lo_ref, "lse_out")
    v64, l64 = reference_f64.merge_attn_states_lse_kway(v, s, dt)
    assert_storage_close_to_real(vo, v64, dt, "v_out vs float64")
    assert_lse_close(lo, l64, "lse_out vs float64")
    if two_pairs:
        assert np.all((vo[0, 0] & 0x7FFF) == 0) and np.isneginf(lo[0, 0])
    assert np.array_equal(vo[-1, -1], v[0, -1, -1]) and lo[-1, -1] == np.float32(3.25), "single live partition is returned unchanged"


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_k2_agrees_with_the_two_way_entry_point(A, dt):
    v, s = _inputs(2, 300, 32, 128, dt, 1)
    vo, lo = _run(A, v, s, dt)
    vad, vbd = to_dev(v[0], dt), to_dev(v[1], dt)
    lad, lbd = torch.from_numpy(s[0]).cuda(), torch.from_numpy(s[1]).cuda()
    vo2, lo2 = torch.empty_like(vad), torch.empty_like(lad)
    A.merge_attn_states_lse(vo2, lo2, vad, lad, vbd, lbd)
    torch.cuda.synchronize()
    assert_storage_close(vo, to_bits(vo2), dt, "K=2 vs two-way v_out")
    assert_lse_close(lo, lo2.cpu().numpy(), "K=2 vs two-way lse_out")


def test_kway_canaries_and_unaligned(A):
    dt = "f16"
    for off in (0, 3):
        v, s = _inputs(3, 5, 4, 64, dt, 2)
        vd, vw = padded(v, dt, offset_elems=off)
        od, ow = padded(np.full(v.shape[1:], 0x1234, np.uint16), dt, offset_elems=off)
        sd = torch.from_numpy(s).cuda()
        lo = torch.empty(s.shape[1:], dtype=torch.float32, device="cuda")
        A.merge_attn_states_lse_kway(od, lo, vd, sd)
        torch.cuda.synchronize()
        vo_ref, lo_ref = O.merge_attn_states_lse_kway(v, s, dt)
        assert_storage_close(to_bits(od), vo_ref, dt, f"v_out offset {off}")
        assert_lse_close(lo.cpu().numpy(), lo_ref, "lse_out")
        assert canaries_intact(ow, vo_ref.size, offset_elems=off) and np.array_equal(to_bits(vd), v)


def test_kway_validation(A):
    buf = torch.zeros(1 << 14, dtype=torch.float16, device="cuda")
    f = torch.zeros(1 << 10, dtype=torch.float32, device="cuda")
    p, q = buf.data_ptr(), f.data_ptr()
    g = A.astra_merge_attn_states_lse_kway
    assert g(p, q, p + 8192, q + 1024, 0, 1, 2, 8, A.ASTRA_F16, None) == 2          # K < 1
    assert g(p, q, p + 8192, q + 1024, 1 << 20, 1, 2, 8, A.ASTRA_F16, None) == 2    # K too large
    assert g(p, q, p + 16, q + 1024, 3, 1, 2, 8, A.ASTRA_F16, None) == 6            # v_out inside v_parts
    assert g(p, q + 8, p + 8192, q, 3, 1, 2, 8, A.ASTRA_F16, None) == 6             # lse_out inside lse_parts
    assert g(p, q, p + 8192, q + 1024, 3, 1, 2, 8, 7, None) == 3
    assert g(p, q, p + 8192, q + 1024, 3, 0, 2, 8, A.ASTRA_F16, None) == 0
    torch.cuda.synchronize()
    assert bool((buf == 0).all()) and bool((f == 0).all())


@pytest.mark.parametrize("dt", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("K,D", [(2, 128), (5, 128), (9, 64), (5, 100), (6, 132)])
def test_kway_never_looks_at_an_empty_partition(A, K, D, dt):
    """NaN / inf in the value buffers of partitions whose score is -inf stay out of the result (vector and ragged paths)"""
    print(f"[kway empty] K={K} D={D} {dt}", flush=True)
    T, NH = 19, 4
    v, s = _inputs(K, T, NH, D, dt, 3, empty_p=0.0)
    clean_v = v.copy()
    s[1::2] = -np.inf                                                    # every second partition empty ...
    v[1::2] = workloads.to_bits(np.array([np.nan], np.float32), dt)[0]   # ... and full of NaN
    s[:, 0, 0] = -np.inf
    v[:, 0, 0] = workloads.to_bits(np.array([np.inf], np.float32), dt)[0]  # one pair with nothing live at all
    clean_v[1::2] = 0
    clean_v[:, 0, 0] = 0
    vo, lo = _run(A, v, s, dt)
    w = reference_f64.widen(vo, dt)
    assert np.all(np.isfinite(w)) and np.all(w[0, 0] == 0) and np.isneginf(lo[0, 0])
    if dt == "f32":
        v64, l64 = reference_f64.merge_attn_states_lse_kway(clean_v, s, dt)
        assert_storage_close_to_real(vo, v64, dt, "v_out vs float64")
        assert_lse_close(lo, l64, "lse_out")
    else:
        vo_ref, lo_ref = O.merge_attn_states_lse_kway(v, s, dt)
        assert_storage_close(vo, vo_ref, dt, "v_out")
        assert_lse_close(lo, lo_ref, "lse_out")
