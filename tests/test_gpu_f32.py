"""Parity of the binary32 storage type (ASTRA_F32, a boundary convenience) against the CPU oracle.

The oracle's all-binary32 forms (``oracle_*_f32``, pinned by the same closed forms as the 16-bit forms) take
and return float32 arrays; the float64 definitions bound both.  Bars: the residual of fused_add_rmsnorm is
bit-exact (one binary32 add, stored unrounded); every other output within rtol 1e-4 / atol 1e-6 (derived
from the arithmetic in tests/util.py); lse within 1e-4.  The K-way merge is compared with its own binary32 oracle,
with the float64 definition and, at K = 2, with the two-way oracle.
"""
import os

import numpy as np
import pytest
import torch

import oracle as O
from oracle import reference_f64
import workloads
from tests.gpu_util import (assert_lse_close, assert_storage_close, assert_storage_close_to_real, canaries_intact,
                            padded, to_bits, to_dev)
from tests.util import assert_bits_equal

pytestmark = pytest.mark.gpu
DT = "f32"


@pytest.fixture(scope="module")
def A():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2509_07506_amd as astra

    astra.load_library()
    O.build()
    O.set_threads(min(16, len(os.sched_getaffinity(0))))
    return astra


def _say(msg):
    print(msg, flush=True)


def _rng(*key):
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([7, *key])))


def u32(a):
    return np.ascontiguousarray(a, np.float32).view(np.uint32)


def check_rmsnorm(A, x, r, w, eps, what):
    xd, rd, wd = to_dev(x, DT), to_dev(r, DT), to_dev(w, DT)
    A.fused_add_rmsnorm(xd, rd, wd, eps)
    torch.cuda.synchronize()
    y, res = to_bits(xd), to_bits(rd)
    s_ref, y_ref = O.fused_add_rmsnorm_f32(x, r, w, eps)
    assert_bits_equal(u32(res), u32(s_ref), f"{what}: residual (bit-exact)")
    assert_storage_close(y, y_ref, DT, f"{what}: normalised output")
    y64, _ = reference_f64.fused_add_rmsnorm(x, r, w, eps, DT)
    assert_storage_close_to_real(y, y64, DT, f"{what}: normalised output vs float64")


@pytest.mark.parametrize("T,H", [(1, 4), (2, 64), (5, 512), (3, 516), (300, 1024), (700, 4096), (40, 8192), (600, 8192),
                                 (1000, 32), (333, 68), (50, 128),             # short rows: several rows per workgroup
                                 (140001, 32), (40000, 128),                   # ... in single-wave workgroups on streaming grids
                                 (9, 16384), (520, 11008), (1024, 4096), (1050, 2048), (1030, 6144),  # last three: paced grids
                                 (4100, 8192),                                   # 32 KiB rows, streaming: one resident workgroup
                                 (2, 32768),                                     # beyond 4096 vectors: element-wise path
                                 (7, 4099), (3, 6), (300, 2050)])                # H % 4 != 0: phased path (aligned chunks)
def test_rmsnorm_tiles(A, T, H):
    plan = A.astra_plan_fused_add_rmsnorm(T, H, True, dtype=A.ASTRA_F32)[1].as_dict()
    _say(f"[f32] rmsnorm T={T} H={H} plan={plan}")
    assert plan["path"] == ("generic" if H > 16384 or H < 4 else "vector" if H % 4 == 0 else "phased")
    x, r, w = workloads.rmsnorm_inputs(T, H, DT, _rng(1, T, H), r_std=2.0)
    check_rmsnorm(A, x, r, w, 1e-5, f"rmsnorm f32 T={T} H={H}")


def test_rmsnorm_unaligned_and_canaries(A):
    T, H = 33, 1032
    x, r, w = workloads.rmsnorm_inputs(T, H, DT, _rng(2))
    s_ref, y_ref = O.fused_add_rmsnorm_f32(x, r, w, 1e-6)
    for off in (0, 1, 6, 31):       # 16-byte aligned; shifted by one element (4-byte aligned); by more than a vector
        _say(f"[f32] rmsnorm canaries offset={off}")
        xv, xw = padded(x, DT, offset_elems=off)
        rv, rw = padded(r, DT, offset_elems=off)
        wv, ww = padded(w, DT, offset_elems=off)
        A.fused_add_rmsnorm(xv, rv, wv, 1e-6)
        torch.cuda.synchronize()
        assert_bits_equal(u32(to_bits(rv)), u32(s_ref), f"offset {off}: residual")
        assert_storage_close(to_bits(xv), y_ref, DT, f"offset {off}: y")
        assert canaries_intact(xw, x.size, offset_elems=off) and canaries_intact(rw, r.size, offset_elems=off)
        assert canaries_intact(ww, w.size, offset_elems=off)
        assert_bits_equal(u32(to_bits(wv)), u32(w), "weight untouched")


@pytest.mark.parametrize("T,d", [(1, 128), (3, 1412), (257, 1408), (64, 8192), (700, 5120), (5, 130), (4, 7), (9, 96),
                                 (333, 4), (50, 88),
                                 (1100, 4096)])            # streaming grid: single-wave workgroups, XCD-aware order
def test_silu_tiles(A, T, d):
    plan = A.astra_plan_silu_and_mul(T, d, True, dtype=A.ASTRA_F32)[1].as_dict()
    _say(f"[f32] silu T={T} d={d} plan={plan}")
    a = workloads.silu_inputs(T, d, DT, _rng(3, T, d))
    ad = to_dev(a, DT)
    out = torch.empty((T, d), dtype=torch.float32, device="cuda")
    A.silu_and_mul(out, ad)
    torch.cuda.synchronize()
    got = to_bits(out)
    assert_storage_close(got, O.silu_and_mul_f32(a), DT, "silu f32")
    assert_storage_close_to_real(got, reference_f64.silu_and_mul(a, DT), DT, "silu f32 vs float64")
    assert_bits_equal(u32(to_bits(ad)), u32(a), "input untouched")


@pytest.mark.parametrize("T,d,off", [(3, 1412, 1), (257, 1408, 3), (5, 4, 2), (64, 8192, 5), (9, 96, 33), (7, 130, 1)])
def test_silu_and_merge_behind_offset_pointers(A, T, d, off):
    """binary32 tensors that start `off` elements into a canary-filled buffer, all of a call alike: the chunked paths
    with four elements per chunk (the last case has rows that are no whole number of vectors)"""
    plan = A.astra_plan_silu_and_mul(T, d, 2 if off % 4 else 1, dtype=A.ASTRA_F32)[1].as_dict()
    _say(f"[f32] silu offset T={T} d={d} off={off} plan={plan}")
    assert plan["path"] == ("vector" if d % 4 == 0 and off % 4 == 0 else "phased" if d >= 32 else "ragged")
    a = workloads.silu_inputs(T, d, DT, _rng(31, T, d, off))
    ad, aw = padded(a, DT, offset_elems=off)
    od, ow = padded(np.zeros((T, d), np.float32), DT, offset_elems=off)
    A.silu_and_mul(od, ad)
    torch.cuda.synchronize()
    assert_storage_close(to_bits(od), O.silu_and_mul_f32(a), DT, "silu f32 offset")
    assert canaries_intact(ow, T * d, offset_elems=off) and canaries_intact(aw, a.size, offset_elems=off)
    assert_bits_equal(u32(to_bits(ad)), u32(a), "input untouched")
    # the same shape as a merge: T x 3 pairs of d elements
    va, la, vb, lb = workloads.merge_inputs(T, 3, d, DT, _rng(32, T, d, off), empty_p=0.1)
    (vad, vaw), (vbd, vbw) = padded(va, DT, offset_elems=off), padded(vb, DT, offset_elems=off)
    vo, vow = padded(np.zeros((T, 3, d), np.float32), DT, offset_elems=off)
    lad, lbd = torch.from_numpy(la).cuda(), torch.from_numpy(lb).cuda()
    lo = torch.empty_like(lad)
    A.merge_attn_states_lse(vo, lo, vad, lad, vbd, lbd)
    torch.cuda.synchronize()
    vo_ref, lo_ref = O.merge_attn_states_lse_f32(va, la, vb, lb)
    assert_storage_close(to_bits(vo), vo_ref, DT, "merge f32 offset v_out")
    assert_lse_close(lo.cpu().numpy(), lo_ref, "merge f32 offset lse")
    assert canaries_intact(vow, va.size, offset_elems=off) and canaries_intact(vaw, va.size, offset_elems=off)
    assert canaries_intact(vbw, vb.size, offset_elems=off)


def test_silu_special_values(A):
    d = 128
    xs = np.array([0.0, -0.0, 1.0, -1.0, 20.0, -20.0, 88.0, -88.0, -89.0, -104.0, 3e38, -3e38, 1e-40, -1e-40, 100.0,
                   -1.2784645], np.float32)
    x = np.resize(xs, d).astype(np.float32)
    g = np.resize(np.array([1.0, -2.5, 0.0, 3e10, 1e-30], np.float32), d)
    a = np.concatenate([x, g])[None, :]
    ad = to_dev(a, DT)
    out = torch.empty((1, d), dtype=torch.float32, device="cuda")
    A.silu_and_mul(out, ad)
    torch.cuda.synchronize()
    got = to_bits(out)
    assert_storage_close(got, O.silu_and_mul_f32(a), DT, "silu f32 specials")
    assert_storage_close_to_real(got, reference_f64.silu_and_mul(a, DT), DT, "silu f32 specials vs float64")


def run_merge(A, va, la, vb, lb):
    vad, vbd = to_dev(va, DT), to_dev(vb, DT)
    lad, lbd = torch.from_numpy(la).cuda(), torch.from_numpy(lb).cuda()
    vo, lo = torch.empty_like(vad), torch.empty_like(lad)
    A.merge_attn_states_lse(vo, lo, vad, lad, vbd, lbd)
    torch.cuda.synchronize()
    return to_bits(vo), lo.cpu().numpy()


@pytest.mark.parametrize("T,NH,D", [(1, 1, 4), (3, 40, 64), (257, 40, 256), (600, 32, 128), (5, 7, 36), (4, 3, 6), (2, 5, 1),
                                    (1100, 32, 128)])      # streaming grid: single-wave workgroups, XCD-aware order
def test_merge_tiles(A, T, NH, D):
    plan = A.astra_plan_merge_attn_states_lse(T, NH, D, True, dtype=A.ASTRA_F32)[1].as_dict()
    _say(f"[f32] merge T={T} NH={NH} D={D} plan={plan}")
    assert plan["path"] == ("vector" if D % 4 == 0 else "phased" if D >= 4 else "ragged")
    va, la, vb, lb = workloads.merge_inputs(T, NH, D, DT, _rng(4, T, NH, D), empty_p=0.1)
    vo, lo = run_merge(A, va, la, vb, lb)
    vo_ref, lo_ref = O.merge_attn_states_lse_f32(va, la, vb, lb)
    assert_storage_close(vo, vo_ref, DT, "merge f32 v_out")
    assert_lse_close(lo, lo_ref, "merge f32 lse")
    v64, l64 = reference_f64.merge_attn_states_lse(va, la, vb, lb, DT)
    assert_storage_close_to_real(vo, v64, DT, "merge f32 v_out vs float64")
    assert_lse_close(lo, l64, "merge f32 lse vs float64")
    # one empty side returns the other side bit for bit; two empty sides give 0 and -inf
    ea, eb = np.isneginf(la), np.isneginf(lb)
    only_a, only_b, none = ~ea & eb, ea & ~eb, ea & eb
    assert np.array_equal(u32(vo[only_a]), u32(va[only_a])) and np.array_equal(u32(lo[only_a]), u32(la[only_a]))
    assert np.array_equal(u32(vo[only_b]), u32(vb[only_b])) and np.array_equal(u32(lo[only_b]), u32(lb[only_b]))
    assert np.all(vo[none] == 0.0) and np.all(np.isneginf(lo[none]))


@pytest.mark.parametrize("K", [1, 2, 3, 5, 8])
@pytest.mark.parametrize("T,NH,D", [(37, 8, 128), (5, 3, 6)])
def test_merge_kway(A, K, T, NH, D):
    _say(f"[f32] kway K={K} T={T} NH={NH} D={D}")
    g = _rng(5, K, T, NH, D)
    v = g.standard_normal((K, T, NH, D), dtype=np.float32)
    s = g.uniform(-5.0, 15.0, size=(K, T, NH)).astype(np.float32)
    s[g.random((K, T, NH)) < 0.2] = -np.inf
    vd, sd = to_dev(v, DT), torch.from_numpy(s).cuda()
    vo = torch.empty((T, NH, D), dtype=torch.float32, device="cuda")
    lo = torch.empty((T, NH), dtype=torch.float32, device="cuda")
    A.merge_attn_states_lse_kway(vo, lo, vd, sd)
    torch.cuda.synchronize()
    vref, lref = O.merge_attn_states_lse_kway_f32(v, s)
    assert_storage_close(to_bits(vo), vref, DT, "kway f32 v_out vs the binary32 oracle")
    assert_lse_close(lo.cpu().numpy(), lref, "kway f32 lse vs the binary32 oracle")
    v64, l64 = reference_f64.merge_attn_states_lse_kway(v, s, DT)
    assert_storage_close_to_real(to_bits(vo), v64, DT, "kway f32 v_out vs float64")
    assert_lse_close(lo.cpu().numpy(), l64, "kway f32 lse vs float64")
    if K == 2:
        v2, l2 = O.merge_attn_states_lse_f32(v[0], s[0], v[1], s[1])
        assert_storage_close(to_bits(vo), v2, DT, "kway f32 K=2 vs two-way oracle")
        assert_lse_close(lo.cpu().numpy(), l2, "kway f32 K=2 lse")
    if K == 1:
        live = ~np.isneginf(s[0])
        assert np.array_equal(u32(to_bits(vo)[live]), u32(v[0][live]))


def test_strided_out_of_place(A):
    T, H, S = 19, 1024, 1536
    x, r, w = workloads.rmsnorm_inputs(T, H, DT, _rng(6))
    s_ref, y_ref = O.fused_add_rmsnorm_f32(x, r, w, 1e-6)
    canary = 12345.0
    bufs = [torch.full((T, S), canary, dtype=torch.float32, device="cuda") for _ in range(4)]
    xs, rs, ys, ro = (b[:, 256:256 + H] for b in bufs)
    xs.copy_(torch.from_numpy(x))
    rs.copy_(torch.from_numpy(r))
    A.fused_add_rmsnorm_strided(ys, ro, xs, rs, to_dev(w, DT), 1e-6)
    torch.cuda.synchronize()
    assert_bits_equal(u32(ro.cpu().numpy()), u32(s_ref), "strided f32 residual")
    assert_storage_close(np.ascontiguousarray(ys.cpu().numpy()), y_ref, DT, "strided f32 y")
    assert_bits_equal(u32(xs.cpu().numpy()), u32(x), "x untouched")
    for b in bufs:
        host = b.cpu().numpy()
        assert np.all(host[:, :256] == canary) and np.all(host[:, 256 + H:] == canary)


def test_ablation_variants_are_16_bit_only(A):
    x = torch.zeros((4, 1024), dtype=torch.float32, device="cuda")
    r = torch.zeros_like(x)
    w = torch.ones(1024, dtype=torch.float32, device="cuda")
    st = A.astra_ablation_fused_add_rmsnorm(x.data_ptr(), r.data_ptr(), w.data_ptr(), 4, 1024, A.ASTRA_F32, 1e-6,
                                            A.ASTRA_VARIANT_SCALAR_LOADS, None)
    assert st == A.ASTRA_ERR_VARIANT
    st = A.astra_ablation_fused_add_rmsnorm(x.data_ptr(), r.data_ptr(), w.data_ptr(), 4, 1024, A.ASTRA_F32, 1e-6,
                                            A.ASTRA_VARIANT_TUNED, None)
    torch.cuda.synchronize()
    assert st == 0


def test_element_wise_variant(A):
    """ASTRA_VARIANT_ELEMENT_WISE (include/astra_ablation.h) also takes binary32 storage."""
    v, code, st = A.ASTRA_VARIANT_ELEMENT_WISE, A.ASTRA_F32, torch.cuda.current_stream().cuda_stream
    for T, H in [(5, 516), (33, 4099), (2, 40000)]:
        x, r, w = workloads.rmsnorm_inputs(T, H, DT, _rng(20, T, H), r_std=2.0)
        xd, rd, wd = to_dev(x, DT), to_dev(r, DT), to_dev(w, DT)
        assert A.astra_ablation_fused_add_rmsnorm(xd.data_ptr(), rd.data_ptr(), wd.data_ptr(), T, H, code, 1e-5, v, st) == 0
        torch.cuda.synchronize()
        s_ref, y_ref = O.fused_add_rmsnorm_f32(x, r, w, 1e-5)
        assert_bits_equal(u32(to_bits(rd)), u32(s_ref), "element-wise rmsnorm: residual (bit-exact)")
        assert_storage_close(to_bits(xd), y_ref, DT, "element-wise rmsnorm: normalised output")
    for T, d in [(7, 1412), (3, 101)]:
        a = workloads.silu_inputs(T, d, DT, _rng(21, T, d))
        ad = to_dev(a, DT)
        out = torch.empty((T, d), dtype=torch.float32, device="cuda")
        assert A.astra_ablation_silu_and_mul(out.data_ptr(), ad.data_ptr(), T, d, code, v, st) == 0
        torch.cuda.synchronize()
        assert_storage_close(to_bits(out), O.silu_and_mul_f32(a), DT, "element-wise silu")
    for T, NH, D in [(9, 8, 128), (5, 7, 37)]:
        va, la, vb, lb = workloads.merge_inputs(T, NH, D, DT, _rng(22, T, NH, D), empty_p=0.1)
        vad, vbd = to_dev(va, DT), to_dev(vb, DT)
        lad, lbd = torch.from_numpy(la).cuda(), torch.from_numpy(lb).cuda()
        vo, lo = torch.empty_like(vad), torch.empty_like(lad)
        assert A.astra_ablation_merge_attn_states_lse(vo.data_ptr(), lo.data_ptr(), vad.data_ptr(), lad.data_ptr(), vbd.data_ptr(),
                                                      lbd.data_ptr(), T, NH, D, code, v, st) == 0
        torch.cuda.synchronize()
        vo_ref, lo_ref = O.merge_attn_states_lse_f32(va, la, vb, lb)
        assert_storage_close(to_bits(vo), vo_ref, DT, "element-wise merge: v_out")
        assert_lse_close(lo.cpu().numpy(), lo_ref, "element-wise merge: lse_out")
