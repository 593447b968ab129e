"""Seeded random-shape parity sweep: shapes nobody hand-picked, across the vector and element-wise paths of all
operators (including the K-way merge and the strided rmsnorm), each against the oracle to the operators' bars."""
import os

import numpy as np
import pytest
import torch

import oracle as O
import workloads
from tests.gpu_util import TORCH_DT, assert_lse_close, assert_storage_close, to_bits, to_dev
from tests.util import assert_bits_equal

pytestmark = pytest.mark.gpu
N_CASES = 48


@pytest.fixture(scope="module")
def A():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2509_07506_amd as astra

    astra.load_library()
    O.build()
    O.set_threads(min(16, len(os.sched_getaffinity(0))))
    return astra


def _pick(rng, choices):
    return choices[int(rng.integers(len(choices)))]


def _row_len(rng, cap):
    """row lengths: mostly multiples of 8 (fast path), sometimes arbitrary (element-wise path)"""
    kind = rng.integers(4)
    if kind == 0:
        return int(rng.integers(1, cap + 1))
    if kind == 1:
        return int(_pick(rng, [64, 128, 256, 512, 1024, 2048, 4096, 5120, 8192]))
    return 8 * int(rng.integers(1, cap // 8 + 1))


def test_rmsnorm_random_shapes(A):
    rng = np.random.default_rng(9001)
    for i in range(N_CASES):
        T, H = int(rng.integers(1, 70)), _row_len(rng, 20000)
        if i % 4 == 3:
            T = int(rng.integers(1024, 1300))      # streaming grids: the paced forms of the row kernel
        dt = _pick(rng, ["bf16", "f16"])
        eps = float(_pick(rng, [0.0, 1e-6, 1e-5, 1e-2]))
        print(f"[random] rmsnorm #{i} T={T} H={H} {dt} eps={eps}", flush=True)
        x, r, w = workloads.rmsnorm_inputs(T, H, dt, rng, r_std=float(_pick(rng, [1.0, 2.0])))
        xd, rd, wd = to_dev(x, dt), to_dev(r, dt), to_dev(w, dt)
        A.fused_add_rmsnorm(xd, rd, wd, eps)
        torch.cuda.synchronize()
        y_ref, res_ref = O.fused_add_rmsnorm(x, r, w, eps, dt)
        assert_bits_equal(to_bits(rd), res_ref, f"#{i} residual T={T} H={H} {dt}")
        assert_storage_close(to_bits(xd), y_ref, dt, f"#{i} y T={T} H={H} {dt}")


def test_rmsnorm_strided_random_shapes(A):
    rng = np.random.default_rng(9002)
    for i in range(N_CASES // 2):
        T, H = int(rng.integers(1, 40)), _row_len(rng, 12000)
        dt = _pick(rng, ["bf16", "f16"])
        pad = [int(_pick(rng, [0, 8, 16, 3, 64])) for _ in range(4)]
        print(f"[random] strided #{i} T={T} H={H} {dt} pads={pad}", flush=True)
        x, r, w = workloads.rmsnorm_inputs(T, H, dt, rng)
        bufs = [torch.zeros((T, H + p), dtype=TORCH_DT[dt], device="cuda") for p in pad]
        yv, rov, xv, rv = (b[:, :H] for b in bufs)
        xv.copy_(to_dev(x, dt))
        rv.copy_(to_dev(r, dt))
        A.fused_add_rmsnorm_strided(yv, rov, xv, rv, to_dev(w, dt), 1e-5)
        torch.cuda.synchronize()
        y_ref, res_ref = O.fused_add_rmsnorm(x, r, w, 1e-5, dt)
        assert_bits_equal(to_bits(rov.contiguous()), res_ref, f"#{i} r_out")
        assert_storage_close(to_bits(yv.contiguous()), y_ref, dt, f"#{i} y_out")
        for b, p in zip(bufs[:2], pad[:2]):
            assert p == 0 or bool((b[:, H:] == 0).all()), "gap between rows was written"


def test_silu_random_shapes(A):
    rng = np.random.default_rng(9003)
    for i in range(N_CASES):
        T, d = int(rng.integers(1, 70)), _row_len(rng, 16000)
        dt = _pick(rng, ["bf16", "f16"])
        print(f"[random] silu #{i} T={T} d={d} {dt}", flush=True)
        a = workloads.silu_inputs(T, d, dt, rng)
        ad = to_dev(a, dt)
        out = torch.empty((T, d), dtype=TORCH_DT[dt], device="cuda")
        A.silu_and_mul(out, ad)
        torch.cuda.synchronize()
        assert_storage_close(to_bits(out), O.silu_and_mul(a, dt), dt, f"#{i} silu T={T} d={d} {dt}")


def test_merge_random_shapes(A):
    rng = np.random.default_rng(9004)
    for i in range(N_CASES):
        T, NH = int(rng.integers(1, 40)), int(rng.integers(1, 48))
        D = int(_pick(rng, [8, 16, 32, 64, 72, 80, 96, 128, 192, 256, 4, 100, 1, 24, 40, 512]))
        dt = _pick(rng, ["bf16", "f16"])
        print(f"[random] merge #{i} T={T} NH={NH} D={D} {dt}", flush=True)
        va, la, vb, lb = workloads.merge_inputs(T, NH, D, dt, rng, empty_p=float(_pick(rng, [0.0, 0.01, 0.3])))
        vad, vbd = to_dev(va, dt), to_dev(vb, dt)
        lad, lbd = torch.from_numpy(la).cuda(), torch.from_numpy(lb).cuda()
        vo, lo = torch.empty_like(vad), torch.empty_like(lad)
        A.merge_attn_states_lse(vo, lo, vad, lad, vbd, lbd)
        torch.cuda.synchronize()
        vo_ref, lo_ref = O.merge_attn_states_lse(va, la, vb, lb, dt)
        assert_storage_close(to_bits(vo), vo_ref, dt, f"#{i} v_out")
        assert_lse_close(lo.cpu().numpy(), lo_ref, f"#{i} lse_out")


def test_merge_kway_random_shapes(A):
    rng = np.random.default_rng(9005)
    for i in range(N_CASES // 2):
        K, T, NH = int(rng.integers(1, 12)), int(rng.integers(1, 24)), int(rng.integers(1, 20))
        D = int(_pick(rng, [8, 64, 72, 128, 256, 4, 100]))
        dt = _pick(rng, ["bf16", "f16"])
        print(f"[random] kway #{i} K={K} T={T} NH={NH} D={D} {dt}", flush=True)
        parts = [workloads.merge_inputs(T, NH, D, dt, rng, empty_p=0.2)[:2] for _ in range(K)]
        v, s = np.stack([p[0] for p in parts]), np.stack([p[1] for p in parts])
        vd, sd = to_dev(v, dt), torch.from_numpy(s).cuda()
        vo = torch.empty((T, NH, D), dtype=TORCH_DT[dt], device="cuda")
        lo = torch.empty((T, NH), dtype=torch.float32, device="cuda")
        A.merge_attn_states_lse_kway(vo, lo, vd, sd)
        torch.cuda.synchronize()
        vo_ref, lo_ref = O.merge_attn_states_lse_kway(v, s, dt)
        assert_storage_close(to_bits(vo), vo_ref, dt, f"#{i} v_out")
        assert_lse_close(lo.cpu().numpy(), lo_ref, f"#{i} lse_out")


def test_random_shapes_behind_random_element_offsets(A):
    """every activation tensor of a call starts the same random number of elements (0 to 70: beyond a vector, beyond a
    128-byte line) into a canary-filled buffer: the chunked paths with rows that start anywhere in a line"""
    from tests.gpu_util import canaries_intact, padded

    rng = np.random.default_rng(9006)
    for i in range(N_CASES):
        dt = _pick(rng, ["bf16", "f16"])
        off = int(rng.integers(0, 71))
        kind = i % 3
        if kind == 0:
            T, H = int(rng.integers(1, 300)), _row_len(rng, 12000)
            print(f"[random] offset rmsnorm #{i} T={T} H={H} off={off} {dt}", flush=True)
            x, r, w = workloads.rmsnorm_inputs(T, H, dt, rng, r_std=2.0)
            (xd, xw), (rd, rw), (wd, ww) = (padded(t, dt, offset_elems=off) for t in (x, r, w))
            A.fused_add_rmsnorm(xd, rd, wd, 1e-5)
            torch.cuda.synchronize()
            y_ref, res_ref = O.fused_add_rmsnorm(x, r, w, 1e-5, dt)
            assert_bits_equal(to_bits(rd), res_ref, f"#{i} residual")
            assert_storage_close(to_bits(xd), y_ref, dt, f"#{i} y")
            assert canaries_intact(xw, x.size, offset_elems=off) and canaries_intact(rw, r.size, offset_elems=off)
            assert canaries_intact(ww, w.size, offset_elems=off) and np.array_equal(to_bits(wd), w)
        elif kind == 1:
            T, d = int(rng.integers(1, 300)), _row_len(rng, 12000)
            print(f"[random] offset silu #{i} T={T} d={d} off={off} {dt}", flush=True)
            a = workloads.silu_inputs(T, d, dt, rng)
            ad, aw = padded(a, dt, offset_elems=off)
            od, ow = padded(np.full((T, d), 0x1234, np.uint16), dt, offset_elems=off)
            A.silu_and_mul(od, ad)
            torch.cuda.synchronize()
            assert_storage_close(to_bits(od), O.silu_and_mul(a, dt), dt, f"#{i} silu")
            assert canaries_intact(ow, T * d, offset_elems=off) and canaries_intact(aw, a.size, offset_elems=off)
            assert np.array_equal(to_bits(ad), a)
        else:
            T, NH = int(rng.integers(1, 60)), int(rng.integers(1, 48))
            D = int(_pick(rng, [8, 16, 64, 72, 128, 256, 4, 100, 1, 129, 132, 24]))
            print(f"[random] offset merge #{i} T={T} NH={NH} D={D} off={off} {dt}", flush=True)
            va, la, vb, lb = workloads.merge_inputs(T, NH, D, dt, rng, empty_p=0.05)
            (vad, vaw), (vbd, vbw) = padded(va, dt, offset_elems=off), padded(vb, dt, offset_elems=off)
            vo, vow = padded(np.full((T, NH, D), 0x1234, np.uint16), dt, offset_elems=off)
            lad, lbd = torch.from_numpy(la).cuda(), torch.from_numpy(lb).cuda()
            lo = torch.empty_like(lad)
            A.merge_attn_states_lse(vo, lo, vad, lad, vbd, lbd)
            torch.cuda.synchronize()
            vo_ref, lo_ref = O.merge_attn_states_lse(va, la, vb, lb, dt)
            assert_storage_close(to_bits(vo), vo_ref, dt, f"#{i} v_out")
            assert_lse_close(lo.cpu().numpy(), lo_ref, f"#{i} lse_out")
            assert canaries_intact(vow, va.size, offset_elems=off) and canaries_intact(vaw, va.size, offset_elems=off)
            assert canaries_intact(vbw, vb.size, offset_elems=off)
            assert np.array_equal(to_bits(vad), va) and np.array_equal(to_bits(vbd), vb)
