"""The strided entry points (include/astra_strided.h): row-strided / out-of-place fused_add_rmsnorm, row-strided
silu_and_mul, merge_attn_states_lse with token and head strides; same bars as the dense operators."""
import os

import numpy as np
import pytest
import torch

import oracle as O
import workloads
from tests.gpu_util import TORCH_DT, assert_storage_close, to_bits, to_dev
from tests.util import assert_bits_equal

pytestmark = pytest.mark.gpu
CANARY = 0x7BCD


@pytest.fixture(scope="module")
def A():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2509_07506_amd as astra

    astra.load_library()
    O.build()
    O.set_threads(min(16, len(os.sched_getaffinity(0))))
    return astra


def _wide(bits, dt, stride, col0):
    """places a [T,H] tensor as a view into a canary-filled [T, stride] buffer starting at column col0"""
    T, H = bits.shape
    whole = torch.full((T, stride), CANARY, dtype=torch.int16).view(TORCH_DT[dt]).cuda()
    view = whole[:, col0:col0 + H]
    view.copy_(to_dev(bits, dt))
    return view, whole


def _gaps_intact(whole, col0, H):
    w = whole.view(torch.int16).cpu().numpy().view(np.uint16)
    return bool(np.all(w[:, :col0] == CANARY) and np.all(w[:, col0 + H:] == CANARY))


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("T,H,strides,col0", [
    (7, 4096, (4096 + 64, 4096 + 8, 8192, 4096 + 128), 0),        # fast path: strides and offsets multiples of 8
    (300, 5120, (5120 + 8, 5120 + 8, 5120 + 8, 5120 + 8), 8),
    (33, 11008, (11008 + 16, 11008, 11008 + 24, 22016), 0),        # long rows (4 vectors per lane)
    (1280, 4096, (4096 + 8, 4096 + 16, 4096 + 8, 4096), 0),        # half-sized workgroups, two vectors per lane
    (300, 128, (128 + 8, 128, 128 + 16, 128 + 8), 0),              # short rows: several rows per workgroup
    (77, 64, (64, 64 + 8, 64 + 8, 64 + 24), 8),
    (140001, 64, (64 + 8, 64, 64 + 16, 64 + 8), 0),                # ... in single-wave workgroups on a streaming grid
    (700, 8192, (8192 + 8, 8192, 8192 + 8, 8192 + 8), 8),          # x requested before r
    (1100, 2048, (2048 + 64, 2048 + 8, 2048, 2048 + 8), 0),        # launch order in chunks
    (5, 4096, (4096 + 3, 4096 + 8, 4096 + 8, 4096 + 8), 0),        # odd stride: ragged path
    (5, 4100, (4100 + 4, 4100, 4111, 4100 + 1), 1),                # odd everything
    (270, 5124, (5124 + 5, 5124 + 1, 5124, 5124 + 3), 3),
    (3, 33000, (33000 + 1, 33000, 33000 + 7, 33000), 0),           # more than 4096 vectors: element-wise path
    (1, 4096, (4096, 4096, 4096, 4096), 0),
    (4096, 14336, (14336 + 8, 14336, 14336 + 16, 14336 + 8), 0),   # long rows on a streaming grid: one resident workgroup
])
def test_strided_out_of_place(A, T, H, strides, col0, dt):
    print(f"[strided] T={T} H={H} strides={strides} col0={col0} {dt}", flush=True)
    x, r, w = workloads.rmsnorm_inputs(T, H, dt, np.random.default_rng([70, T, H, col0]), r_std=2.0)
    ys, ros, xs, rs = (s + col0 for s in strides)
    xv, xw = _wide(x, dt, xs, col0)
    rv, rw = _wide(r, dt, rs, col0)
    yv, yw = _wide(np.full((T, H), 0x1234, np.uint16), dt, ys, col0)
    rov, row = _wide(np.full((T, H), 0x1234, np.uint16), dt, ros, col0)
    wd = to_dev(w, dt)
    A.fused_add_rmsnorm_strided(yv, rov, xv, rv, wd, 1e-5)
    torch.cuda.synchronize()
    y_ref, res_ref = O.fused_add_rmsnorm(x, r, w, 1e-5, dt)
    assert_bits_equal(to_bits(rov.contiguous()), res_ref, "r_out (bit-exact)")
    assert_storage_close(to_bits(yv.contiguous()), y_ref, dt, "y_out")
    assert np.array_equal(to_bits(xv.contiguous()), x) and np.array_equal(to_bits(rv.contiguous()), r), "inputs must be untouched"
    for whole in (xw, rw, yw, row):
        assert _gaps_intact(whole, col0, H)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_strided_in_place_equals_the_plain_operator(A, dt):
    T, H, stride = 129, 8192, 8192 + 64
    x, r, w = workloads.rmsnorm_inputs(T, H, dt, np.random.default_rng(71), r_std=2.0)
    xv, xw = _wide(x, dt, stride, 0)
    rv, rw = _wide(r, dt, stride, 0)
    wd = to_dev(w, dt)
    A.fused_add_rmsnorm_strided(xv, rv, xv, rv, wd, 1e-5)            # outputs are the input views: in place
    xd, rd = to_dev(x, dt), to_dev(r, dt)
    A.fused_add_rmsnorm(xd, rd, wd, 1e-5)
    torch.cuda.synchronize()
    assert np.array_equal(to_bits(xv.contiguous()), to_bits(xd)) and np.array_equal(to_bits(rv.contiguous()), to_bits(rd))
    y_ref, res_ref = O.fused_add_rmsnorm(x, r, w, 1e-5, dt)
    assert_bits_equal(to_bits(rv.contiguous()), res_ref, "residual")
    assert _gaps_intact(xw, 0, H) and _gaps_intact(rw, 0, H)


def test_strided_validation(A):
    buf = torch.zeros(1 << 16, dtype=torch.float16, device="cuda")
    p = buf.data_ptr()
    f = A.astra_fused_add_rmsnorm_strided
    y, ro, x, r, w = p, p + 16384, p + 32768, p + 49152, p + 65536
    assert f(y, 4, ro, 16, x, 16, r, 16, w, 4, 8, A.ASTRA_F16, 1e-6, None) == 2          # stride < H
    assert f(y, 16, ro, 16, x, 16, r, 16, w, 4, 8, 9, 1e-6, None) == 3
    assert f(y, 16, ro, 16, x, 16, r, 16, w, 4, 8, A.ASTRA_F16, -1.0, None) == 4
    assert f(y + 1, 16, ro, 16, x, 16, r, 16, w, 4, 8, A.ASTRA_F16, 1e-6, None) == 5
    assert f(x, 24, ro, 16, x, 16, r, 16, w, 4, 8, A.ASTRA_F16, 1e-6, None) == 6         # y_out on x with another stride
    assert f(y, 16, y + 8, 16, x, 16, r, 16, w, 4, 8, A.ASTRA_F16, 1e-6, None) == 6      # the two outputs interleave
    assert f(y, 16, ro, 16, x, 16, r, 16, w, 0, 8, A.ASTRA_F16, 1e-6, None) == 0
    torch.cuda.synchronize()
    assert bool((buf == 0).all())


# ---------------------------------------------------------------------------------------------------
# silu_and_mul and merge_attn_states_lse on strided views

from tests.gpu_util import assert_lse_close  # noqa: E402


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("T,d,in_stride,out_stride,col0", [
    (9, 1408, 2 * 1408 + 64, 1408 + 8, 0),          # fast path
    (300, 5120, 2 * 5120 + 8, 5120 + 16, 8),
    (1100, 176, 2 * 176 + 24, 176 + 8, 0),          # short rows
    (5, 1408, 2 * 1408 + 3, 1408 + 8, 0),           # odd stride: ragged path
    (4, 100, 2 * 100 + 1, 100 + 7, 1),              # odd everything
    (270, 1411, 2 * 1411 + 5, 1411 + 3, 3),
    (1, 4096, 2 * 4096, 4096, 0),
    (4100, 2048, 2 * 2048 + 64, 2048 + 8, 0),       # streaming grid: single-wave workgroups, XCD-aware order
    (100, 1024, 2 * 1024 + 8, 1024 + 8, 8),         # fewer 256-lane workgroups than compute units: 128 lanes
])
def test_silu_strided(A, T, d, in_stride, out_stride, col0, dt):
    print(f"[strided] silu T={T} d={d} in_stride={in_stride} out_stride={out_stride} col0={col0} {dt}", flush=True)
    a = workloads.silu_inputs(T, d, dt, np.random.default_rng([71, T, d, col0]))
    av, aw = _wide(a, dt, in_stride + col0, col0)
    ov, ow = _wide(np.full((T, d), 0x1234, np.uint16), dt, out_stride + col0, col0)
    A.silu_and_mul_strided(ov, av)
    torch.cuda.synchronize()
    assert_storage_close(to_bits(ov.contiguous()), O.silu_and_mul(a, dt), dt, "strided silu out")
    assert_bits_equal(to_bits(av.contiguous()), a, "input untouched")
    assert _gaps_intact(ow, col0, d) and _gaps_intact(aw, col0, 2 * d)
    # dense views give what the dense entry point gives, bit for bit
    if in_stride == 2 * d and out_stride == d and col0 == 0:
        dense = torch.empty((T, d), dtype=TORCH_DT[dt], device="cuda")
        A.silu_and_mul(dense, to_dev(a, dt))
        torch.cuda.synchronize()
        assert_bits_equal(to_bits(ov.contiguous()), to_bits(dense), "strided == dense")


def _wide3(bits, dt, head_stride, token_pad, col0):
    """places a [T,NH,D] tensor as a view into a canary-filled [T, NH*head_stride + token_pad] buffer; head h of
    token t starts at column col0 + h*head_stride"""
    T, NH, D = bits.shape
    width = NH * head_stride + token_pad + col0
    whole = torch.full((T, width), CANARY, dtype=torch.int16).view(TORCH_DT[dt]).cuda()
    view = whole[:, col0:col0 + NH * head_stride].view(T, NH, head_stride)[:, :, :D]
    view.copy_(to_dev(bits, dt))
    return view, whole


def _gaps_intact3(whole, NH, D, head_stride, col0):
    w = whole.view(torch.int16).cpu().numpy().view(np.uint16)
    mask = np.ones(w.shape[1], bool)
    for h in range(NH):
        mask[col0 + h * head_stride: col0 + h * head_stride + D] = False
    return bool(np.all(w[:, mask] == CANARY))


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("T,NH,D,head_strides,token_pad,col0", [
    (33, 8, 128, (192, 128, 136), 64, 0),            # fast path: head_dim slices of wider heads
    (300, 40, 64, (64, 72, 64), 0, 8),
    (5, 7, 72, (80, 72, 96), 16, 0),                 # head_dim not a power of two
    (6, 4, 128, (131, 128, 128), 0, 0),              # odd head stride: ragged path
    (3, 5, 36, (40, 37, 36), 3, 1),                  # odd everything
    (70, 9, 100, (103, 100, 109), 5, 3),
    (1, 1, 256, (256, 256, 256), 0, 0),
    (2051, 32, 128, (136, 128, 144), 8, 0),          # streaming grid: single-wave workgroups, XCD-aware order
    (60, 32, 128, (128, 136, 128), 0, 8),            # fewer 256-lane workgroups than compute units: 128 lanes
])
def test_merge_strided(A, T, NH, D, head_strides, token_pad, col0, dt):
    print(f"[strided] merge T={T} NH={NH} D={D} head_strides={head_strides} pad={token_pad} col0={col0} {dt}", flush=True)
    va, la, vb, lb = workloads.merge_inputs(T, NH, D, dt, np.random.default_rng([72, T, NH, D]), empty_p=0.15)
    ho, ha, hb = head_strides
    vav, vaw = _wide3(va, dt, ha, token_pad, col0)
    vbv, vbw = _wide3(vb, dt, hb, token_pad, col0)
    vov, vow = _wide3(np.full((T, NH, D), 0x1234, np.uint16), dt, ho, token_pad, col0)
    lad, lbd = torch.from_numpy(la).cuda(), torch.from_numpy(lb).cuda()
    lo = torch.empty_like(lad)
    A.merge_attn_states_lse_strided(vov, lo, vav, lad, vbv, lbd)
    torch.cuda.synchronize()
    vo_ref, lo_ref = O.merge_attn_states_lse(va, la, vb, lb, dt)
    assert_storage_close(to_bits(vov.contiguous()), vo_ref, dt, "strided merge v_out")
    assert_lse_close(lo.cpu().numpy(), lo_ref, "strided merge lse_out")
    assert_bits_equal(to_bits(vav.contiguous()), va, "v_a untouched")
    assert_bits_equal(to_bits(vbv.contiguous()), vb, "v_b untouched")
    assert _gaps_intact3(vow, NH, D, ho, col0) and _gaps_intact3(vaw, NH, D, ha, col0)
    # in place on v_a (the very same view).  The two calls may take different kernels (the output view of the first one
    # can have another stride); every merge kernel forms the blend as the same explicit fused multiply-add, so the
    # results are the same bits all the same
    first = to_bits(vov.contiguous())
    A.merge_attn_states_lse_strided(vav, lo, vav, lad, vbv, lbd)
    torch.cuda.synchronize()
    assert_storage_close(to_bits(vav.contiguous()), vo_ref, dt, "in place on v_a")
    assert_bits_equal(to_bits(vav.contiguous()), first, "in place on v_a: same bits as out of place")
    assert_lse_close(lo.cpu().numpy(), lo_ref, "in place on v_a: lse_out")
    assert _gaps_intact3(vaw, NH, D, ha, col0)


def test_merge_strided_dense_views_equal_the_dense_entry_point(A):
    T, NH, D, dt = 65, 16, 128, "bf16"
    va, la, vb, lb = workloads.merge_inputs(T, NH, D, dt, np.random.default_rng(73))
    vad, vbd = to_dev(va, dt), to_dev(vb, dt)
    lad, lbd = torch.from_numpy(la).cuda(), torch.from_numpy(lb).cuda()
    o1, l1, o2, l2 = torch.empty_like(vad), torch.empty_like(lad), torch.empty_like(vad), torch.empty_like(lad)
    A.merge_attn_states_lse(o1, l1, vad, lad, vbd, lbd)
    A.merge_attn_states_lse_strided(o2, l2, vad, lad, vbd, lbd)
    torch.cuda.synchronize()
    assert_bits_equal(to_bits(o1), to_bits(o2), "v_out")
    assert np.array_equal(l1.cpu().numpy().view(np.uint32), l2.cpu().numpy().view(np.uint32))
