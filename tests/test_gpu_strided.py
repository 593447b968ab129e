"""Row-strided / out-of-place fused_add_rmsnorm (include/astra_strided.h): same bars as the in-place operator."""
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
    (5, 4096, (4096 + 3, 4096 + 8, 4096 + 8, 4096 + 8), 0),        # odd stride: element-wise path
    (5, 4100, (4100 + 4, 4100, 4111, 4100 + 1), 1),                # odd everything
    (1, 4096, (4096, 4096, 4096, 4096), 0),
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
