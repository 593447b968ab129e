"""The ablation variants (include/astra_ablation.h) compute the same operators: each is checked against the
oracle to the operators' own bars, on the paper's Table-4 shapes and on shapes that cross tile edges."""
import os

import numpy as np
import pytest
import torch

import oracle as O
import workloads
from tests.gpu_util import TORCH_DT, assert_lse_close, assert_storage_close, to_bits, to_dev
from tests.util import assert_bits_equal

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


def _code(A, dt):
    return A.ASTRA_BF16 if dt == "bf16" else A.ASTRA_F16


def _rmsnorm(A, x, r, w, eps, dt, variant):
    xd, rd, wd = to_dev(x, dt), to_dev(r, dt), to_dev(w, dt)
    T, H = x.shape
    st = A.astra_ablation_fused_add_rmsnorm(xd.data_ptr(), rd.data_ptr(), wd.data_ptr(), T, H, _code(A, dt), eps, variant,
                                            torch.cuda.current_stream().cuda_stream)
    assert st == 0, A.astra_status_string(st)
    torch.cuda.synchronize()
    y_ref, res_ref = O.fused_add_rmsnorm(x, r, w, eps, dt)
    assert_bits_equal(to_bits(rd), res_ref, f"variant {variant}: residual (bit-exact)")
    assert_storage_close(to_bits(xd), y_ref, dt, f"variant {variant}: normalised output")


def _silu(A, a, dt, variant):
    ad = to_dev(a, dt)
    T, d = a.shape[0], a.shape[1] // 2
    out = torch.empty((T, d), dtype=TORCH_DT[dt], device="cuda")
    st = A.astra_ablation_silu_and_mul(out.data_ptr(), ad.data_ptr(), T, d, _code(A, dt), variant,
                                       torch.cuda.current_stream().cuda_stream)
    assert st == 0, A.astra_status_string(st)
    torch.cuda.synchronize()
    assert_storage_close(to_bits(out), O.silu_and_mul(a, dt), dt, f"variant {variant}: out")


def _merge(A, va, la, vb, lb, dt, variant):
    vad, vbd = to_dev(va, dt), to_dev(vb, dt)
    lad, lbd = torch.from_numpy(la).cuda(), torch.from_numpy(lb).cuda()
    vo, lo = torch.empty_like(vad), torch.empty_like(lad)
    T, NH, D = va.shape
    st = A.astra_ablation_merge_attn_states_lse(vo.data_ptr(), lo.data_ptr(), vad.data_ptr(), lad.data_ptr(), vbd.data_ptr(),
                                                lbd.data_ptr(), T, NH, D, _code(A, dt), variant,
                                                torch.cuda.current_stream().cuda_stream)
    assert st == 0, A.astra_status_string(st)
    torch.cuda.synchronize()
    vo_ref, lo_ref = O.merge_attn_states_lse(va, la, vb, lb, dt)
    assert_storage_close(to_bits(vo), vo_ref, dt, f"variant {variant}: v_out")
    assert_lse_close(lo.cpu().numpy(), lo_ref, f"variant {variant}: lse_out")


RMS_VARIANTS = (0, 1, 2)     # tuned, scalar loads, LDS tree reduction
SILU_VARIANTS = (0, 1, 4)    # tuned, scalar loads, libm exp + divide
MERGE_VARIANTS = (0, 1, 3)   # tuned, scalar loads, unhoisted weights


@pytest.mark.parametrize("name", sorted(workloads.PAPER_SHAPE_CASES))
def test_paper_table4_shapes_all_variants(A, name):
    c = workloads.case(name)
    print(f"[ablation] {name}", flush=True)
    data = c.generate()
    if c.kernel == "rmsnorm":
        for v in RMS_VARIANTS:
            _rmsnorm(A, *data, c.eps, c.dtype, v)
    elif c.kernel == "silu":
        for v in SILU_VARIANTS:
            _silu(A, data[0], c.dtype, v)
    else:
        for v in MERGE_VARIANTS:
            _merge(A, *data, c.dtype, v)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("T,H", [(3, 8), (5, 520), (7, 5120), (300, 7168), (2, 8192), (4, 11008), (600, 14336), (3, 16384),
                                 (4096, 14336)])                   # long rows, streaming: one resident workgroup per compute unit
def test_rmsnorm_variants_edge_shapes(A, T, H, dt):
    x, r, w = workloads.rmsnorm_inputs(T, H, dt, np.random.default_rng([31, T, H]), r_std=2.0)
    for v in RMS_VARIANTS[1:]:
        _rmsnorm(A, x, r, w, 1e-5, dt, v)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("T,d", [(1, 256), (3, 264), (7, 1000), (19, 5120), (257, 1408)])
def test_silu_variants_edge_shapes(A, T, d, dt):
    a = workloads.silu_inputs(T, d, dt, np.random.default_rng([32, T, d]))
    a[0, :6] = workloads.to_bits(np.array([-100.0, -89.0, -20.0, 0.0, 20.0, 90.0], np.float32), dt)
    for v in SILU_VARIANTS[1:]:
        _silu(A, a, dt, v)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("T,NH,D", [(1, 1, 8), (7, 3, 72), (9, 8, 80), (257, 40, 64), (33, 32, 128)])
def test_merge_variants_edge_shapes(A, T, NH, D, dt):
    m = workloads.merge_inputs(T, NH, D, dt, np.random.default_rng([33, T, NH, D]), empty_p=0.15)
    for v in MERGE_VARIANTS[1:]:
        _merge(A, *m, dt, v)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_element_wise_variant_on_any_input(A, dt):
    """ASTRA_VARIANT_ELEMENT_WISE: the plain element-wise kernels, which astra.h itself only takes for inputs beyond
    the limits of its other paths, on fast-path, ragged and long-row shapes."""
    v = A.ASTRA_VARIANT_ELEMENT_WISE
    for T, H in [(3, 8), (5, 523), (7, 5120), (40, 8192), (2, 70000), (300, 4099), (4, 1)]:
        print(f"[ablation] element-wise rmsnorm T={T} H={H} {dt}", flush=True)
        x, r, w = workloads.rmsnorm_inputs(T, H, dt, np.random.default_rng([34, T, H]), r_std=2.0)
        _rmsnorm(A, x, r, w, 1e-5, dt, v)
    for T, d in [(1, 256), (3, 263), (19, 5120), (257, 1409), (5, 1)]:
        print(f"[ablation] element-wise silu T={T} d={d} {dt}", flush=True)
        _silu(A, workloads.silu_inputs(T, d, dt, np.random.default_rng([35, T, d])), dt, v)
    for T, NH, D in [(1, 1, 8), (7, 3, 75), (257, 40, 64), (33, 32, 128), (5, 2, 1)]:
        print(f"[ablation] element-wise merge T={T} NH={NH} D={D} {dt}", flush=True)
        _merge(A, *workloads.merge_inputs(T, NH, D, dt, np.random.default_rng([36, T, NH, D]), empty_p=0.15), dt, v)


def test_variant_validation_on_device(A):
    buf = torch.zeros(1 << 16, dtype=torch.float16, device="cuda")
    p = buf.data_ptr()
    E = A.ASTRA_ERR_VARIANT
    assert A.astra_ablation_fused_add_rmsnorm(p, p + 8192, p + 16384, 2, 512, A.ASTRA_F16, 1e-6, 3, None) == E
    assert A.astra_ablation_fused_add_rmsnorm(p, p + 8192, p + 16384, 2, 516, A.ASTRA_F16, 1e-6, 2, None) == E   # not the fast path
    assert A.astra_ablation_silu_and_mul(p, p + 65536, 2, 512, A.ASTRA_F16, 2, None) == E
    assert A.astra_ablation_merge_attn_states_lse(p, p + 1024, p + 2048, p + 3072, p + 4096, p + 5120, 1, 2, 8, A.ASTRA_F16, 4, None) == E
    assert A.astra_ablation_silu_and_mul(p, p + 65536, 2, 512, A.ASTRA_F16, 99, None) == E
    torch.cuda.synchronize()
    assert bool((buf == 0).all())


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("T,H", [(3, 4096), (700, 2048), (1100, 5120), (300, 8192), (65, 10240), (20, 20480), (1500, 512),
                                 (40, 4104), (9, 8200),            # rows that are no whole 128-byte lines
                                 (4096, 16384)])                   # the tuned kernel holds one workgroup per compute unit here
def test_forced_pacing_gives_the_tuned_kernels_bits(A, T, H, dt):
    """The pace-forcing variants run the tuned row kernel with another order of memory requests: same arithmetic, so
    the same bits as astra_fused_add_rmsnorm, and the oracle's bars."""
    print(f"[pace] T={T} H={H} {dt}", flush=True)
    x, r, w = workloads.rmsnorm_inputs(T, H, dt, np.random.default_rng([31, T, H]), r_std=2.0)
    xd, rd, wd = to_dev(x, dt), to_dev(r, dt), to_dev(w, dt)
    A.fused_add_rmsnorm(xd, rd, wd, 1e-5)
    torch.cuda.synchronize()
    y0, r0 = to_bits(xd), to_bits(rd)
    for v in (A.ASTRA_VARIANT_PACE_NONE, A.ASTRA_VARIANT_PACE_STORE_GAP, A.ASTRA_VARIANT_PACE_X_BEFORE_R, A.ASTRA_VARIANT_PACE_WEIGHT_X_R,
              A.ASTRA_VARIANT_STORE_DEVICE_SCOPE_WHOLE_LINES, A.ASTRA_VARIANT_STORE_DEVICE_SCOPE):   # ... or another form of its stores
        _rmsnorm(A, x, r, w, 1e-5, dt, v)          # against the oracle
        xd, rd = to_dev(x, dt), to_dev(r, dt)
        st = A.astra_ablation_fused_add_rmsnorm(xd.data_ptr(), rd.data_ptr(), wd.data_ptr(), T, H, _code(A, dt), 1e-5, v,
                                                torch.cuda.current_stream().cuda_stream)
        assert st == 0
        torch.cuda.synchronize()
        assert np.array_equal(to_bits(xd), y0) and np.array_equal(to_bits(rd), r0), f"variant {v} differs from the tuned kernel"


def test_stream_probes_move_what_they_say(A):
    """astra_stream_probe: results of every mode on sizes around the workgroup and grid-padding edges; untouched
    buffers stay untouched."""
    s = torch.cuda.current_stream().cuda_stream
    for nvec in (1, 63, 64, 257, 4096 * 256 + 5, 70000):
        n = nvec * 16
        g = torch.Generator(device="cpu").manual_seed(nvec)
        a0 = torch.randint(-2**31, 2**31 - 1, (nvec * 4,), dtype=torch.int32, generator=g)
        b0 = torch.randint(-2**31, 2**31 - 1, (nvec * 4,), dtype=torch.int32, generator=g)
        pad = 64
        def dev(t):
            whole = torch.full((pad + t.numel() + pad,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
            whole[pad:pad + t.numel()] = t.cuda()
            return whole, whole[pad:pad + t.numel()]
        def edges_ok(whole):
            return bool((whole[:pad] == 0x5A5A5A5A).all() and (whole[-pad:] == 0x5A5A5A5A).all())
        for mode in range(5):
            (aw, a), (bw, b), (cw, c) = dev(a0), dev(b0), dev(torch.zeros_like(a0))
            st = A.astra_stream_probe(a.data_ptr(), b.data_ptr(), c.data_ptr(), n, mode, s)
            assert st == 0, (nvec, mode, st)
            torch.cuda.synchronize()
            ah, bh, ch = a.cpu(), b.cpu(), c.cpu()
            if mode == A.ASTRA_PROBE_COPY:
                assert torch.equal(ch, a0) and torch.equal(ah, a0) and torch.equal(bh, b0)
            elif mode == A.ASTRA_PROBE_READ2:
                assert torch.equal(ah, a0) and torch.equal(bh, b0) and not ch.any()
            elif mode == A.ASTRA_PROBE_WRITE1:
                assert torch.equal(ch.view(-1, 4), torch.arange(nvec, dtype=torch.int32).view(-1, 1).expand(-1, 4))
                assert torch.equal(ah, a0) and torch.equal(bh, b0)
            elif mode == A.ASTRA_PROBE_READ2_WRITE1:
                assert torch.equal(ch, a0 ^ b0) and torch.equal(ah, a0) and torch.equal(bh, b0)
            else:
                assert torch.equal(ah, a0 ^ b0) and torch.equal(bh, a0 + b0) and not ch.any()
            assert edges_ok(aw) and edges_ok(bw) and edges_ok(cw)
