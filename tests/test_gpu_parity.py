"""Parity of the HIP library (called through its C ABI via the ctypes binding) against the CPU oracle.

Bars (fixed by the benchmark statement): the stored residual of fused_add_rmsnorm is bit-exact; every
other 16-bit output is within rtol 1.6e-2 / atol 1e-2 (bf16) or rtol 2e-3 / atol 1e-3 (fp16); the merged
lse is within 1e-4.  Every workload of the benchmark's config list is checked element by element at
its full size, then the edge cases: empty input, the element-wise path (odd row lengths, unaligned
pointers), canary-padded buffers, aliasing, special values, determinism, error codes.
"""
import os

import numpy as np
import pytest
import torch

import oracle as O
from oracle import reference_f64
import workloads
from tests.gpu_util import (TORCH_DT, assert_lse_close, assert_storage_close, assert_storage_close_to_real,
                            canaries_intact, padded, to_bits, to_dev)
from tests.util import assert_bits_equal

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def A():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2509_07506_amd as astra

    astra.load_library()          # raises if the HIP library is missing: there is no fallback
    O.build()
    O.set_threads(min(16, len(os.sched_getaffinity(0))))
    return astra


def _say(msg):
    print(msg, flush=True)


# ---------------------------------------------------------------------------------------------------
# runners: one launch on fresh buffers, result back on the host as bit patterns

def run_rmsnorm(A, x, r, w, eps, dt):
    xd, rd, wd = to_dev(x, dt), to_dev(r, dt), to_dev(w, dt)
    A.fused_add_rmsnorm(xd, rd, wd, eps)
    torch.cuda.synchronize()
    return to_bits(xd), to_bits(rd)


def run_silu(A, a, dt):
    ad = to_dev(a, dt)
    out = torch.empty((a.shape[0], a.shape[1] // 2), dtype=TORCH_DT[dt], device="cuda")
    A.silu_and_mul(out, ad)
    torch.cuda.synchronize()
    return to_bits(out)


def run_merge(A, va, la, vb, lb, dt):
    vad, vbd = to_dev(va, dt), to_dev(vb, dt)
    lad, lbd = torch.from_numpy(la).cuda(), torch.from_numpy(lb).cuda()
    vo = torch.empty_like(vad)
    lo = torch.empty_like(lad)
    A.merge_attn_states_lse(vo, lo, vad, lad, vbd, lbd)
    torch.cuda.synchronize()
    return to_bits(vo), lo.cpu().numpy()


def check_rmsnorm(A, x, r, w, eps, dt, what, f64=True):
    y, res = run_rmsnorm(A, x, r, w, eps, dt)
    y_ref, res_ref = O.fused_add_rmsnorm(x, r, w, eps, dt)
    assert_bits_equal(res, res_ref, f"{what}: residual (bit-exact)")
    assert_storage_close(y, y_ref, dt, f"{what}: normalised output")
    if f64:
        y64, _ = reference_f64.fused_add_rmsnorm(x, r, w, eps, dt)
        assert_storage_close_to_real(y, y64, dt, f"{what}: normalised output vs float64")


def check_silu(A, a, dt, what, f64=True):
    out = run_silu(A, a, dt)
    assert_storage_close(out, O.silu_and_mul(a, dt), dt, f"{what}: out")
    if f64:
        assert_storage_close_to_real(out, reference_f64.silu_and_mul(a, dt), dt, f"{what}: out vs float64")


def check_merge(A, va, la, vb, lb, dt, what, f64=True):
    vo, lo = run_merge(A, va, la, vb, lb, dt)
    vo_ref, lo_ref = O.merge_attn_states_lse(va, la, vb, lb, dt)
    assert_storage_close(vo, vo_ref, dt, f"{what}: v_out")
    assert_lse_close(lo, lo_ref, f"{what}: lse_out")
    if f64:
        v64, l64 = reference_f64.merge_attn_states_lse(va, la, vb, lb, dt)
        assert_storage_close_to_real(vo, v64, dt, f"{what}: v_out vs float64")
        assert_lse_close(lo, l64, f"{what}: lse_out vs float64")
    return vo, lo


# ---------------------------------------------------------------------------------------------------
# every workload of the benchmark's config list, full size, element by element

BIG = 1 << 26   # elements above which the float64 cross-check is skipped (host memory / time)


@pytest.mark.parametrize("name", sorted(workloads.CASES))
def test_benchmark_workload(A, name):
    c = workloads.case(name)
    _say(f"[parity] {name} shape={c.shape} dtype={c.dtype}")
    data = c.generate()
    small = data[0].size <= BIG
    if c.kernel == "rmsnorm":
        st, info = A.astra_plan_fused_add_rmsnorm(c.shape["T"], c.shape["H"], True)
        assert st == 0 and info.as_dict()["path"] == "vector"
        check_rmsnorm(A, *data, c.eps, c.dtype, name, f64=small)
    elif c.kernel == "silu":
        st, info = A.astra_plan_silu_and_mul(c.shape["T"], c.shape["d"], True)
        assert st == 0 and info.as_dict()["path"] == "vector"
        check_silu(A, data[0], c.dtype, name, f64=small)
    else:
        st, info = A.astra_plan_merge_attn_states_lse(c.shape["T"], c.shape["NH"], c.shape["D"], True)
        assert st == 0 and info.as_dict()["path"] == "vector"
        va, la, vb, lb = data
        check_merge(A, va, la, vb, lb, c.dtype, name, f64=small)


# ---------------------------------------------------------------------------------------------------
# shapes around the kernels' tiles: every vectors-per-lane variant, ragged last wave, row loop

@pytest.mark.parametrize("T,H,dt,pace", [(4100, 16384, "bf16", 11), (4096, 14336, "f16", 11), (4097, 15360, "bf16", 11)])
def test_rmsnorm_long_rows_one_workgroup_per_compute_unit(A, T, H, dt, pace):
    """two-vector rows of 28 KiB or more on streaming grids: the row kernel reserves LDS so that a compute unit holds one workgroup at
    a time (ASTRA_PACE_ONE_RESIDENT = 8 in the plan's pace); same results as every other instantiation"""
    st, info = A.astra_plan_fused_add_rmsnorm(T, H, True)
    _say(f"[parity] rmsnorm one resident workgroup T={T} H={H} {dt} plan={info.as_dict()}")
    assert st == 0 and info.as_dict()["pace"] == pace and info.as_dict()["path"] == "vector"
    x, r, w = workloads.rmsnorm_inputs(T, H, dt, np.random.default_rng([12, T, H]), r_std=2.0)
    check_rmsnorm(A, x, r, w, 1e-5, dt, f"rmsnorm T={T} H={H} {dt}", f64=False)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("T,H", [(1, 8), (2, 64), (5, 512), (3, 520), (300, 1024), (700, 2048), (513, 4096), (600, 6144),
                                 (530, 11008), (515, 14336), (520, 16384), (4, 16384), (2, 32768), (530, 28672),
                                 (7, 12288)])
def test_rmsnorm_tile_shapes(A, T, H, dt):
    _say(f"[parity] rmsnorm tiles T={T} H={H} {dt} plan={A.astra_plan_fused_add_rmsnorm(T, H, True)[1].as_dict()}")
    x, r, w = workloads.rmsnorm_inputs(T, H, dt, np.random.default_rng([1, T, H]), r_std=2.0)
    check_rmsnorm(A, x, r, w, 1e-5, dt, f"rmsnorm T={T} H={H} {dt}")


@pytest.mark.parametrize("T,H,dt", [(1100, 2048, "bf16"), (1030, 1032, "f16"), (1024, 8192, "f16"), (1025, 11008, "bf16"),
                                    (1024, 16384, "f16"), (1030, 28672, "bf16"), (1100, 20000, "f16"), (2050, 512, "bf16"),
                                    (1040, 4096, "bf16"), (1029, 3072, "f16"), (1024, 32768, "bf16")])
def test_rmsnorm_streaming_grids(A, T, H, dt):
    """On larger grids the row kernel paces its requests (which wait goes where depends on the row length, the
    vectors per lane and the grid size); the results must not depend on it."""
    _say(f"[parity] rmsnorm streaming T={T} H={H} {dt} plan={A.astra_plan_fused_add_rmsnorm(T, H, True)[1].as_dict()}")
    x, r, w = workloads.rmsnorm_inputs(T, H, dt, np.random.default_rng([11, T, H]), r_std=2.0)
    check_rmsnorm(A, x, r, w, 1e-5, dt, f"rmsnorm T={T} H={H} {dt}")


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("T,H,rows", [(1, 8, 32), (7, 16, 32), (33, 24, 32), (1000, 64, 32), (5000, 72, 16), (257, 128, 16),
                                      (4099, 136, 8), (65, 200, 8), (3, 256, 8), (60000, 128, 16),
                                      # streaming grids of rows that fill their lane groups: single-wave workgroups
                                      (140001, 64, 8), (70003, 128, 4), (33001, 256, 2)])
def test_rmsnorm_short_rows_share_a_workgroup(A, T, H, rows, dt):
    """Rows of at most 32 vectors: 8, 16 or 32 lanes per row, several rows per workgroup, the sum inside the wave;
    ragged last workgroups and rows that leave lanes of their group idle included."""
    plan = A.astra_plan_fused_add_rmsnorm(T, H, True)[1].as_dict()
    _say(f"[parity] rmsnorm short rows T={T} H={H} {dt} plan={plan}")
    lanes_per_row = 8 if H <= 64 else 16 if H <= 128 else 32
    assert plan.get("rows_per_block") == rows and plan["block"] == rows * lanes_per_row == (64 if T > 30000 and T != 60000 else 256)
    x, r, w = workloads.rmsnorm_inputs(T, H, dt, np.random.default_rng([13, T, H]), r_std=2.0)
    check_rmsnorm(A, x, r, w, 1e-5, dt, f"rmsnorm T={T} H={H} {dt}")


@pytest.mark.parametrize("T,H,dt,vpt,pace", [(1280, 4096, "bf16", 2, 2), (1024, 5120, "f16", 2, 2), (600, 7168, "bf16", 2, 2),
                                             (1537, 3072, "f16", 2, 2), (2560, 2048, "bf16", 2, 2), (5000, 1024, "f16", 2, 2),
                                             (700, 5000, "bf16", 2, 2), (760, 6136, "f16", 2, 2),
                                             (768, 8192, "bf16", 1, 2), (1024, 4096, "f16", 1, 2), (2047, 2048, "bf16", 1, 2),
                                             (500, 7168, "f16", 1, 2), (1100, 7680, "bf16", 1, 2), (2000, 5120, "f16", 1, 0),
                                             (512, 14336, "f16", 4, 2), (300, 12288, "bf16", 4, 2), (500, 11000, "bf16", 4, 2)])
def test_rmsnorm_grids_of_few_rounds(A, T, H, dt, vpt, pace):
    """Grids of one to three rounds of resident workgroups: x is requested before r, and rows that just no longer fit
    at once go to half-sized workgroups with two vectors per lane (also where the last vector of a lane falls off
    the end of the row), two-vector rows that fill the machine exactly to four; the results must not depend on any
    of it."""
    plan = A.astra_plan_fused_add_rmsnorm(T, H, True)[1].as_dict()
    _say(f"[parity] rmsnorm few rounds T={T} H={H} {dt} plan={plan}")
    assert (plan["vectors_per_lane"], plan["pace"]) == (vpt, pace)
    x, r, w = workloads.rmsnorm_inputs(T, H, dt, np.random.default_rng([12, T, H]), r_std=2.0)
    check_rmsnorm(A, x, r, w, 1e-5, dt, f"rmsnorm T={T} H={H} {dt}")


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("T,d", [(1, 256), (3, 264), (2, 512), (7, 1000), (33, 2048), (5, 4096), (19, 5120), (2, 12288),
                                 (1, 14336), (129, 3584),
                                 (300, 8), (17, 64), (1000, 176), (5, 248), (4099, 24),    # rows under 32 vectors
                                 (50000, 176)])            # ... on a streaming grid (single-wave workgroups, per-lane division)
def test_silu_tile_shapes(A, T, d, dt):
    _say(f"[parity] silu tiles T={T} d={d} {dt} plan={A.astra_plan_silu_and_mul(T, d, True)[1].as_dict()}")
    a = workloads.silu_inputs(T, d, dt, np.random.default_rng([2, T, d]))
    check_silu(A, a, dt, f"silu T={T} d={d} {dt}")


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("T,NH,D", [(1, 1, 8), (3, 5, 16), (7, 3, 72), (9, 8, 80), (5, 32, 96), (512, 32, 256), (512, 40, 128),
                                    (11, 64, 128), (2, 7, 192), (1, 1, 1024), (3, 2, 576),
                                    (4000, 32, 72)])       # streaming grid, head_dim no power of two (single-wave workgroups)
def test_merge_tile_shapes(A, T, NH, D, dt):
    _say(f"[parity] merge tiles T={T} NH={NH} D={D} {dt} plan={A.astra_plan_merge_attn_states_lse(T, NH, D, True)[1].as_dict()}")
    va, la, vb, lb = workloads.merge_inputs(T, NH, D, dt, np.random.default_rng([3, T, NH, D]), empty_p=0.1)
    check_merge(A, va, la, vb, lb, dt, f"merge T={T} NH={NH} D={D} {dt}")


# ---------------------------------------------------------------------------------------------------
# ragged and element-wise paths: odd row lengths and pointers that are only 2-byte aligned; canaries around buffers

@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("T,H,off", [(3, 4100, 0), (2, 4097, 0), (5, 1, 0), (4, 7, 0), (3, 4096, 1), (2, 8192, 3), (3, 333, 5),
                                     (2, 8, 1), (5, 9, 0), (3, 15, 7), (257, 5124, 0), (300, 11009, 0), (33, 32767, 1),
                                     (1030, 4098, 3), (600, 16383, 5), (40, 32761, 0), (7, 32775, 0), (300, 8199, 1),
                                     (2, 70000, 0), (1, 65536, 0),
                                     # offsets beyond one vector: the row starts in the middle of a 128-byte line
                                     (70, 4097, 9), (3, 4096, 37), (130, 1001, 63), (40, 32705, 0), (5, 32705, 63), (3, 8, 57),
                                     # whole vectors but no whole 128-byte lines, aligned tensors: the same kernel
                                     (5, 4104, 0), (300, 8200, 0), (130, 11016, 0), (70, 2056, 0), (8200, 2056, 0), (8192, 4104, 0)])
def test_rmsnorm_ragged_and_generic_paths_and_canaries(A, T, H, off, dt):
    _say(f"[parity] rmsnorm ragged/generic T={T} H={H} offset={off} {dt}")
    x, r, w = workloads.rmsnorm_inputs(T, H, dt, np.random.default_rng([4, T, H, off]), r_std=2.0)
    xd, xw = padded(x, dt, offset_elems=off)
    rd, rw = padded(r, dt, offset_elems=off)
    wd, ww = padded(w, dt, offset_elems=off)
    # x and r carry the same offset, so they are in step with each other: the phased kernel (aligned chunks)
    st, info = A.astra_plan_fused_add_rmsnorm(T, H, 1 if off == 0 else 2)
    if H % 8 or off:
        assert info.as_dict()["path"] == ("generic" if H < 8 or H // 8 > 4096 else "phased" if (H + 63 + 7) // 8 <= 4096 else "ragged")
    else:  # aligned tensors, rows of whole vectors
        assert info.as_dict()["path"] == ("generic" if H // 8 > 4096 else "phased" if T >= 8192 and H * 2 % 128 else "vector")
    A.fused_add_rmsnorm(xd, rd, wd, 1e-5)
    torch.cuda.synchronize()
    y_ref, res_ref = O.fused_add_rmsnorm(x, r, w, 1e-5, dt)
    assert_bits_equal(to_bits(rd), res_ref, "residual (bit-exact)")
    assert_storage_close(to_bits(xd), y_ref, dt, "normalised output")
    assert canaries_intact(xw, x.size, offset_elems=off) and canaries_intact(rw, r.size, offset_elems=off)
    assert canaries_intact(ww, w.size, offset_elems=off) and np.array_equal(to_bits(wd), w)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("T,H,offs", [(3, 4100, (0, 1, 0)), (5, 4096, (1, 0, 0)), (4, 4097, (3, 6, 1)), (300, 5124, (2, 5, 7)),
                                      (7, 9, (0, 4, 0)), (257, 11009, (1, 2, 3)), (33, 32767, (7, 0, 2)), (600, 16383, (4, 0, 0)),
                                      (1030, 2056, (0, 0, 3)), (3, 8, (1, 2, 0))])
def test_rmsnorm_tensors_at_unrelated_offsets(A, T, H, offs, dt):
    """x, r and the weight each at an offset of its own into the 16-byte grid: the ragged kernel (16-byte accesses at
    element alignment) when x and r are out of step, the phased one with an offset weight when only the weight is."""
    _say(f"[parity] rmsnorm mixed offsets T={T} H={H} offsets={offs} {dt}")
    x, r, w = workloads.rmsnorm_inputs(T, H, dt, np.random.default_rng([14, T, H]), r_std=2.0)
    xd, xw = padded(x, dt, offset_elems=offs[0])
    rd, rw = padded(r, dt, offset_elems=offs[1])
    wd, ww = padded(w, dt, offset_elems=offs[2])
    A.fused_add_rmsnorm(xd, rd, wd, 1e-5)
    torch.cuda.synchronize()
    y_ref, res_ref = O.fused_add_rmsnorm(x, r, w, 1e-5, dt)
    assert_bits_equal(to_bits(rd), res_ref, "residual (bit-exact)")
    assert_storage_close(to_bits(xd), y_ref, dt, "normalised output")
    assert canaries_intact(xw, x.size, offset_elems=offs[0]) and canaries_intact(rw, r.size, offset_elems=offs[1])
    assert canaries_intact(ww, w.size, offset_elems=offs[2]) and np.array_equal(to_bits(wd), w)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("T,H", [(3, 4096), (257, 5120), (2, 8192), (300, 7168)])
def test_rmsnorm_vector_path_canaries(A, T, H, dt):
    x, r, w = workloads.rmsnorm_inputs(T, H, dt, np.random.default_rng([5, T, H]))
    xd, xw = padded(x, dt)
    rd, rw = padded(r, dt)
    wd, ww = padded(w, dt)
    assert all(t.data_ptr() % 16 == 0 for t in (xd, rd, wd))
    A.fused_add_rmsnorm(xd, rd, wd, 1e-6)
    torch.cuda.synchronize()
    y_ref, res_ref = O.fused_add_rmsnorm(x, r, w, 1e-6, dt)
    assert_bits_equal(to_bits(rd), res_ref, "residual (bit-exact)")
    assert_storage_close(to_bits(xd), y_ref, dt, "normalised output")
    assert canaries_intact(xw, x.size) and canaries_intact(rw, r.size) and canaries_intact(ww, w.size)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("T,d,off", [(3, 100, 0), (2, 1412, 0), (5, 1, 0), (4, 2049, 0), (3, 1408, 1), (2, 248, 0), (3, 11008, 2),
                                     (4, 1408, 0), (257, 11008, 0),
                                     (300, 11009, 0), (1000, 7, 3), (257, 1410, 5), (64, 8, 1), (129, 13825, 0), (50, 11012, 7),
                                     # offset pointers: aligned chunks of the output, one per row across the row end
                                     # (rows of eight vectors or more; shorter rows at element alignment)
                                     (1, 8, 7), (1, 16, 3), (2, 8, 4), (513, 1408, 4), (1030, 64, 5), (257, 11008, 6),
                                     (40, 14336, 9), (3, 24, 15)])
def test_silu_paths_and_canaries(A, T, d, off, dt):
    _say(f"[parity] silu T={T} d={d} offset={off} {dt}")
    a = workloads.silu_inputs(T, d, dt, np.random.default_rng([6, T, d, off]))
    ad, aw = padded(a, dt, offset_elems=off)
    out_init = np.full((T, d), 0x1234, np.uint16)
    od, ow = padded(out_init, dt, offset_elems=off)
    st, info = A.astra_plan_silu_and_mul(T, d, 1 if off % 8 == 0 else 2)
    assert info.as_dict()["path"] == ("vector" if d % 8 == 0 and off % 8 == 0 else "phased" if d >= 64 else "ragged")
    A.silu_and_mul(od, ad)
    torch.cuda.synchronize()
    assert_storage_close(to_bits(od), O.silu_and_mul(a, dt), dt, "out")
    assert canaries_intact(ow, T * d, offset_elems=off) and canaries_intact(aw, a.size, offset_elems=off)
    assert np.array_equal(to_bits(ad), a)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("T,d,off_in,off_out", [(5, 1408, 1, 2), (300, 11008, 0, 3), (64, 8, 5, 0), (33, 1416, 7, 7)])
def test_silu_input_and_output_at_unrelated_offsets(A, T, d, off_in, off_out, dt):
    """input and output out of step with each other: the aligned chunks of the output, loads at element alignment (the
    last case is in step)"""
    _say(f"[parity] silu T={T} d={d} offsets in={off_in} out={off_out} {dt}")
    a = workloads.silu_inputs(T, d, dt, np.random.default_rng([66, T, d, off_in, off_out]))
    ad, aw = padded(a, dt, offset_elems=off_in)
    od, ow = padded(np.full((T, d), 0x1234, np.uint16), dt, offset_elems=off_out)
    A.silu_and_mul(od, ad)
    torch.cuda.synchronize()
    assert_storage_close(to_bits(od), O.silu_and_mul(a, dt), dt, "out")
    assert canaries_intact(ow, T * d, offset_elems=off_out) and canaries_intact(aw, a.size, offset_elems=off_in)
    assert np.array_equal(to_bits(ad), a)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("T,NH,D,off", [(3, 5, 4, 0), (2, 3, 100, 0), (5, 2, 1, 0), (3, 4, 128, 1), (2, 40, 64, 3), (4, 40, 256, 0),
                                        (257, 40, 64, 0), (3, 6, 72, 0),
                                        (257, 40, 129, 0), (100, 7, 132, 5), (300, 32, 7, 0), (65, 40, 128, 1), (33, 5, 9, 3)])
def test_merge_paths_and_canaries(A, T, NH, D, off, dt):
    _say(f"[parity] merge T={T} NH={NH} D={D} offset={off} {dt}")
    va, la, vb, lb = workloads.merge_inputs(T, NH, D, dt, np.random.default_rng([7, T, NH, D, off]), empty_p=0.15)
    vad, vaw = padded(va, dt, offset_elems=off)
    vbd, vbw = padded(vb, dt, offset_elems=off)
    vod, vow = padded(np.full(va.shape, 0x1234, np.uint16), dt, offset_elems=off)
    pad = 16
    lo_whole = torch.full((pad + T * NH + pad,), 1234.5, dtype=torch.float32, device="cuda")
    lod = lo_whole[pad:pad + T * NH].view(T, NH)
    lad, lbd = torch.from_numpy(la).cuda(), torch.from_numpy(lb).cuda()
    A.merge_attn_states_lse(vod, lod, vad, lad, vbd, lbd)
    torch.cuda.synchronize()
    vo_ref, lo_ref = O.merge_attn_states_lse(va, la, vb, lb, dt)
    assert_storage_close(to_bits(vod), vo_ref, dt, "v_out")
    assert_lse_close(lod.cpu().numpy(), lo_ref, "lse_out")
    assert canaries_intact(vow, va.size, offset_elems=off)
    edge = lo_whole.cpu().numpy()
    assert np.all(edge[:pad] == 1234.5) and np.all(edge[pad + T * NH:] == 1234.5)
    assert np.array_equal(to_bits(vad), va) and np.array_equal(to_bits(vbd), vb)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("T,NH,D,offs", [(3, 5, 100, (0, 1, 0)), (65, 40, 128, (1, 0, 0)), (257, 40, 129, (2, 5, 7)), (33, 5, 9, (0, 0, 3)),
                                         (100, 7, 132, (4, 4, 0)), (9, 3, 8, (1, 1, 2))])
def test_merge_tensors_at_unrelated_offsets(A, T, NH, D, offs, dt):
    """v_a, v_b and v_out each at an offset of its own into the 16-byte grid: the aligned chunks of the output, loads at
    element alignment (head_dim >= 8; below that the ragged kernel)"""
    _say(f"[parity] merge mixed offsets T={T} NH={NH} D={D} offsets={offs} {dt}")
    va, la, vb, lb = workloads.merge_inputs(T, NH, D, dt, np.random.default_rng([15, T, NH, D]), empty_p=0.15)
    vad, vaw = padded(va, dt, offset_elems=offs[0])
    vbd, vbw = padded(vb, dt, offset_elems=offs[1])
    vod, vow = padded(np.full(va.shape, 0x1234, np.uint16), dt, offset_elems=offs[2])
    lad, lbd = torch.from_numpy(la).cuda(), torch.from_numpy(lb).cuda()
    lod = torch.empty_like(lad)
    A.merge_attn_states_lse(vod, lod, vad, lad, vbd, lbd)
    torch.cuda.synchronize()
    vo_ref, lo_ref = O.merge_attn_states_lse(va, la, vb, lb, dt)
    assert_storage_close(to_bits(vod), vo_ref, dt, "v_out")
    assert_lse_close(lod.cpu().numpy(), lo_ref, "lse_out")
    assert canaries_intact(vow, va.size, offset_elems=offs[2])
    assert np.array_equal(to_bits(vad), va) and np.array_equal(to_bits(vbd), vb)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("T,NH,D,off", [(1, 1, 8, 1), (1, 1, 9, 0), (2, 3, 15, 7), (1000, 8, 129, 0), (4099, 40, 65, 3), (300, 5, 1000, 5),
                                        (64, 4, 257, 0), (7, 1, 2049, 2)])
def test_merge_phased_path_pair_boundaries(A, T, NH, D, off, dt):
    """the phased kernel's chunks straddle pair boundaries at every position; S_out must come from the right lane, and
    empty pairs next to live ones must not bleed into each other"""
    _say(f"[parity] merge phased T={T} NH={NH} D={D} offset={off} {dt}")
    st, info = A.astra_plan_merge_attn_states_lse(T, NH, D, 1 if off == 0 else 2)
    assert info.as_dict()["path"] == ("phased" if (D % 8 or off) else "vector")
    va, la, vb, lb = workloads.merge_inputs(T, NH, D, dt, np.random.default_rng([16, T, NH, D]), empty_p=0.3)
    vad, vaw = padded(va, dt, offset_elems=off)
    vbd, vbw = padded(vb, dt, offset_elems=off)
    vod, vow = padded(np.full(va.shape, 0x1234, np.uint16), dt, offset_elems=off)
    pad = 16
    lo_whole = torch.full((pad + T * NH + pad,), 1234.5, dtype=torch.float32, device="cuda")
    lod = lo_whole[pad:pad + T * NH].view(T, NH)
    lad, lbd = torch.from_numpy(la).cuda(), torch.from_numpy(lb).cuda()
    A.merge_attn_states_lse(vod, lod, vad, lad, vbd, lbd)
    torch.cuda.synchronize()
    vo_ref, lo_ref = O.merge_attn_states_lse(va, la, vb, lb, dt)
    assert_storage_close(to_bits(vod), vo_ref, dt, "v_out")
    assert_lse_close(lod.cpu().numpy(), lo_ref, "lse_out")
    assert canaries_intact(vow, va.size, offset_elems=off)
    edge = lo_whole.cpu().numpy()
    assert np.all(edge[:pad] == 1234.5) and np.all(edge[pad + T * NH:] == 1234.5)
    # in place on v_a
    A.merge_attn_states_lse(vad, lod, vad, lad, vbd, lbd)
    torch.cuda.synchronize()
    assert_storage_close(to_bits(vad), vo_ref, dt, "v_out in place on v_a")
    assert canaries_intact(vaw, va.size, offset_elems=off)


# ---------------------------------------------------------------------------------------------------
# degenerate and special-value cases

def test_empty_inputs_are_no_ops(A):
    for dt in ("bf16", "f16"):
        x = torch.empty((0, 4096), dtype=TORCH_DT[dt], device="cuda")
        w = torch.ones(4096, dtype=TORCH_DT[dt], device="cuda")
        A.fused_add_rmsnorm(x, x.clone(), w, 1e-6)
        A.silu_and_mul(torch.empty((0, 128), dtype=TORCH_DT[dt], device="cuda"),
                       torch.empty((0, 256), dtype=TORCH_DT[dt], device="cuda"))
        v = torch.empty((0, 4, 64), dtype=TORCH_DT[dt], device="cuda")
        s = torch.empty((0, 4), dtype=torch.float32, device="cuda")
        A.merge_attn_states_lse(v.clone(), s.clone(), v, s, v.clone(), s.clone())
    torch.cuda.synchronize()
    # T == 0 with valid non-null pointers through the raw entry points
    buf = torch.zeros(64, dtype=torch.float16, device="cuda")
    p = buf.data_ptr()
    assert A.astra_fused_add_rmsnorm(p, p + 32, p + 64, 0, 8, A.ASTRA_F16, 1e-6, None) == 0
    assert A.astra_silu_and_mul(p, p + 64, 0, 8, A.ASTRA_F16, None) == 0


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_rmsnorm_special_rows(A, dt):
    """all-zero row (y = 0, no NaN), constant row (closed form), tiny values (fp16 subnormal sums)."""
    T, H = 6, 4096
    x, r, w = workloads.rmsnorm_inputs(T, H, dt, np.random.default_rng(8))
    x[0] = 0
    r[0] = 0
    x[1] = workloads.to_bits(np.full(H, 0.5, np.float32), dt)
    r[1] = workloads.to_bits(np.full(H, 1.0, np.float32), dt)
    x[2] = workloads.to_bits(np.random.default_rng(9).standard_normal(H).astype(np.float32) * 2.0 ** -15, dt)
    r[2] = workloads.to_bits(np.random.default_rng(10).standard_normal(H).astype(np.float32) * 2.0 ** -16, dt)
    x[3] = workloads.to_bits(np.full(H, 3.0e4 if dt == "f16" else 1e30, np.float32), dt)     # large but finite sums
    r[3] = workloads.to_bits(np.full(H, 2.0e4 if dt == "f16" else 1e30, np.float32), dt)
    y, res = run_rmsnorm(A, x, r, w, 1e-6, dt)
    y_ref, res_ref = O.fused_add_rmsnorm(x, r, w, 1e-6, dt)
    assert_bits_equal(res, res_ref, "residual (bit-exact, incl. subnormal sums)")
    if dt == "bf16":
        # 1e30^2 overflows binary32 in both implementations: inf mean square -> scale 0 -> y = 0 (or NaN
        # from inf * 0); compare only the finite rows strictly and row 3 for agreement in kind
        assert_storage_close(np.delete(y, 3, axis=0), np.delete(y_ref, 3, axis=0), dt, "y")
    else:
        assert_storage_close(y, y_ref, dt, "y")
    assert np.all((y[0] & 0x7FFF) == 0)
    wf = reference_f64.widen(w, dt)
    assert_storage_close_to_real(y[1], 1.5 / np.sqrt(1.5 ** 2 + 1e-6) * wf, dt, "constant row closed form")
    if dt == "f16":
        sub = (res[2] & 0x7C00) == 0
        assert sub.sum() > 100, "expected fp16-subnormal residuals in the tiny row"


@pytest.mark.parametrize("dt", ["bf16", "f32"])
@pytest.mark.parametrize("H", [4096, 64, 4100, 40000])
def test_rmsnorm_rows_whose_mean_square_is_subnormal(A, dt, H):
    """|x + r| around 1e-20 with eps = 0: the mean square (about 1e-40) is a binary32 subnormal, which the hardware
    reciprocal square root alone would read as zero.  The scale must stay finite and y close to the oracle's, on the
    row, short-row, ragged and element-wise kernels.  (fp16 cannot hold such values.)"""
    _say(f"[tiny rows] {dt} H={H}")
    T = 5
    rng = np.random.default_rng([13, H])
    x = workloads.to_bits((rng.standard_normal((T, H)) * 1e-20).astype(np.float32), dt)
    r = workloads.to_bits((rng.standard_normal((T, H)) * 1e-20).astype(np.float32), dt)
    w = workloads.to_bits((1.0 + 0.3 * rng.standard_normal(H)).astype(np.float32), dt)
    x[1], r[1] = x[1] * 0, r[1] * 0
    x[1, 0] = workloads.to_bits(np.array([3e-22], np.float32), dt)[0]      # mean square far below the subnormal range
    for eps in (0.0, 1e-42):
        y, res = run_rmsnorm(A, x, r, w, eps, dt)
        if dt == "f32":
            res_ref, y_ref = O.fused_add_rmsnorm_f32(x, r, w, eps)
        else:
            y_ref, res_ref = O.fused_add_rmsnorm(x, r, w, eps, dt)
        assert_bits_equal(res, res_ref, "residual")
        yw, yr = reference_f64.widen(y, dt), reference_f64.widen(y_ref, dt)
        rows = [0, 2, 3, 4]                                                # row 1: a total that underflows to 0 in
        assert np.all(np.isfinite(yw[rows])), "scale must stay finite"     # binary32 gives inf * s in both forms
        # the squares are subnormal (about 16 significant bits), so compare with the 16-bit bar for both storage types
        np.testing.assert_allclose(yw[rows], yr[rows], rtol=1.6e-2, atol=1e-2)
        y64, _ = reference_f64.fused_add_rmsnorm(x[rows], r[rows], w, eps, dt)
        np.testing.assert_allclose(yw[rows], y64, rtol=1.6e-2, atol=1e-2)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_silu_special_values(A, dt):
    xs = np.array([0.0, -0.0, 1.0, -1.0, -1.2784645, 20.0, 88.0, 100.0, -20.0, -87.0, -88.0, -89.0, -100.0, -200.0, 3e4, -3e4,
                   1e-6, -1e-6, 6e-8, 2.0 ** -15, 0.5, 10.0], np.float32)
    gs = np.array([1.0, -2.0, 0.0, 0.5, 3.0, 2.0 ** -10], np.float32)
    X, G = np.meshgrid(xs, gs, indexing="ij")
    d = 256
    row_x = np.zeros(d, np.float32)
    row_g = np.ones(d, np.float32)
    row_x[: X.size] = X.ravel()
    row_g[: G.size] = G.ravel()
    a = workloads.to_bits(np.concatenate([row_x, row_g]).reshape(1, 2 * d), dt)
    out = run_silu(A, a, dt)
    ref = O.silu_and_mul(a, dt)
    assert_storage_close(out, ref, dt, "special values")
    assert_storage_close_to_real(out, reference_f64.silu_and_mul(a, dt), dt, "special values vs float64")
    xb = reference_f64.widen(a[0, :d], dt)
    assert np.all((out[0][xb == 0] & 0x7FFF) == 0), "silu(0) * g must be zero"
    assert not np.isnan(reference_f64.widen(out, dt)).any()


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_merge_empty_partitions_and_symmetry(A, dt):
    T, NH, D = 64, 8, 128
    va, la, vb, lb = workloads.merge_inputs(T, NH, D, dt, np.random.default_rng(11), empty_p=0.0)
    la[:, 0] = -np.inf                      # side a empty
    lb[:, 1] = -np.inf                      # side b empty
    la[:, 2] = -np.inf
    lb[:, 2] = -np.inf                      # both empty
    lb[:, 3] = la[:, 3]                     # equal scores
    la[:, 4] = 14.0
    lb[:, 4] = -95.0                        # dominance: e^(Sb-Sa) underflows
    vo, lo = check_merge(A, va, la, vb, lb, dt, "merge special")
    assert np.array_equal(vo[:, 0], vb[:, 0]) and np.array_equal(lo[:, 0], lb[:, 0]), "empty a must return b bit-exactly"
    assert np.array_equal(vo[:, 1], va[:, 1]) and np.array_equal(lo[:, 1], la[:, 1]), "empty b must return a bit-exactly"
    assert np.all((vo[:, 2] & 0x7FFF) == 0) and np.all(np.isneginf(lo[:, 2]))
    assert np.allclose(lo[:, 3], la[:, 3] + np.log(2.0), rtol=0, atol=1e-5)
    assert np.array_equal(vo[:, 4], va[:, 4]) and np.all(lo[:, 4] == 14.0)
    # symmetry within tolerance, lse symmetric exactly (max and sum commute)
    vo2, lo2 = run_merge(A, vb, lb, va, la, dt)
    assert_storage_close(vo2, vo, dt, "symmetry v_out")
    assert np.array_equal(lo2.view(np.uint32), lo.view(np.uint32))


@pytest.mark.parametrize("dt", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("D,offset,variant", [(128, 0, 0), (64, 0, 0), (100, 0, 0), (129, 0, 0), (128, 1, 0), (128, 0, 5),
                                              (128, 0, 1), (128, 0, 3)])
def test_merge_never_looks_at_an_empty_partition(A, dt, D, offset, variant):
    """NaN / inf left in the value buffer of a partition whose score is -inf must not reach the output: the other
    side comes back bit for bit (a negative zero included) on every path -- vector, ragged (odd head_dim, pointer
    offset by one element), element-wise and the ablation variants."""
    if dt == "f32" and variant in (1, 3):
        pytest.skip("ablation variants exist for the 16-bit types only")
    if dt == "f32" and D == 129:
        D = 130
    _say(f"[merge empty] {dt} D={D} offset={offset} variant={variant}")
    T, NH = 37, 6
    va, la, vb, lb = workloads.merge_inputs(T, NH, D, dt, np.random.default_rng([12, D]), empty_p=0.0)
    nan_bits = workloads.to_bits(np.array([np.nan], np.float32), dt)[0]
    inf_bits = workloads.to_bits(np.array([np.inf], np.float32), dt)[0]
    va[0, 0, :2] = workloads.to_bits(np.array([-0.0, 0.0], np.float32), dt)
    lb[:, 0] = -np.inf
    vb[:, 0] = nan_bits            # side b empty and full of NaN
    la[:, 1] = -np.inf
    va[:, 1] = inf_bits            # side a empty and full of +inf
    la[:, 2] = -np.inf
    lb[:, 2] = -np.inf
    va[:, 2] = nan_bits
    vb[:, 2] = inf_bits            # both empty, both garbage
    la[:, 3] = 12.0
    lb[:, 3] = -150.0
    vb[:, 3] = nan_bits            # weight underflows to exactly zero
    vad, _ = padded(va, dt, offset_elems=offset)
    vbd, _ = padded(vb, dt, offset_elems=offset)
    vod, whole = padded(np.zeros_like(va), dt, offset_elems=offset)
    lad, lbd = torch.from_numpy(la).cuda(), torch.from_numpy(lb).cuda()
    lod = torch.empty_like(lad)
    code = {"bf16": A.ASTRA_BF16, "f16": A.ASTRA_F16, "f32": A.ASTRA_F32}[dt]
    args = (vod.data_ptr(), lod.data_ptr(), vad.data_ptr(), lad.data_ptr(), vbd.data_ptr(), lbd.data_ptr(), T, NH, D, code)
    st = A.astra_merge_attn_states_lse(*args, None) if variant == 0 else A.astra_ablation_merge_attn_states_lse(*args, variant, None)
    if variant in (1, 3) and (D % 8 or offset):
        assert st == A.ASTRA_ERR_VARIANT
        return
    assert st == 0
    torch.cuda.synchronize()
    vo, lo = to_bits(vod), lod.cpu().numpy()
    as_bits = (lambda a: a.view(np.uint32)) if dt == "f32" else (lambda a: a)
    assert np.array_equal(as_bits(vo[:, 0]), as_bits(va[:, 0])) and np.array_equal(lo[:, 0], la[:, 0])
    assert np.array_equal(as_bits(vo[:, 1]), as_bits(vb[:, 1])) and np.array_equal(lo[:, 1], lb[:, 1])
    assert np.all(reference_f64.widen(vo[:, 2], dt) == 0) and np.all(np.isneginf(lo[:, 2]))
    assert np.array_equal(as_bits(vo[:, 3]), as_bits(va[:, 3])) and np.all(lo[:, 3] == 12.0)
    vo_ref, lo_ref = (O.merge_attn_states_lse_f32 if dt == "f32" else lambda *a: O.merge_attn_states_lse(*a, dt))(va, la, vb, lb)
    assert_storage_close(vo, vo_ref, dt, "merge with garbage in empty partitions")
    assert_lse_close(lo, lo_ref, "lse")
    assert canaries_intact(whole, va.size, offset_elems=offset)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_merge_output_may_alias_an_input(A, dt):
    T, NH, D = 33, 8, 128
    va, la, vb, lb = workloads.merge_inputs(T, NH, D, dt, np.random.default_rng(12), empty_p=0.05)
    vo_ref, lo_ref = O.merge_attn_states_lse(va, la, vb, lb, dt)
    for alias in ("a", "b"):
        vad, vbd = to_dev(va, dt), to_dev(vb, dt)
        lad, lbd = torch.from_numpy(la).cuda(), torch.from_numpy(lb).cuda()
        lo = torch.empty_like(lad)
        vo = vad if alias == "a" else vbd
        A.merge_attn_states_lse(vo, lo, vad, lad, vbd, lbd)
        torch.cuda.synchronize()
        assert_storage_close(to_bits(vo), vo_ref, dt, f"v_out aliasing v_{alias}")
        assert_lse_close(lo.cpu().numpy(), lo_ref, "lse_out")


def test_results_are_deterministic(A):
    """every output element has one writer and the reduction order is fixed: two runs give the same bits"""
    dt = "bf16"
    x, r, w = workloads.rmsnorm_inputs(700, 8192, dt, np.random.default_rng(13), r_std=2.0)
    y1, r1 = run_rmsnorm(A, x, r, w, 1e-5, dt)
    y2, r2 = run_rmsnorm(A, x, r, w, 1e-5, dt)
    assert np.array_equal(y1, y2) and np.array_equal(r1, r2)
    a = workloads.silu_inputs(300, 11008, dt, np.random.default_rng(14))
    assert np.array_equal(run_silu(A, a, dt), run_silu(A, a, dt))
    m = workloads.merge_inputs(300, 40, 128, dt, np.random.default_rng(15))
    o1, o2 = run_merge(A, *m, dt), run_merge(A, *m, dt)
    assert np.array_equal(o1[0], o2[0]) and np.array_equal(o1[1].view(np.uint32), o2[1].view(np.uint32))


def test_runs_on_a_non_default_stream(A):
    dt = "f16"
    x, r, w = workloads.rmsnorm_inputs(64, 5120, dt, np.random.default_rng(16))
    xd, rd, wd = to_dev(x, dt), to_dev(r, dt), to_dev(w, dt)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        A.fused_add_rmsnorm(xd, rd, wd, 1e-6)          # picks up torch's current stream
    s.synchronize()
    y_ref, res_ref = O.fused_add_rmsnorm(x, r, w, 1e-6, dt)
    assert_bits_equal(to_bits(rd), res_ref, "residual")
    assert_storage_close(to_bits(xd), y_ref, dt, "y")
    xd2, rd2 = to_dev(x, dt), to_dev(r, dt)
    torch.cuda.synchronize()
    st = A.astra_fused_add_rmsnorm(xd2.data_ptr(), rd2.data_ptr(), wd.data_ptr(), 64, 5120, A.ASTRA_F16, 1e-6, s.cuda_stream)
    assert st == 0
    s.synchronize()
    assert_bits_equal(to_bits(rd2), res_ref, "residual (explicit stream)")


def test_error_codes_with_device_pointers(A):
    """validation happens before any launch; the buffers must come back untouched"""
    buf = torch.full((4096,), 7.0, dtype=torch.float16, device="cuda")
    p = buf.data_ptr()
    E = {"null": 1, "shape": 2, "dtype": 3, "eps": 4, "align": 5, "alias": 6}
    assert A.astra_fused_add_rmsnorm(p, p + 2048, p + 4096, 2, 512, 9, 1e-6, None) == E["dtype"]
    assert A.astra_fused_add_rmsnorm(p, p + 2048, p + 4096, 2, 512, A.ASTRA_F16, float("nan"), None) == E["eps"]
    assert A.astra_fused_add_rmsnorm(p, p + 1024, p + 4096, 2, 512, A.ASTRA_F16, 1e-6, None) == E["alias"]
    assert A.astra_fused_add_rmsnorm(p, p + 2049, p + 4096, 2, 512, A.ASTRA_F16, 1e-6, None) == E["align"]
    assert A.astra_silu_and_mul(p, p + 512, 2, 512, A.ASTRA_F16, None) == E["alias"]
    assert A.astra_silu_and_mul(p, p + 4096, -1, 512, A.ASTRA_F16, None) == E["shape"]
    f = torch.zeros(64, dtype=torch.float32, device="cuda")
    q = f.data_ptr()
    assert A.astra_merge_attn_states_lse(p, q, p + 8, q + 64, p + 4096, q + 128, 1, 2, 4, A.ASTRA_F16, None) == E["alias"]
    assert A.astra_merge_attn_states_lse(p, q, p + 2048, q, p + 4096, q + 128, 1, 2, 4, A.ASTRA_F16, None) == E["alias"]
    assert A.astra_merge_attn_states_lse(p, q + 2, p + 2048, q + 64, p + 4096, q + 128, 1, 2, 4, A.ASTRA_F16, None) == E["align"]
    torch.cuda.synchronize()
    assert bool((buf == 7.0).all()) and bool((f == 0).all())


def test_stream_copy(A):
    src = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    A.stream_copy(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    n = (1 << 20) * 4 - 16 * 3        # ragged tail: not a multiple of the block span
    dst.zero_()
    assert A.astra_stream_copy(dst.data_ptr(), src.data_ptr(), n, None) == 0
    torch.cuda.synchronize()
    assert torch.equal(dst[: n // 4], src[: n // 4]) and bool((dst[n // 4:] == 0).all())


# ---------------------------------------------------------------------------------------------------
# maximum sizes: more than 2^31 elements per tensor (byte offsets beyond 32 bits), and more rows than the
# row kernel's grid limit (row loop).  A small seeded block is tiled on the device; the first tile is
# checked against the oracle and every other tile must be bit-identical to the first.

def _tile_rows(block_dev, reps):
    return block_dev.repeat((reps,) + (1,) * (block_dev.dim() - 1))


def _all_tiles_equal(t, rows_per_tile):
    ref = t[:rows_per_tile]
    n = t.shape[0] // rows_per_tile
    v = t[: n * rows_per_tile].view(torch.int16).view((n, rows_per_tile) + tuple(t.shape[1:]))
    same = bool((v == ref.view(torch.int16).unsqueeze(0)).all())
    tail = t[n * rows_per_tile:]
    return same and bool((tail.view(torch.int16) == ref[: tail.shape[0]].view(torch.int16)).all())


def test_rmsnorm_beyond_2_31_elements(A):
    dt, B, H = "bf16", 64, 16384
    T = (1 << 17) + 3                                     # T*H = 2^31 + 49152 elements, 4 GiB per tensor
    print(f"[parity] rmsnorm huge T={T} H={H}", flush=True)
    x, r, w = workloads.rmsnorm_inputs(B, H, dt, np.random.default_rng(50), r_std=2.0)
    reps = -(-T // B)
    xd = _tile_rows(to_dev(x, dt), reps)[:T].contiguous()
    rd = _tile_rows(to_dev(r, dt), reps)[:T].contiguous()
    wd = to_dev(w, dt)
    A.fused_add_rmsnorm(xd, rd, wd, 1e-5)
    torch.cuda.synchronize()
    y_ref, res_ref = O.fused_add_rmsnorm(x, r, w, 1e-5, dt)
    assert_bits_equal(to_bits(rd[:B]), res_ref, "residual, first tile")
    assert_storage_close(to_bits(xd[:B]), y_ref, dt, "y, first tile")
    assert _all_tiles_equal(xd, B) and _all_tiles_equal(rd, B), "rows beyond the first tile differ"


@pytest.mark.parametrize("H,path", [(264, "vector"), (12, "phased")])
def test_rmsnorm_more_rows_than_the_grid_limit(A, H, path):
    dt, B = "f16", 256
    T = (1 << 21) + 259                                   # the row kernels launch at most 2^21 workgroups
    st, info = A.astra_plan_fused_add_rmsnorm(T, H, True)
    assert info.as_dict()["grid"] == 1 << 21 and info.as_dict()["path"] == path
    x, r, w = workloads.rmsnorm_inputs(B, H, dt, np.random.default_rng(51))
    reps = -(-T // B)
    xd = _tile_rows(to_dev(x, dt), reps)[:T].contiguous()
    rd = _tile_rows(to_dev(r, dt), reps)[:T].contiguous()
    A.fused_add_rmsnorm(xd, rd, to_dev(w, dt), 1e-6)
    torch.cuda.synchronize()
    y_ref, res_ref = O.fused_add_rmsnorm(x, r, w, 1e-6, dt)
    assert_bits_equal(to_bits(rd[:B]), res_ref, "residual, first tile")
    assert_storage_close(to_bits(xd[:B]), y_ref, dt, "y, first tile")
    assert _all_tiles_equal(xd, B) and _all_tiles_equal(rd, B)


def test_silu_beyond_2_31_elements(A):
    dt, B, d = "f16", 32, 32768
    T = (1 << 15) + 5                                     # input T*2d = 2^31 + 327680 elements
    print(f"[parity] silu huge T={T} d={d}", flush=True)
    a = workloads.silu_inputs(B, d, dt, np.random.default_rng(52))
    ad = _tile_rows(to_dev(a, dt), -(-T // B))[:T].contiguous()
    out = torch.empty((T, d), dtype=TORCH_DT[dt], device="cuda")
    A.silu_and_mul(out, ad)
    torch.cuda.synchronize()
    assert_storage_close(to_bits(out[:B]), O.silu_and_mul(a, dt), dt, "out, first tile")
    assert _all_tiles_equal(out, B)


def test_merge_beyond_2_31_elements(A):
    dt, B, NH, D = "bf16", 32, 32, 256
    T = (1 << 18) + 7                                     # T*NH*D = 2^31 + 57344 elements per v tensor
    print(f"[parity] merge huge T={T} NH={NH} D={D}", flush=True)
    va, la, vb, lb = workloads.merge_inputs(B, NH, D, dt, np.random.default_rng(53), empty_p=0.05)
    reps = -(-T // B)
    vad = _tile_rows(to_dev(va, dt), reps)[:T].contiguous()
    vbd = _tile_rows(to_dev(vb, dt), reps)[:T].contiguous()
    lad = _tile_rows(torch.from_numpy(la).cuda(), reps)[:T].contiguous()
    lbd = _tile_rows(torch.from_numpy(lb).cuda(), reps)[:T].contiguous()
    vo, lo = torch.empty_like(vad), torch.empty_like(lad)
    A.merge_attn_states_lse(vo, lo, vad, lad, vbd, lbd)
    torch.cuda.synchronize()
    vo_ref, lo_ref = O.merge_attn_states_lse(va, la, vb, lb, dt)
    assert_storage_close(to_bits(vo[:B]), vo_ref, dt, "v_out, first tile")
    assert_lse_close(lo[:B].cpu().numpy(), lo_ref, "lse_out, first tile")
    assert _all_tiles_equal(vo, B)
    n = T // B
    assert bool((lo[: n * B].view(torch.int32).view(n, B, NH) == lo[:B].view(torch.int32).unsqueeze(0)).all())


def test_output_chunk_kernels_at_their_index_limit(A):
    """silu_and_mul and merge_attn_states_lse on odd row lengths just below the 2^31 (2^32) flat output elements their
    chunk kernels index with 32 bits: every row starts at another phase, the last chunks sit at the top of the index
    range"""
    dt, B = "bf16", 32
    T, d = 1 << 16, 32767                                 # T*d = 2^31 - 65536 output elements
    assert A.astra_plan_silu_and_mul(T, d, True)[1].as_dict()["path"] == "phased"
    assert A.astra_plan_silu_and_mul(T + 3, d, True)[1].as_dict()["path"] == "ragged"
    print(f"[parity] silu at the chunk kernel's limit T={T} d={d}", flush=True)
    a = workloads.silu_inputs(B, d, dt, np.random.default_rng(54))
    ad = _tile_rows(to_dev(a, dt), T // B).contiguous()
    out = torch.empty((T, d), dtype=TORCH_DT[dt], device="cuda")
    A.silu_and_mul(out, ad)
    torch.cuda.synchronize()
    assert_storage_close(to_bits(out[:B]), O.silu_and_mul(a, dt), dt, "silu out, first tile")
    assert _all_tiles_equal(out, B)
    del ad, out
    torch.cuda.empty_cache()
    T, NH, D = 1 << 17, 32, 1023                          # 2^22 pairs of 1023 elements: 2^32 - 2^22 elements
    assert A.astra_plan_merge_attn_states_lse(T, NH, D, True)[1].as_dict()["path"] == "phased"
    assert A.astra_plan_merge_attn_states_lse(T, NH, D + 2, True)[1].as_dict()["path"] == "ragged"
    print(f"[parity] merge at the chunk kernel's limit T={T} NH={NH} D={D}", flush=True)
    va, la, vb, lb = workloads.merge_inputs(B, NH, D, dt, np.random.default_rng(55), empty_p=0.05)
    reps = T // B
    vad, vbd = _tile_rows(to_dev(va, dt), reps).contiguous(), _tile_rows(to_dev(vb, dt), reps).contiguous()
    lad, lbd = _tile_rows(torch.from_numpy(la).cuda(), reps).contiguous(), _tile_rows(torch.from_numpy(lb).cuda(), reps).contiguous()
    vo, lo = torch.empty_like(vad), torch.empty_like(lad)
    A.merge_attn_states_lse(vo, lo, vad, lad, vbd, lbd)
    torch.cuda.synchronize()
    vo_ref, lo_ref = O.merge_attn_states_lse(va, la, vb, lb, dt)
    assert_storage_close(to_bits(vo[:B]), vo_ref, dt, "merge v_out, first tile")
    assert_lse_close(lo[:B].cpu().numpy(), lo_ref, "merge lse_out, first tile")
    assert _all_tiles_equal(vo, B)
    assert bool((lo.view(torch.int32).view(reps, B, NH) == lo[:B].view(torch.int32).unsqueeze(0)).all())


def test_graph_capture_and_replay(A):
    """The entry points only enqueue kernels on the caller's stream (no allocation, no synchronisation,
    no memset), so a HIP graph can capture them.  Replays are checked against the eager result several
    times with eager work and synchronisations in between."""
    dt = "bf16"
    x, r, w = workloads.rmsnorm_inputs(16, 4096, dt, np.random.default_rng(60))
    a = workloads.silu_inputs(16, 5120, dt, np.random.default_rng(61))
    va, la, vb, lb = workloads.merge_inputs(16, 32, 128, dt, np.random.default_rng(62))
    x0, r0, wd = to_dev(x, dt), to_dev(r, dt), to_dev(w, dt)
    xd, rd = x0.clone(), r0.clone()
    ad = to_dev(a, dt)
    so = torch.empty((16, 5120), dtype=TORCH_DT[dt], device="cuda")
    vad, vbd = to_dev(va, dt), to_dev(vb, dt)
    lad, lbd = torch.from_numpy(la).cuda(), torch.from_numpy(lb).cuda()
    vo, lo = torch.empty_like(vad), torch.empty_like(lad)
    y_ref, res_ref = O.fused_add_rmsnorm(x, r, w, 1e-6, dt)
    s_ref = O.silu_and_mul(a, dt)
    vo_ref, lo_ref = O.merge_attn_states_lse(va, la, vb, lb, dt)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up on the capture stream before capturing
        A.fused_add_rmsnorm(xd, rd, wd, 1e-6)
        A.silu_and_mul(so, ad)
        A.merge_attn_states_lse(vo, lo, vad, lad, vbd, lbd)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        A.fused_add_rmsnorm(xd, rd, wd, 1e-6)
        A.silu_and_mul(so, ad)
        A.merge_attn_states_lse(vo, lo, vad, lad, vbd, lbd)
    for rep in range(4):
        xd.copy_(x0)                                   # eager work between replays: restore the in-place operands
        rd.copy_(r0)
        so.fill_(7.0)
        vo.fill_(7.0)
        lo.fill_(7.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert_bits_equal(to_bits(rd), res_ref, f"replay {rep}: residual")
        assert_storage_close(to_bits(xd), y_ref, dt, f"replay {rep}: y")
        assert_storage_close(to_bits(so), s_ref, dt, f"replay {rep}: silu")
        assert_storage_close(to_bits(vo), vo_ref, dt, f"replay {rep}: v_out")
        assert_lse_close(lo.cpu().numpy(), lo_ref, f"replay {rep}: lse_out")


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_non_finite_inputs_propagate_like_the_oracle(A, dt):
    """inf and NaN operands are outside every benchmark config; the kernels follow the formulas literally, like
    the oracle: NaN where the oracle has NaN, the same infinity where it has one, tolerance elsewhere."""
    inf, nan = np.float32(np.inf), np.float32(np.nan)
    # rmsnorm: a NaN row, a row with +inf, a row with -inf and +inf, a clean row
    T, H = 4, 4096
    x, r, w = workloads.rmsnorm_inputs(T, H, dt, np.random.default_rng(80))
    x[0, 5] = workloads.to_bits(np.array([nan]), dt)[0]
    x[1, 7] = workloads.to_bits(np.array([inf]), dt)[0]
    x[2, 9] = workloads.to_bits(np.array([inf]), dt)[0]
    r[2, 9] = workloads.to_bits(np.array([-inf]), dt)[0]
    y, res = run_rmsnorm(A, x, r, w, 1e-6, dt)
    y_ref, res_ref = O.fused_add_rmsnorm(x, r, w, 1e-6, dt)
    fin = ~np.isnan(reference_f64.widen(res_ref, dt))
    assert np.array_equal(res[fin], res_ref[fin]) and np.all(np.isnan(reference_f64.widen(res, dt)[~fin]))
    assert_storage_close(y, y_ref, dt, "rmsnorm with non-finite operands")
    # silu: x in {+inf, -inf, NaN}, g in {1, 0, inf, NaN}
    d = 256
    xs = np.zeros(d, np.float32)
    gs = np.ones(d, np.float32)
    k = 0
    for xv in (inf, -inf, nan, 2.0, -3.0, 0.0):
        for gv in (1.0, 0.0, inf, -inf, nan):
            xs[k], gs[k] = xv, gv
            k += 1
    a = workloads.to_bits(np.concatenate([xs, gs]).reshape(1, 2 * d), dt)
    assert_storage_close(run_silu(A, a, dt), O.silu_and_mul(a, dt), dt, "silu with non-finite operands")
    # merge: NaN / +inf scores and non-finite values in live and in empty partitions
    va, la, vb, lb = workloads.merge_inputs(8, 4, 64, dt, np.random.default_rng(81), empty_p=0.0)
    la[0, 0] = nan
    la[1, 0] = inf
    lb[2, 0] = -inf
    vb[2, 0, 3] = workloads.to_bits(np.array([nan]), dt)[0]       # garbage in an empty partition: never looked at
    va[3, 0, 4] = workloads.to_bits(np.array([inf]), dt)[0]
    la[4, 0] = inf
    lb[4, 0] = inf
    vo, lo = run_merge(A, va, la, vb, lb, dt)
    vo_ref, lo_ref = O.merge_attn_states_lse(va, la, vb, lb, dt)
    assert_storage_close(vo, vo_ref, dt, "merge with non-finite operands")
    assert_lse_close(lo, lo_ref, "merge lse with non-finite scores")
