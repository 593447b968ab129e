"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the headers
declare, rejects bad arguments before touching the device, and plans launches sensibly."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def A():
    import paper_2509_07506_amd as astra

    if not os.path.exists(astra.library_path()):
        from paper_2509_07506_amd import build

        build.build()
    astra.load_library()
    return astra


def _declared_functions():
    names = []
    for h in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b(astra_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


def test_every_declared_symbol_is_exported(A):
    L = ctypes.CDLL(A.library_path())
    declared = _declared_functions()
    assert {"astra_fused_add_rmsnorm", "astra_silu_and_mul", "astra_merge_attn_states_lse", "astra_status_string",
            "astra_stream_copy", "astra_plan_fused_add_rmsnorm", "astra_plan_silu_and_mul",
            "astra_plan_merge_attn_states_lse", "astra_plan_xcd_chunked", "astra_device_memory_info", "astra_merge_attn_states_lse_kway",
            "astra_fused_add_rmsnorm_strided", "astra_silu_and_mul_strided", "astra_merge_attn_states_lse_strided",
            "astra_ablation_fused_add_rmsnorm", "astra_ablation_silu_and_mul", "astra_ablation_merge_attn_states_lse"} <= set(declared)
    for name in declared:
        assert hasattr(L, name), f"{name} declared in include/ but not exported"


def test_status_strings(A):
    seen = {A.astra_status_string(i) for i in range(9)}
    assert len(seen) == 9 and A.astra_status_string(0) == "ok"
    assert "unknown" in A.astra_status_string(99)


def test_rmsnorm_validation_order(A):
    f = A.astra_fused_add_rmsnorm
    a, b, c = 0x10000, 0x20000, 0x30000          # never dereferenced: every call below fails validation
    assert f(0, b, c, 1, 8, 1, 1e-6) == 1 and f(a, 0, c, 1, 8, 1, 1e-6) == 1 and f(a, b, 0, 1, 8, 1, 1e-6) == 1
    assert f(a, b, c, -1, 8, 1, 1e-6) == 2 and f(a, b, c, 1, 0, 1, 1e-6) == 2 and f(a, b, c, 1 << 40, 1 << 40, 1, 1e-6) == 2
    assert f(a, b, c, 1, 8, 3, 1e-6) == 3 and f(a, b, c, 1, 8, -1, 1e-6) == 3
    assert f(a, b, c, 1, 8, 1, -1e-6) == 4 and f(a, b, c, 1, 8, 1, float("nan")) == 4
    assert f(a, b, c, 0, 1 << 62, 1, 1e-6) == 2                       # the row length is bounded on its own, also when T == 0
    assert f((1 << 64) - 0x1000, b, c, 64, 4096, 1, 1e-6) == 6        # a tensor that wraps around the address space is refused
    assert f(a + 1, b, c, 1, 8, 1, 1e-6) == 5
    assert f(a, a + 8, c, 1, 8, 1, 1e-6) == 6 and f(a, b, a + 2, 1, 8, 1, 1e-6) == 6
    # precedence: null before shape before dtype before eps before alignment before aliasing
    assert f(0, b, c, -1, 8, 7, -1.0) == 1
    assert f(a, b, c, -1, 8, 7, -1.0) == 2
    assert f(a, b, c, 1, 8, 7, -1.0) == 3
    assert f(a + 1, b, c, 1, 8, 1, -1.0) == 4
    assert f(a + 1, a + 3, c, 1, 8, 1, 1.0) == 5
    # T == 0 is fine and launches nothing (works without a GPU)
    assert f(a, b, c, 0, 8, 1, 1e-6) == 0
    # binary32 storage (dtype 2): 4-byte alignment, and extents counted in 4-byte elements
    assert f(a + 2, b, c, 1, 8, 2, 1e-6) == 5 and f(a + 2, b, c, 0, 8, 1, 1e-6) == 0
    assert f(a, a + 16, c, 1, 8, 2, 1e-6) == 6 and f(a, a + 32, c, 0, 8, 2, 1e-6) == 0
    assert f(a, b, b + 4 * 8 * 4 - 4, 4, 8, 2, 1e-6) == 6      # weight inside the last residual row


def test_silu_validation(A):
    f = A.astra_silu_and_mul
    a, b = 0x10000, 0x40000
    assert f(0, b, 1, 8, 1) == 1 and f(a, 0, 1, 8, 1) == 1
    assert f(a, b, -2, 8, 1) == 2 and f(a, b, 1, 0, 1) == 2 and f(a, b, 1 << 62, 8, 1) == 2
    assert f(a, b, 1, 8, 3) == 3
    assert f(a + 1, b, 1, 8, 1) == 5
    assert f(a, a + 16, 4, 8, 1) == 6 and f(a + 32, a, 4, 8, 1) == 6
    assert f(a, b, 0, 8, 0) == 0
    assert f(a + 2, b, 1, 8, 2) == 5 and f(a, a + 16, 1, 8, 2) == 6   # binary32: out spans 32 bytes


def test_merge_validation(A):
    f = A.astra_merge_attn_states_lse
    vo, lo, va, la, vb, lb = 0x10000, 0x20000, 0x30000, 0x40000, 0x50000, 0x60000
    for i in range(6):
        args = [vo, lo, va, la, vb, lb]
        args[i] = 0
        assert f(*args, 1, 2, 8, 1) == 1
    assert f(vo, lo, va, la, vb, lb, -1, 2, 8, 1) == 2 and f(vo, lo, va, la, vb, lb, 1, 0, 8, 1) == 2
    assert f(vo, lo, va, la, vb, lb, 1, 2, 0, 1) == 2 and f(vo, lo, va, la, vb, lb, 1 << 30, 1 << 30, 1 << 30, 1) == 2
    assert f(vo, lo, va, la, vb, lb, 1, 2, 8, 4) == 3
    assert f(vo, lo + 2, va, la, vb, lb, 1, 2, 8, 1) == 5 and f(vo + 1, lo, va, la, vb, lb, 1, 2, 8, 1) == 5
    assert f(vo, lo, vo + 2, la, vb, lb, 4, 2, 8, 1) == 6          # partial overlap of v_out and v_a
    assert f(vo, la, va, la, vb, lb, 4, 2, 8, 1) == 6              # lse_out on lse_a
    assert f(vo, lo, va, la, vb, lb, 0, 2, 8, 1) == 0
    assert f(va, lo, va, la, vb, lb, 0, 2, 8, 1) == 0              # exact aliasing of v_out and v_a is allowed
    assert f(vo + 2, lo, va, la, vb, lb, 1, 2, 8, 2) == 5          # binary32 storage: 4-byte alignment
    assert f(vo, lo, vo + 32, la, vb, lb, 1, 2, 8, 2) == 6          # 64-byte tensors 32 bytes apart


def test_strided_silu_and_merge_validation(A):
    f = A.astra_silu_and_mul_strided
    a, b = 0x10000, 0x40000
    assert f(0, 8, b, 16, 1, 8, 1) == 1 and f(a, 8, 0, 16, 1, 8, 1) == 1
    assert f(a, 7, b, 16, 2, 8, 1) == 2 and f(a, 8, b, 15, 2, 8, 1) == 2 and f(a, 8, b, 16, -1, 8, 1) == 2
    assert f(a, 1 << 61, b, 1 << 61, 8, 8, 1) == 2                      # extent overflows
    assert f(a, 8, b, 16, 2, 8, 9) == 3
    assert f(a + 1, 8, b, 16, 2, 8, 1) == 5
    assert f(a, 8, a + 24, 16, 2, 8, 1) == 6                            # out rows [a, a+32) meet input [a+24, ...)
    assert f(a, 64, a + 64, 64, 2, 8, 1) == 6                           # interleaved views: bounding ranges overlap
    assert f(a, 8, b, 16, 0, 8, 1) == 0
    big_d = (1 << 14) + 8                                               # 2049 vectors per row, 2^20 rows: over 2^31 vectors
    assert f(a, big_d, b, 2 * big_d, 1 << 20, big_d, 1) == 2
    g = A.astra_merge_attn_states_lse_strided
    vo, lo, va, la, vb, lb = 0x100000, 0x200000, 0x300000, 0x400000, 0x500000, 0x600000

    def call(T=2, NH=2, D=8, dt=1, **kw):
        p = dict(vo=vo, ots=16, ohs=8, lo=lo, va=va, ats=16, ahs=8, la=la, vb=vb, bts=16, bhs=8, lb=lb)
        p.update(kw)
        return g(p["vo"], p["ots"], p["ohs"], p["lo"], p["va"], p["ats"], p["ahs"], p["la"], p["vb"], p["bts"], p["bhs"],
                 p["lb"], T, NH, D, dt)

    for key in ("vo", "lo", "va", "la", "vb", "lb"):
        assert call(**{key: 0}) == 1
    assert call(T=-1) == 2 and call(NH=0) == 2 and call(ahs=7) == 2 and call(ats=15) == 2 and call(ots=1 << 61) == 2
    assert call(dt=5) == 3
    assert call(va=va + 1) == 5 and call(lo=lo + 2) == 5
    assert call(va=vo + 8) == 6                                          # v_out partly on v_a
    assert call(T=0, va=vo) == 0                                         # same view, nothing to do
    assert call(va=vo, ats=32) == 6                                      # same pointer but another stride: not the same view
    assert call(lo=la) == 6
    assert call(T=0) == 0
    assert call(T=1 << 24, NH=64, D=136, ots=64 * 136, ohs=136, ats=64 * 136, ahs=136, bts=64 * 136, bhs=136) == 2   # 2^30 pairs x 17 vectors


def test_stream_copy_validation(A):
    f = A.astra_stream_copy
    assert f(0, 16, 16) == 1 and f(0x1000, 0x2000, -16) == 2 and f(0x1000, 0x2000, 24) == 2
    assert f(0x1008, 0x2000, 16) == 5 and f(0x1000, 0x1010, 32) == 6 and f(0x1000, 0x2000, 0) == 0


def test_rmsnorm_plans(A):
    def plan(T, H, al=True):
        st, i = A.astra_plan_fused_add_rmsnorm(T, H, al)
        assert st == 0
        return i.as_dict()

    assert plan(0, 4096)["path"] == "none"
    for T in (1, 8):                          # decode: widest block, one vector per lane, plain launch order
        assert plan(T, 8192) == {"path": "vector", "block": 1024, "vectors_per_lane": 1, "log2_xcd_chunk": 0, "grid": T,
                                 "pace": 0}
    assert plan(16, 4096) == {"path": "vector", "block": 512, "vectors_per_lane": 1, "log2_xcd_chunk": 0, "grid": 16,
                              "pace": 0}
    for T, H in [(8192, 8192), (32768, 8192), (4099, 5120), (4099, 7168), (1024, 4096), (512, 14336), (128, 11008),
                 (64, 8192), (257, 5120)]:
        p = plan(T, H)
        lc = p["log2_xcd_chunk"]
        assert p["path"] == "vector" and p["block"] % 64 == 0 and p["block"] <= 1024
        assert p["block"] * p["vectors_per_lane"] * 8 >= H           # the whole row is register resident
        assert p["block"] * p["vectors_per_lane"] * 8 < 1.25 * H + 512
        assert T <= p["grid"] < T + (8 << lc) and (lc == 0 or p["grid"] % (8 << lc) == 0)
        assert lc == 0 or (T >= (64 << lc) and T >= 1024)              # small grids keep the plain launch order
        if T >= 4096:
            assert 128 * 1024 <= (H * 2) << lc <= 512 * 1024           # about 256 KiB per XCD run
    # rows that are no whole number of vectors on tensors that are in step with each other (16-byte aligned, al=1, or all
    # offset alike, al=2): phased path -- lanes own the aligned chunks a row covers, counted from the start of the 128-byte
    # line the row begins in: at most floor((H + 63 + 7) / 8) chunk slots
    assert plan(4, 4100) == {"path": "phased", "block": 576, "vectors_per_lane": 1, "log2_xcd_chunk": 0, "grid": 4, "pace": 0}
    assert plan(4, 4096, al=2) == {"path": "phased", "block": 576, "vectors_per_lane": 1, "log2_xcd_chunk": 0, "grid": 4, "pace": 0}
    assert plan(9, 32700)["path"] == "phased" and plan(3, 8)["path"] == "vector" and plan(3, 9)["path"] == "phased"
    assert plan(3, 8, al=2)["path"] == "phased" and plan(4, 8129)["block"] == 1024 and plan(4, 8130)["vectors_per_lane"] == 2
    assert plan(4, 32705)["path"] == "phased" and plan(4, 32706)["path"] == "ragged"       # one chunk slot more than 4096: old form
    p = plan(4099, 5124)
    assert p["path"] == "phased" and p["log2_xcd_chunk"] == 5 and p["grid"] == 4352 and p["block"] == 704
    # rows of whole vectors that are no whole number of 128-byte lines (from 4 KiB on): the same kernel, whose waves stay on
    # whole lines; below 4 KiB and for whole lines the fast kernel
    # (streaming grids only: 32 rows per compute unit or more)
    assert plan(8192, 4104) == {"path": "phased", "block": 576, "vectors_per_lane": 1, "log2_xcd_chunk": 5, "grid": 8192, "pace": 0}
    assert plan(8192, 8200)["path"] == "phased" and plan(8192, 8200)["vectors_per_lane"] == 2
    assert plan(8192, 2056)["path"] == "phased" and plan(8192, 2040)["path"] == "vector" and plan(8192, 1032)["path"] == "vector"
    assert plan(8192, 4160)["path"] == "vector" and plan(8192, 32712)["path"] == "vector"  # 65 lines; too long for the line grid
    assert plan(8191, 4104)["path"] == "vector" and plan(4, 8200)["path"] == "vector"
    # tensors at unrelated offsets into the 16-byte grid (al=0): ragged path, row in registers (lanes for the whole
    # vectors; the tail of fewer than 8 elements rides in the last lane)
    assert plan(4, 4100, al=0) == {"path": "ragged", "block": 512, "vectors_per_lane": 1, "log2_xcd_chunk": 0, "grid": 4, "pace": 0}
    assert plan(4, 4096, al=0)["path"] == "ragged" and plan(9, 32767, al=0)["path"] == "ragged" and plan(3, 9, al=0)["path"] == "ragged"
    assert plan(3, 8, al=0)["path"] == "ragged"
    for al in (0, 1, 2):
        assert plan(3, 1, al)["path"] == "generic" and plan(3, 7, al)["path"] == "generic"      # not one whole vector in a row
        assert plan(4, 65536 + (al != 1), al)["path"] == "generic" and plan(4, 32776, al)["path"] == "generic"   # more than 4096 vectors
    assert plan(4, 11009, al=0)["vectors_per_lane"] == 2 and plan(4, 32767, al=0)["vectors_per_lane"] == 4
    assert plan(1 << 22, 100, al=0) == {"path": "ragged", "block": 64, "vectors_per_lane": 1, "log2_xcd_chunk": 8, "grid": 1 << 21,
                                        "pace": 0}
    assert plan(1 << 22, 100)["path"] == "phased" and plan(1 << 22, 100)["grid"] == 1 << 21
    p = plan(4099, 5124, al=0)
    assert p["path"] == "ragged" and p["log2_xcd_chunk"] == 5 and p["grid"] == 4352 and p["block"] == 640
    assert plan(4, 32775, al=0)["path"] == "ragged" and plan(4, 8199, al=0)["vectors_per_lane"] == 1
    big = plan(1 << 23, 264)                                           # row loop beyond the grid limit
    assert big["grid"] == 1 << 21 and big["grid"] % (8 << big["log2_xcd_chunk"]) == 0
    # rows of at most 32 vectors share a workgroup: 8, 16 or 32 lanes per row, 256-lane workgroups
    # ... and single-wave workgroups on streaming grids when the rows fill their lane groups (H = 64, 128, 256)
    assert plan(1 << 23, 64) == {"path": "vector", "block": 64, "vectors_per_lane": 1, "log2_xcd_chunk": 8, "grid": 1 << 20,
                                 "pace": 0, "rows_per_block": 8}
    assert plan(1 << 21, 256)["block"] == 64 and plan(1 << 21, 256)["rows_per_block"] == 2
    assert plan(1 << 22, 128)["block"] == 64 and plan(1 << 22, 128)["rows_per_block"] == 4
    assert plan(1 << 23, 72)["block"] == 256 and plan(1 << 22, 192)["block"] == 256      # rows that leave lanes of their group idle
    assert plan(100000, 64)["block"] == 256                                               # under 4096 workgroups of 256 lanes
    assert plan(1 << 25, 64)["block"] == 256 and plan(1 << 25, 64)["rows_per_block"] == 32  # 64-lane workgroups: over the grid limit
    assert plan(1000, 128)["rows_per_block"] == 16 and plan(1000, 128)["grid"] == 63 and plan(1000, 136)["rows_per_block"] == 8
    assert plan(5, 256)["rows_per_block"] == 8 and plan(5, 256)["grid"] == 1 and "rows_per_block" not in plan(5, 264)
    assert "rows_per_block" not in plan(5, 260) and plan(5, 260)["path"] == "phased" and plan(5, 260, al=0)["path"] == "ragged"
    assert plan(1 << 26, 8)["rows_per_block"] == 32 and plan(1 << 26, 8)["grid"] == 1 << 21
    assert "rows_per_block" not in plan((1 << 26) + 1, 8) and plan((1 << 26) + 1, 8)["block"] == 64   # beyond the grid limit: row loop
    assert A.astra_plan_fused_add_rmsnorm(-1, 8, True)[0] == 2
    # request pacing: none while a compute unit requests under 48 KiB at once and for the row-loop kernel; on streaming
    # grids (three rounds or more) "store gap" (4) by default on long grids, and a pace of its own for the row lengths that
    # beat the default on nearly every buffer placement (bench.py --pacing): weight-then-x-then-r (1 | 2), x-then-r (2)
    assert plan(255, 8192)["pace"] == 0 and plan(512, 4096)["pace"] == 0 and big["pace"] == 0
    for T, H, pace in [(32768, 8192, 3), (32768, 2048, 3), (32768, 1024, 3), (32768, 1536, 3), (2048, 14336, 3), (32768, 10240, 3),
                       (32768, 2560, 2), (32768, 3072, 2), (2048, 16384, 2),
                       (32768, 4096, 4), (32768, 5120, 4), (32768, 6144, 4), (32768, 7168, 4), (32768, 7680, 4), (32768, 11008, 4),
                       (32768, 12288, 4), (16384, 32768, 4), (1 << 20, 512, 4)]:
        assert plan(T, H)["pace"] == pace, (T, H, plan(T, H))
    # two-vector rows of 28 KiB or more on grids of 16 rows per compute unit or more: one workgroup per compute unit at a
    # time (8), paced weight-then-x-then-r
    for T, H, pace in [(4096, 14336, 11), (8192, 16384, 11), (4096, 15360, 11), (4096, 20480, 0), (4096, 24576, 0),
                       (4095, 16384, 11), (3840, 16384, 2), (4096, 14328, 0), (4096, 16392, 0), (4096, 28672, 0), (4096, 12288, 0)]:
        assert plan(T, H)["pace"] == pace, (T, H, plan(T, H))
    # ... the gap only where its extra microsecond at the end of the grid is small change (32 rounds or more)
    assert plan(4099, 5120)["pace"] == 0 and plan(2048, 28672)["pace"] == 0 and plan(4099, 7168)["pace"] == 0
    assert plan(13107, 20480)["pace"] == 0 and plan(9362, 28672)["pace"] == 0
    assert plan(2048, 3072)["pace"] == 2 and plan(2048, 32768)["pace"] == 0
    assert plan(2048, 11008)["vectors_per_lane"] == 2 and plan(2048, 28672)["vectors_per_lane"] == 4
    # grids of under three rounds: x-then-r once a compute unit requests 48 KiB at once ...
    for T, H in [(1023, 8192), (512, 8192), (768, 8192), (1024, 4096), (2048, 4096), (2048, 2048), (1024, 7168)]:
        p = plan(T, H)
        assert p["pace"] == 2 and p["vectors_per_lane"] == 1, (T, H)
    # ... and half-sized workgroups with two vectors per lane where the rows no longer fit at once but stay within
    # 88 KiB per compute unit
    for T, H, block in [(1280, 4096, 256), (1024, 5120, 320), (768, 5120, 320), (1536, 3072, 192), (2560, 2048, 128),
                        (768, 6144, 384), (600, 7168, 448), (5000, 1024, 64)]:
        p = plan(T, H)
        assert (p["vectors_per_lane"], p["block"], p["pace"]) == (2, block, 2), (T, H, p)
    for T, H in [(1024, 4096), (1536, 4096), (1024, 8192), (768, 8192), (3072, 2048), (512, 5120), (1280, 5120)]:
        assert plan(T, H)["vectors_per_lane"] == 1, (T, H)
    # two-vector rows that fill the compute units exactly: four vectors per lane in half-sized workgroups
    for T, H, block in [(512, 14336, 448), (300, 12288, 384), (512, 16384, 512), (400, 10240, 320)]:
        p = plan(T, H)
        assert (p["vectors_per_lane"], p["block"], p["pace"]) == (4, block, 2), (T, H, p)
    for T, H in [(256, 14336), (513, 14336), (512, 9216), (1024, 16384)]:
        assert plan(T, H)["vectors_per_lane"] == 2, (T, H)
    assert A.astra_plan_fused_add_rmsnorm(1280, 2048, True, dtype=A.ASTRA_F32)[1].as_dict()["vectors_per_lane"] == 2
    assert A.astra_plan_fused_add_rmsnorm(32768, 4096, True, dtype=A.ASTRA_F32)[1].as_dict()["pace"] == 3   # 16 KiB rows
    assert A.astra_plan_fused_add_rmsnorm(32768, 8192, True, dtype=A.ASTRA_F32)[1].as_dict()["pace"] == 11  # 32 KiB rows: one resident workgroup
    assert A.astra_plan_silu_and_mul(4096, 14336, True)[1].as_dict()["pace"] == 0


def test_binary32_plans(A):
    """Four elements per 16-byte vector: the same geometry rules in vectors, twice the vectors per row."""
    F32 = A.ASTRA_F32
    p = A.astra_plan_fused_add_rmsnorm(8192, 4096, True, dtype=F32)[1].as_dict()
    q = A.astra_plan_fused_add_rmsnorm(8192, 8192, True, dtype=A.ASTRA_BF16)[1].as_dict()
    assert p == q                                                     # 16 KiB rows either way
    for T, H in [(1, 8192), (600, 8192), (64, 16384), (4099, 5120)]:
        p = A.astra_plan_fused_add_rmsnorm(T, H, True, dtype=F32)[1].as_dict()
        assert p["path"] == "vector" and p["block"] * p["vectors_per_lane"] * 4 >= H and p["block"] <= 1024
    assert A.astra_plan_fused_add_rmsnorm(4, 4098, True, dtype=F32)[1].as_dict()["path"] == "phased"    # H % 4 != 0
    assert A.astra_plan_fused_add_rmsnorm(4, 4098, 0, dtype=F32)[1].as_dict()["path"] == "ragged"
    assert A.astra_plan_fused_add_rmsnorm(4, 4128, True, dtype=F32)[1].as_dict()["path"] == "vector"    # H % 4 == 0, whole lines
    assert A.astra_plan_fused_add_rmsnorm(4, 4100, True, dtype=F32)[1].as_dict()["path"] == "vector"
    assert A.astra_plan_fused_add_rmsnorm(8192, 4100, True, dtype=F32)[1].as_dict()["path"] == "phased"  # H % 4 == 0, no whole lines
    assert A.astra_plan_fused_add_rmsnorm(4, 32768, True, dtype=F32)[1].as_dict()["path"] == "generic"  # > 4096 vectors
    s = A.astra_plan_silu_and_mul(4096, 14336, True, dtype=F32)[1].as_dict()
    assert s["path"] == "vector" and s["block"] == 64 and s["grid"] * s["block"] >= 4096 * 14336 // 4
    assert A.astra_plan_silu_and_mul(3, 1410, True, dtype=F32)[1].as_dict()["path"] == "phased"
    assert A.astra_plan_silu_and_mul(3, 3, True, dtype=F32)[1].as_dict()["path"] == "ragged"            # rows under one vector
    assert A.astra_plan_silu_and_mul(3, 1412, True, dtype=F32)[1].as_dict()["path"] == "vector"
    m = A.astra_plan_merge_attn_states_lse(4096, 32, 128, True, dtype=F32)[1].as_dict()
    assert m["path"] == "vector" and m["block"] == 64 and m["grid"] * m["block"] == 4096 * 32 * 32
    assert A.astra_plan_merge_attn_states_lse(3, 5, 6, True, dtype=F32)[1].as_dict()["path"] == "phased"
    assert A.astra_plan_merge_attn_states_lse(3, 5, 6, 0, dtype=F32)[1].as_dict()["path"] == "phased"
    assert A.astra_plan_merge_attn_states_lse(3, 5, 3, True, dtype=F32)[1].as_dict()["path"] == "ragged"     # head_dim under one vector
    assert A.astra_plan_merge_attn_states_lse(3, 5, 4, True, dtype=F32)[1].as_dict()["path"] == "vector"
    assert A.astra_plan_merge_attn_states_lse(3, 5, 4, True, dtype=7)[0] == 3
    assert A.astra_plan_merge_attn_states_lse(-3, 5, 4, True, dtype=7)[0] == 2                          # shape before dtype


def test_silu_and_merge_plans(A):
    st, i = A.astra_plan_silu_and_mul(4096, 14336, True)
    p = i.as_dict()
    work = 4096 * 14336 // 8
    assert st == 0 and p["path"] == "vector"
    assert work <= p["grid"] * p["block"] * p["vectors_per_lane"] < work + (8 << p["log2_xcd_chunk"]) * 256
    assert p["grid"] % (8 << p["log2_xcd_chunk"]) == 0
    # every other dense call with rows of at least one vector: the aligned chunks of memory the output covers (aligned
    # stores, loads at element alignment), at most one more than its vectors; rows under eight vectors: 16-byte accesses
    # at element alignment
    assert A.astra_plan_silu_and_mul(3, 100, True)[1].as_dict() == {"path": "phased", "block": 256, "vectors_per_lane": 1,
                                                                    "log2_xcd_chunk": 0, "grid": 1, "pace": 0}   # 38 + 1 chunks
    assert A.astra_plan_silu_and_mul(3, 7, True)[1].as_dict() == {"path": "ragged", "block": 256, "vectors_per_lane": 1,
                                                                  "log2_xcd_chunk": 0, "grid": 1, "pace": 0}
    assert A.astra_plan_silu_and_mul(3, 63, True)[1].as_dict()["path"] == "ragged"          # rows under eight vectors
    assert A.astra_plan_silu_and_mul(3, 65, True)[1].as_dict()["path"] == "phased" and A.astra_plan_silu_and_mul(3, 64, 2)[1].as_dict()["path"] == "phased"
    assert A.astra_plan_silu_and_mul(3, 1408, False)[1].as_dict()["path"] == "phased"
    ph = A.astra_plan_silu_and_mul(4096, 14336, 2)[1].as_dict()
    assert ph == {"path": "phased", "block": 64, "vectors_per_lane": 1, "log2_xcd_chunk": 8, "grid": 114688 + 2048, "pace": 0}
    assert A.astra_plan_silu_and_mul(3, 1408, 2)[1].as_dict() == {"path": "phased", "block": 256, "vectors_per_lane": 1,
                                                                  "log2_xcd_chunk": 0, "grid": 3, "pace": 0}
    assert A.astra_plan_silu_and_mul(3, 1410, 2)[1].as_dict()["path"] == "phased" and A.astra_plan_silu_and_mul(3, 1410, 0)[1].as_dict()["path"] == "phased"
    assert A.astra_plan_silu_and_mul(1 << 17, 1 << 14, 2)[1].as_dict()["path"] == "phased"  # 2^31 output elements: the most
    assert A.astra_plan_silu_and_mul((1 << 17) + 1, 1 << 14, 2)[1].as_dict()["path"] == "ragged"
    assert A.astra_plan_silu_and_mul(1 << 20, (1 << 14) + 1, True)[1].as_dict()["path"] == "generic"
    assert A.astra_plan_silu_and_mul(3, 128, True)[1].as_dict()["path"] == "vector"       # short rows: per-lane division
    assert A.astra_plan_silu_and_mul(1000, 8, True)[1].as_dict() == {"path": "vector", "block": 256, "vectors_per_lane": 1,
                                                                     "log2_xcd_chunk": 0, "grid": 8, "pace": 0,
                                                                     "access_bytes": 8, "non_temporal": 0}   # small: half vectors
    # the input's 2^32 vectors are beyond the vector kernel's 32-bit index; the ragged kernel indexes the 2^31 output vectors
    assert A.astra_plan_silu_and_mul(1 << 20, 1 << 14, True)[1].as_dict()["path"] == "ragged"
    small = A.astra_plan_silu_and_mul(3, 1408, True)[1].as_dict()
    assert small["log2_xcd_chunk"] == 0 and small["grid"] == 5                           # 3 * 352 half vectors, no padding for small grids
    st, i = A.astra_plan_merge_attn_states_lse(4096, 32, 128, True)
    p = i.as_dict()
    assert st == 0 and p["path"] == "vector" and p["grid"] * p["block"] * p["vectors_per_lane"] == 4096 * 32 * 16
    # workgroup width of the flat kernels: one wave on streaming grids, 128 lanes when 256-lane workgroups would be
    # fewer than the compute units (but more than 32), 256 lanes otherwise; the grid always covers the work
    for T, d, block in [(64, 8192, 256), (100, 4096, 128), (128, 11008, 256), (2048, 11008, 64)]:
        q = A.astra_plan_silu_and_mul(T, d, True)[1].as_dict()
        assert q["block"] == block and "access_bytes" not in q and "non_temporal" not in q, (T, d, q)
        assert T * d // 8 <= q["grid"] * block < T * d // 8 + max(block, (8 << q["log2_xcd_chunk"]) * block), (T, d, q)
    # small problems (under 2^15 output vectors): plain accesses; silu_and_mul with half a vector per lane
    for T, d in [(1, 8), (16, 4096), (32, 5120), (16, 12288), (63, 4160)]:
        q = A.astra_plan_silu_and_mul(T, d, True)[1].as_dict()
        assert q["access_bytes"] == 8 and q["non_temporal"] == 0 and q["block"] == 256 and q["log2_xcd_chunk"] == 0, (T, d, q)
        assert T * d // 4 <= q["grid"] * 256 < T * d // 4 + 256
    assert "access_bytes" not in A.astra_plan_silu_and_mul(64, 4096, True)[1].as_dict()        # exactly 2^15 vectors: streaming form
    for T, block, nt in [(1, 256, 0), (16, 256, 0), (63, 128, 0), (64, 128, 1), (200, 256, 1), (1024, 256, 1), (2048, 64, 1), (32768, 64, 1)]:
        q = A.astra_plan_merge_attn_states_lse(T, 32, 128, True)[1].as_dict()
        assert q["block"] == block and q.get("non_temporal", 1) == nt and "access_bytes" not in q, (T, q)
    assert A.astra_plan_merge_attn_states_lse(3, 5, 4, True)[1].as_dict()["path"] == "ragged"                 # head_dim under one vector
    assert A.astra_plan_merge_attn_states_lse(3, 5, 72, False)[1].as_dict()["path"] == "phased"
    # head_dim or pointers off the 16-byte grid: aligned chunks of the flat output (loads at element alignment)
    q = A.astra_plan_merge_attn_states_lse(257, 40, 129, True)[1].as_dict()
    assert q["path"] == "phased" and q["block"] == 256 and q["grid"] * 256 >= (257 * 40 * 129 + 7) // 8 + 1
    # workgroup width as for the fast kernel: single waves on streaming grids, 128 lanes under one workgroup per compute unit
    for T, block in [(16384, 64), (4096, 64), (64, 128), (3, 256)]:
        q = A.astra_plan_merge_attn_states_lse(T, 32, 129, True)[1].as_dict()
        chunks = (T * 32 * 129 + 7) // 8 + 1
        assert q["path"] == "phased" and q["block"] == block and q["grid"] * block >= chunks, (T, q)
        assert q["grid"] % (8 << q["log2_xcd_chunk"]) == 0 or q["log2_xcd_chunk"] == 0
    assert A.astra_plan_merge_attn_states_lse(3, 5, 72, 2)[1].as_dict()["path"] == "phased"
    assert A.astra_plan_merge_attn_states_lse(1 << 16, 512, 129, True)[1].as_dict()["path"] == "ragged"       # 2^32 elements and more
    assert A.astra_plan_merge_attn_states_lse(1 << 24, 64, 129, True)[1].as_dict()["path"] == "generic"   # 2^30 * 17 vectors
    assert A.astra_plan_merge_attn_states_lse(3, 5, 72, True)[1].as_dict()["path"] == "vector"
    assert A.astra_plan_merge_attn_states_lse(0, 5, 72, True)[1].as_dict()["path"] == "none"


def test_xcd_chunked_is_a_permutation_with_contiguous_runs(A):
    """workgroup b runs on XCD b % 8; the map must cover [0, G) exactly once and give each XCD runs of
    2^lc consecutive units."""
    for lc in range(0, 9):
        C = 1 << lc
        G = 8 * C * 3
        image = [A.astra_plan_xcd_chunked(b, lc) for b in range(G)]
        assert sorted(image) == list(range(G))
        for xcd in range(8):
            seq = [image[b] for b in range(xcd, G, 8)]           # what this XCD executes, in launch order
            for k in range(0, len(seq), C):
                run = seq[k:k + C]
                assert run == list(range(run[0], run[0] + C)) and run[0] % C == 0
    assert [A.astra_plan_xcd_chunked(b, 0) for b in range(20)] == list(range(20))
    assert A.astra_plan_xcd_chunked(5, 99) == 5


def test_ablation_variant_validation(A):
    """same validation as the plain entry points, then the variant check; nothing here reaches the device"""
    a, b, c = 0x10000, 0x20000, 0x30000
    f = A.astra_ablation_fused_add_rmsnorm
    assert f(0, b, c, 1, 8, 1, 1e-6, 1) == 1 and f(a, b, c, -1, 8, 1, 1e-6, 1) == 2 and f(a, b, c, 1, 8, 9, 1e-6, 1) == 3
    assert f(a, b, c, 1, 8, 1, 1e-6, 3) == 8 and f(a, b, c, 1, 8, 1, 1e-6, 4) == 8 and f(a, b, c, 1, 8, 1, 1e-6, -1) == 8
    assert f(a, b, c, 1, 12, 1, 1e-6, 2) == 8            # H % 8 != 0: not the fast path
    assert f(a, b, c, 1, 32768, 1, 1e-6, 1) == 8         # scalar-load variant keeps at most 16 elements per lane
    assert f(a, b, c, 0, 8, 1, 1e-6, 2) == 0
    g = A.astra_ablation_silu_and_mul
    assert g(a, b, 1, 512, 1, 2) == 8 and g(a, b, 1, 512, 1, 3) == 8 and g(a, b, 1, 100, 1, 1) == 8 and g(a, b, 0, 512, 1, 4) == 0
    h = A.astra_ablation_merge_attn_states_lse
    vo, lo, va, la, vb, lb = 0x10000, 0x20000, 0x30000, 0x40000, 0x50000, 0x60000
    assert h(vo, lo, va, la, vb, lb, 1, 2, 8, 1, 2) == 8 and h(vo, lo, va, la, vb, lb, 1, 2, 8, 1, 4) == 8
    assert h(vo, lo, va, la, vb, lb, 1, 2, 4, 1, 3) == 8 and h(vo, lo, va, la, vb, lb, 0, 2, 8, 1, 3) == 0


def test_kway_validation_without_gpu(A):
    g = A.astra_merge_attn_states_lse_kway
    vo, lo, vp, lp = 0x10000, 0x20000, 0x100000, 0x200000
    assert g(0, lo, vp, lp, 2, 1, 2, 8, 1) == 1 and g(vo, lo, vp, 0, 2, 1, 2, 8, 1) == 1
    assert g(vo, lo, vp, lp, 0, 1, 2, 8, 1) == 2 and g(vo, lo, vp, lp, 65537, 1, 2, 8, 1) == 2 and g(vo, lo, vp, lp, 2, -1, 2, 8, 1) == 2
    assert g(vo, lo, vp, lp, 2, 1, 2, 8, 5) == 3
    assert g(vo + 1, lo, vp, lp, 2, 1, 2, 8, 1) == 5 and g(vo, lo + 2, vp, lp, 2, 1, 2, 8, 1) == 5
    assert g(vp + 32, lo, vp, lp, 3, 1, 2, 8, 1) == 6                  # output inside the second part
    assert g(vo, lo, vp, lp, 2, 0, 2, 8, 1) == 0
    assert g(vo, lo, vp, lp, 2, 1 << 24, 64, 136, 1) == 2             # 2^30 pairs x 17 vectors: over 2^31 output vectors


def test_strided_validation_without_gpu(A):
    f = A.astra_fused_add_rmsnorm_strided
    y, ro, x, r, w = 0x100000, 0x200000, 0x300000, 0x400000, 0x500000
    assert f(0, 16, ro, 16, x, 16, r, 16, w, 4, 8, 1, 1e-6) == 1 and f(y, 16, ro, 16, x, 16, r, 16, 0, 4, 8, 1, 1e-6) == 1
    assert f(y, 7, ro, 16, x, 16, r, 16, w, 4, 8, 1, 1e-6) == 2 and f(y, 16, ro, 16, x, 16, r, 1 << 62, w, 4, 8, 1, 1e-6) == 2
    assert f(y, 16, ro, 16, x, 16, r, 16, w, 4, 8, 3, 1e-6) == 3 and f(y, 16, ro, 16, x, 16, r, 16, w, 4, 8, 1, float("nan")) == 4
    assert f(y, 16, ro + 1, 16, x, 16, r, 16, w, 4, 8, 1, 1e-6) == 5
    assert f(x, 32, ro, 16, x, 16, r, 16, w, 4, 8, 1, 1e-6) == 6 and f(y, 16, r + 2, 16, x, 16, r, 16, w, 4, 8, 1, 1e-6) == 6
    assert f(x, 16, r, 16, x, 16, r, 16, w, 0, 8, 1, 1e-6) == 0          # in place, nothing to do


def test_binding_refuses_cpu_tensors(A):
    import torch

    x = torch.zeros((2, 64), dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        A.fused_add_rmsnorm(x, x.clone(), torch.ones(64, dtype=torch.bfloat16), 1e-6)


def test_stream_probe_validation(A):
    f = A.astra_stream_probe
    a, b, c = 0x10000, 0x20000, 0x30000          # never dereferenced: every call below fails validation or moves nothing
    assert f(a, b, c, 16, 5) == 2 and f(a, b, c, 16, -1) == 2                       # unknown mode
    assert f(0, b, c, 16, A.ASTRA_PROBE_COPY) == 1 and f(a, 0, 0, 16, A.ASTRA_PROBE_COPY) == 1
    assert f(a, 0, c, 16, A.ASTRA_PROBE_READ2) == 1 and f(a, b, 0, 16, A.ASTRA_PROBE_READ2_WRITE1) == 1
    assert f(0, 0, 0, 16, A.ASTRA_PROBE_WRITE1) == 1 and f(a, 0, 0, 16, A.ASTRA_PROBE_UPDATE2) == 1
    assert f(a, b, c, -16, 0) == 2 and f(a, b, c, 24, 0) == 2 and f(a, b, c, (1 << 35) + 16, 0) == 2
    assert f(a + 8, b, c, 16, 0) == 5 and f(a, b + 4, c, 16, 3) == 5 and f(a, b, c + 2, 16, 2) == 5
    assert f(a, b, a + 16, 64, 0) == 6 and f(a, a, c, 64, 3) == 6 and f(a, b, b, 64, 3) == 6 and f(a, a + 32, 0, 64, 4) == 6
    assert f(a, 0, c, 0, 0) == 0 and f(0, 0, c, 0, 2) == 0 and f(a, b, 0, 0, 1) == 0    # nothing to move
    # buffers a mode does not use are not looked at
    assert f(a, 1, c, 0, A.ASTRA_PROBE_COPY) == 0 and f(3, 5, c, 0, A.ASTRA_PROBE_WRITE1) == 0


def test_pace_variants_validate_like_the_operator(A):
    f = A.astra_ablation_fused_add_rmsnorm
    a, b, c = 1 << 40, 2 << 40, 3 << 40          # never dereferenced
    for v in (A.ASTRA_VARIANT_PACE_NONE, A.ASTRA_VARIANT_PACE_STORE_GAP, A.ASTRA_VARIANT_PACE_X_BEFORE_R, A.ASTRA_VARIANT_PACE_WEIGHT_X_R,
              A.ASTRA_VARIANT_STORE_DEVICE_SCOPE_WHOLE_LINES, A.ASTRA_VARIANT_STORE_DEVICE_SCOPE):   # the store-form variants: the same shapes
        assert f(0, b, c, 1, 8, 1, 1e-6, v) == 1 and f(a, b, c, -1, 8, 1, 1e-6, v) == 2 and f(a, b, c, 1, 8, 7, 1e-6, v) == 3
        assert f(a, b, c, 1, 8, 1, -1.0, v) == 4 and f(a + 1, b, c, 1, 8, 1, 1e-6, v) == 5 and f(a, a, c, 1, 8, 1, 1e-6, v) == 6
        assert f(a, b, c, 0, 8, 1, 1e-6, v) == 0                                          # T == 0: nothing to do
        assert f(a + 2, b, c, 4, 4096, 1, 1e-6, v) == A.ASTRA_ERR_VARIANT                 # ragged path: no row kernel to pace
        assert f(a, b, c, 4, 4100, 1, 1e-6, v) == A.ASTRA_ERR_VARIANT
        assert f(a, b, c, 4, 40000, 1, 1e-6, v) == A.ASTRA_ERR_VARIANT                    # element-wise path
        assert f(a, b, c, 1 << 22, 264, 1, 1e-6, v) == A.ASTRA_ERR_VARIANT                # row loop beyond the grid limit
    assert f(a, b, c, 4, 4096, 1, 1e-6, 12) == A.ASTRA_ERR_VARIANT and f(a, b, c, 4, 4096, 1, 1e-6, -1) == A.ASTRA_ERR_VARIANT
