"""Host-side contract of bench.py that can be checked without a GPU: one-GPU-only, no silent fallback,
and the committed traffic figures it reports are consistent with the algorithmic byte counts."""
import json
import os
import subprocess
import sys

import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def _run(args, env=None):
    e = dict(os.environ)
    e.update(env or {})
    return subprocess.run([sys.executable, BENCH, *args], capture_output=True, text=True, env=e, cwd=ROOT, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run(["--gpus", "2"])
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
    r = _run([], env={"WORLD_SIZE": "4"})
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_step_workloads_are_the_bandwidth_configs():
    sys.path.insert(0, ROOT)
    import bench

    cases = [workloads.case(n) for n in bench.STEP_CASES]
    assert [c.kernel for c in cases] == ["rmsnorm", "silu", "merge"] and all(c.dtype == "bf16" for c in cases)
    assert cases[0].shape == {"T": 32768, "H": 8192} and cases[1].shape == {"T": 4096, "d": 14336}
    assert cases[2].shape == {"T": 4096, "NH": 32, "D": 128}
    # per-token figures of the measurement plan: 65 536 / 86 016 / 24 960 bytes
    assert cases[0].algorithmic_bytes() == 65536 * 32768 + 8192 * 2
    assert cases[1].algorithmic_bytes() == 86016 * 4096 and cases[2].algorithmic_bytes() == 24960 * 4096
    assert bench.HBM_PEAK_GBS == 8000.0


def test_committed_traffic_matches_algorithmic_bytes():
    with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
        traffic = json.load(f)
    sys.path.insert(0, ROOT)
    import bench

    assert set(traffic) == set(bench.STEP_CASES)
    for name, t in traffic.items():
        c = workloads.case(name)
        assert t["algorithmic_bytes"] == c.algorithmic_bytes()
        assert t["total_bytes"] == t["read_bytes"] + t["write_bytes"]
        assert abs(t["total_bytes"] / c.algorithmic_bytes() - 1.0) < 0.01      # one pass, no re-reads
        assert os.path.exists(os.path.join(ROOT, t["source"]))


def test_committed_traffic_was_counted_on_the_geometry_the_library_plans_now():
    """The counter figures bench.py reports are a committed file; they name the kernel instantiation and the launch
    geometry they were collected on.  When a kernel or policy change makes the library plan something else for the
    benchmark workloads, the figures are stale: bench.py then reports traffic null, and this test fails until the
    counters are collected again."""
    import paper_2509_07506_amd as astra

    with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
        traffic = json.load(f)
    sys.path.insert(0, ROOT)
    import bench

    for name, t in traffic.items():
        c = workloads.case(name)
        s = c.shape
        if c.kernel == "rmsnorm":
            st, info = astra.astra_plan_fused_add_rmsnorm(s["T"], s["H"], True)
        elif c.kernel == "silu":
            st, info = astra.astra_plan_silu_and_mul(s["T"], s["d"], True)
        else:
            st, info = astra.astra_plan_merge_attn_states_lse(s["T"], s["NH"], s["D"], True)
        assert st == 0
        assert t["launch"] == info.as_dict(), f"{name}: counters were collected on {t['launch']}, the library plans {info.as_dict()}"
        assert bench.KERNEL_NAMES[c.kernel] in t["kernel"]
        got, why = bench.traffic_for(traffic, name, info.as_dict())
        assert got is t and why is None
        stale, why = bench.traffic_for(traffic, name, dict(info.as_dict(), block=info.block * 2))
        assert stale is None and "stale" in why


def test_median():
    sys.path.insert(0, ROOT)
    import bench

    assert bench._median([3.0, 1.0, 2.0]) == 2.0 and bench._median([4.0, 1.0, 2.0, 3.0]) == 2.5
