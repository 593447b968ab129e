"""The suite generator and the candidate validator (the deterministic halves of the paper's testing and
profiling agents)."""
import json
import os
import subprocess
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def suite_dir(tmp_path_factory):
    from tests import generate_suite

    d = str(tmp_path_factory.mktemp("suite"))
    generate_suite.main([d, "--suite", "small"])
    return d


def test_suite_files_are_complete_and_deterministic(suite_dir, tmp_path):
    from tests import generate_suite

    files = sorted(os.listdir(suite_dir))
    assert len(files) == len(generate_suite.SMALL)
    generate_suite.main([str(tmp_path), "--suite", "small"])
    for f in files:
        a, b = np.load(os.path.join(suite_dir, f)), np.load(os.path.join(tmp_path, f))
        assert sorted(a.files) == sorted(b.files)
        for k in a.files:
            assert np.array_equal(a[k].view(np.uint8) if a[k].dtype.kind != "U" else a[k], b[k].view(np.uint8) if b[k].dtype.kind != "U" else b[k])
        meta = json.loads(str(a["meta"]))
        assert meta["kernel"] in ("rmsnorm", "silu", "merge") and meta["rtol"] > 0


def test_compare_accepts_expected_and_rejects_perturbed(suite_dir):
    from paper_2509_07506_amd import candidate

    for f in sorted(os.listdir(suite_dir)):
        z = np.load(os.path.join(suite_dir, f))
        meta = json.loads(str(z["meta"]))
        if meta["kernel"] == "rmsnorm":
            good = {"input": z["exp_input"], "residual": z["exp_residual"]}
            bad = {"input": z["exp_input"], "residual": z["exp_residual"] ^ np.uint16(1)}       # one ulp off: not bit-exact
            worse = {"input": z["exp_input"] ^ np.uint16(0x0040), "residual": z["exp_residual"]}
            assert not all(candidate.compare_case(meta, z, worse).values())
        elif meta["kernel"] == "silu":
            good = {"out": z["exp_out"]}
            bad = {"out": z["exp_out"] ^ np.uint16(0x0100)}
        else:
            good = {"v_out": z["exp_v_out"], "lse_out": z["exp_lse_out"]}
            lse = z["exp_lse_out"].copy()
            lse[np.isfinite(lse)] += np.float32(1e-3)
            bad = {"v_out": z["exp_v_out"], "lse_out": lse}
        assert all(candidate.compare_case(meta, z, good).values()), f
        assert not all(candidate.compare_case(meta, z, bad).values()), f


@pytest.mark.gpu
def test_own_library_passes_and_a_wrong_expectation_is_caught(suite_dir, tmp_path):
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2509_07506_amd as astra

    cmd = [sys.executable, "-m", "paper_2509_07506_amd.candidate", "--lib", astra.library_path(), "--suite", suite_dir,
           "--round", "3", "--code-id", "tuned"]
    r = subprocess.run(cmd, cwd=ROOT, capture_output=True, text=True)
    rows = [json.loads(l) for l in r.stdout.splitlines() if l.startswith("{")]
    assert r.returncode == 0, r.stdout + r.stderr
    assert len(rows) == len(os.listdir(suite_dir)) + 1 and all(x["correctness"] for x in rows)
    assert all(x["round"] == 3 and x["code"] == "tuned" for x in rows) and rows[-1]["performance"]["geomean_us"] > 0
    # tamper with one expectation: the validator must report that case as incorrect
    bad_dir = tmp_path / "bad"
    bad_dir.mkdir()
    name = sorted(os.listdir(suite_dir))[3]
    z = dict(np.load(os.path.join(suite_dir, name)))
    key = [k for k in z if k.startswith("exp_") and z[k].dtype == np.uint16][0]
    z[key] = z[key] ^ np.uint16(0x0200)
    np.savez(os.path.join(bad_dir, name), **z)
    r = subprocess.run(cmd[:5] + ["--suite", str(bad_dir)], cwd=ROOT, capture_output=True, text=True)
    rows = [json.loads(l) for l in r.stdout.splitlines() if l.startswith("{")]
    assert r.returncode == 1 and rows[0]["correctness"] is False and rows[-1]["correctness"] is False
