"""The C ABI used from a plain C++ host program (tests/c_abi/check_abi.cpp): HIP runtime of the ROCm
installation, hipMalloc'ed buffers, its own stream; no Python or PyTorch in that process.  The program
compares every result with the CPU oracle itself and reports through its exit status."""
import os
import subprocess

import pytest
import torch

from tests import c_abi

pytestmark = pytest.mark.gpu


def test_c_program_passes_all_checks():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    if not os.path.exists(c_abi.BINARY):        # normally built beforehand by __graft_entry__.build()
        print("[c_abi] building check_abi (host code only)", flush=True)
        c_abi.build()
    print(f"[c_abi] running {c_abi.BINARY}", flush=True)
    r = subprocess.run([c_abi.BINARY], capture_output=True, text=True, timeout=120)
    print(r.stdout[-4000:], r.stderr[-2000:], flush=True)
    assert r.returncode == 0, f"check_abi exit status {r.returncode}"
    lines = r.stdout.strip().splitlines()
    assert lines[-1] == "c_abi: all checks passed"
    assert sum(1 for l in lines if l.startswith("c_abi: ok ")) == 36 and not any("FAILED" in l for l in lines)
