"""Builds the stand-alone C++ check of the C ABI (check_abi.cpp): a host program that links the HIP library and
the CPU oracle directly, without Python or PyTorch in the process."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
SOURCE = os.path.join(HERE, "check_abi.cpp")
BINARY = os.path.join(HERE, "check_abi")


def build() -> str:
    """Compiles check_abi.cpp with hipcc (host code only) against the two libraries, building them first if absent."""
    import oracle
    from paper_2509_07506_amd import build as hip_build

    oracle.build()
    if not os.path.exists(hip_build.LIB):
        hip_build.build()
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-O2", "-std=c++17", "-Wall", "-Wextra", "-I", os.path.join(ROOT, "include"), SOURCE, "-o", BINARY,
           "-L", os.path.join(ROOT, "paper_2509_07506_amd"), "-lastra_hip", "-L", os.path.join(ROOT, "oracle"), "-loracle",
           # found relative to the binary, wherever the tree is checked out
           "-Wl,-rpath,$ORIGIN/../../paper_2509_07506_amd", "-Wl,-rpath,$ORIGIN/../../oracle"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("building check_abi failed:\n" + r.stdout + r.stderr)
    return BINARY
