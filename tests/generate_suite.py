#!/usr/bin/env python3
"""Writes a test suite T = {(x_i, y_i)} to disk: seeded inputs of diverse shapes and values, and the
expected outputs y_i := S(x_i) with S the CPU oracle (the deterministic half of the paper's testing
agent, Algorithm 1 line 1 and Section 3.1).  A candidate library is later judged against these files by
``python -m paper_2509_07506_amd.candidate`` without needing the oracle.

    python tests/generate_suite.py OUT_DIR [--suite small|paper|bench]

One ``<case>.npz`` per case holds the inputs and expected outputs as raw bit patterns plus a JSON ``meta``
string (kernel, dtype, shape, eps, tolerances).  This script is test infrastructure: it is the only
part of the candidate workflow that calls the oracle.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import oracle  # noqa: E402
import workloads  # noqa: E402
from tests.util import LSE_ATOL, TOL  # noqa: E402

SMALL = [
    workloads.Case("s_rmsnorm_T5_H4096_bf16", "rmsnorm", 6, 0, "bf16", {"T": 5, "H": 4096}, eps=1e-6),
    workloads.Case("s_rmsnorm_T33_H5120_f16", "rmsnorm", 6, 1, "f16", {"T": 33, "H": 5120}, eps=1e-5, r_std=2.0),
    workloads.Case("s_rmsnorm_T3_H4100_f16", "rmsnorm", 6, 2, "f16", {"T": 3, "H": 4100}, eps=1e-5),
    workloads.Case("s_silu_T7_d1408_bf16", "silu", 6, 3, "bf16", {"T": 7, "d": 1408}),
    workloads.Case("s_silu_T3_d100_f16", "silu", 6, 4, "f16", {"T": 3, "d": 100}),
    workloads.Case("s_merge_T9_NH8_D128_bf16", "merge", 6, 5, "bf16", {"T": 9, "NH": 8, "D": 128}),
    workloads.Case("s_merge_T4_NH40_D64_f16", "merge", 6, 6, "f16", {"T": 4, "NH": 40, "D": 64}),
]


def suite_cases(which: str):
    if which == "small":
        return SMALL
    if which == "paper":
        return [workloads.PAPER_SHAPE_CASES[n] for n in sorted(workloads.PAPER_SHAPE_CASES)]
    if which == "bench":
        return [workloads.CASES[n] for n in sorted(workloads.CASES) if workloads.CASES[n].algorithmic_bytes() < (600 << 20)]
    raise ValueError(which)


def write_case(c: workloads.Case, out_dir: str) -> str:
    data = c.generate()
    rtol, atol = TOL[c.dtype]
    meta = {"name": c.name, "kernel": c.kernel, "dtype": c.dtype, "shape": c.shape, "eps": c.eps, "rtol": rtol, "atol": atol,
            "lse_atol": LSE_ATOL, "residual": "bit-exact", "algorithmic_bytes": c.algorithmic_bytes()}
    arrays = {}
    if c.kernel == "rmsnorm":
        x, r, w = data
        y, res = oracle.fused_add_rmsnorm(x, r, w, c.eps, c.dtype)
        arrays = {"in_input": x, "in_residual": r, "in_weight": w, "exp_input": y, "exp_residual": res}
    elif c.kernel == "silu":
        (a,) = data
        arrays = {"in_input": a, "exp_out": oracle.silu_and_mul(a, c.dtype)}
    else:
        va, la, vb, lb = data
        vo, lo = oracle.merge_attn_states_lse(va, la, vb, lb, c.dtype)
        arrays = {"in_v_a": va, "in_lse_a": la, "in_v_b": vb, "in_lse_b": lb, "exp_v_out": vo, "exp_lse_out": lo}
    path = os.path.join(out_dir, c.name + ".npz")
    np.savez(path, meta=np.array(json.dumps(meta)), **arrays)
    return path


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("out_dir")
    ap.add_argument("--suite", default="small", choices=("small", "paper", "bench"))
    args = ap.parse_args(argv)
    os.makedirs(args.out_dir, exist_ok=True)
    oracle.build()
    for c in suite_cases(args.suite):
        print(write_case(c, args.out_dir), flush=True)


if __name__ == "__main__":
    main()
