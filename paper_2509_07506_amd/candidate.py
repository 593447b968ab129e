"""Validate and time ANY shared library that exports the C ABI of ``include/astra.h`` against a test
suite on disk -- the deterministic half of the paper's Validate and Profile steps (arxiv 2509.07506,
Algorithm 1; correctness criterion max_i d(S'(x_i), y_i) <= eps of Section 3.1; 20 warm-up and 100
timed repetitions per shape as in Section 4).  One JSON line per case, shaped like a row of the paper's
Log: round, code, correctness, performance.

    python -m paper_2509_07506_amd.candidate --lib path/to/libcandidate.so --suite SUITE_DIR [--round 0] [--code-id name]

The suite files are written by ``tests/generate_suite.py``; this module never touches the oracle.  The
candidate runs on the GPU; PyTorch only holds the device buffers.
"""
from __future__ import annotations

import argparse
import ctypes
import glob
import json
import math
import os
import sys

import numpy as np

DT_CODE = {"f16": 0, "bf16": 1}


def widen(bits: np.ndarray, dtype: str) -> np.ndarray:
    """16-bit patterns -> float64 (numpy only)."""
    bits = np.ascontiguousarray(bits)
    if dtype == "bf16":
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return bits.view(np.float16).astype(np.float64)


def discrepancy_ok(got, ref, rtol, atol) -> bool:
    """d(got, ref) <= eps in the allclose form; equal infinities match, NaN matches only NaN."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    with np.errstate(invalid="ignore"):
        ok = np.abs(got - ref) <= atol + rtol * np.abs(ref)
    inf = np.isinf(got) | np.isinf(ref)
    ok = np.where(inf, got == ref, ok)
    nan = np.isnan(got) | np.isnan(ref)
    ok = np.where(nan, np.isnan(got) & np.isnan(ref), ok)
    return bool(ok.all())


def compare_case(meta: dict, expected: dict, got: dict) -> dict:
    """Per-output verdicts for one case.  `expected` / `got` map output names to arrays (bit patterns for
    16-bit tensors, float32 for lse)."""
    dt = meta["dtype"]
    out = {}
    if meta["kernel"] == "rmsnorm":
        out["residual_bit_exact"] = bool(np.array_equal(got["residual"], expected["exp_residual"]))
        out["input"] = discrepancy_ok(widen(got["input"], dt), widen(expected["exp_input"], dt), meta["rtol"], meta["atol"])
    elif meta["kernel"] == "silu":
        out["out"] = discrepancy_ok(widen(got["out"], dt), widen(expected["exp_out"], dt), meta["rtol"], meta["atol"])
    else:
        out["v_out"] = discrepancy_ok(widen(got["v_out"], dt), widen(expected["exp_v_out"], dt), meta["rtol"], meta["atol"])
        out["lse_out"] = discrepancy_ok(got["lse_out"], expected["exp_lse_out"], 0.0, meta["lse_atol"])
    return out


def load_candidate(path: str) -> ctypes.CDLL:
    # PyTorch ships its own HIP runtime; it must be in the process before the candidate is loaded so that
    # the candidate binds to the same runtime as the streams and buffers it is handed.
    import torch  # noqa: F401

    L = ctypes.CDLL(os.path.abspath(path))
    vp, i64, i32, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float
    L.astra_fused_add_rmsnorm.argtypes = [vp, vp, vp, i64, i64, i32, f32, vp]
    L.astra_silu_and_mul.argtypes = [vp, vp, i64, i64, i32, vp]
    L.astra_merge_attn_states_lse.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, i32, vp]
    for n in ("astra_fused_add_rmsnorm", "astra_silu_and_mul", "astra_merge_attn_states_lse"):
        getattr(L, n).restype = i32
    return L


def run_case(L, path: str, warmup: int = 20, reps: int = 100) -> dict:
    import torch

    z = np.load(path, allow_pickle=False)
    meta = json.loads(str(z["meta"]))
    dt = meta["dtype"]
    tdt = {"bf16": torch.bfloat16, "f16": torch.float16}[dt]
    code = DT_CODE[dt]
    s = meta["shape"]
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream

    def dev16(a):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(tdt).cuda()

    def bits(t):
        return t.cpu().view(torch.int16).numpy().view(np.uint16)

    if meta["kernel"] == "rmsnorm":
        x0, r0, w = dev16(z["in_input"]), dev16(z["in_residual"]), dev16(z["in_weight"])
        x, r = x0.clone(), r0.clone()
        call = lambda: L.astra_fused_add_rmsnorm(x.data_ptr(), r.data_ptr(), w.data_ptr(), s["T"], s["H"], code, meta["eps"], sh)
        fetch = lambda: {"input": bits(x), "residual": bits(r)}
    elif meta["kernel"] == "silu":
        a = dev16(z["in_input"])
        out = torch.empty((s["T"], s["d"]), dtype=tdt, device="cuda")
        call = lambda: L.astra_silu_and_mul(out.data_ptr(), a.data_ptr(), s["T"], s["d"], code, sh)
        fetch = lambda: {"out": bits(out)}
    else:
        va, vb = dev16(z["in_v_a"]), dev16(z["in_v_b"])
        la, lb = torch.from_numpy(z["in_lse_a"]).cuda(), torch.from_numpy(z["in_lse_b"]).cuda()
        vo, lo = torch.empty_like(va), torch.empty_like(la)
        call = lambda: L.astra_merge_attn_states_lse(vo.data_ptr(), lo.data_ptr(), va.data_ptr(), la.data_ptr(), vb.data_ptr(),
                                                     lb.data_ptr(), s["T"], s["NH"], s["D"], code, sh)
        fetch = lambda: {"v_out": bits(vo), "lse_out": lo.cpu().numpy()}

    status = call()                      # the judged launch: fresh buffers, one call
    torch.cuda.synchronize()
    verdict = compare_case(meta, z, fetch()) if status == 0 else {"status": False}
    correct = status == 0 and all(verdict.values())
    us = None
    if status == 0:
        for _ in range(warmup):
            call()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(stream)
        for _ in range(reps):
            call()
        e1.record(stream)
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
    return {"case": meta["name"], "status": int(status), "checks": verdict, "correctness": bool(correct),
            "performance": None if us is None else {"us": round(us, 3), "GBs": round(meta["algorithmic_bytes"] / us / 1e3, 1)}}


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--lib", required=True)
    ap.add_argument("--suite", required=True)
    ap.add_argument("--round", type=int, default=0)
    ap.add_argument("--code-id", default=None)
    args = ap.parse_args(argv)
    files = sorted(glob.glob(os.path.join(args.suite, "*.npz")))
    if not files:
        print(f"no suite files in {args.suite}", file=sys.stderr)
        return 2
    L = load_candidate(args.lib)
    code_id = args.code_id or os.path.basename(args.lib)
    all_ok, times = True, []
    for f in files:
        row = run_case(L, f)
        all_ok &= row["correctness"]
        if row["performance"]:
            times.append(row["performance"]["us"])
        print(json.dumps({"round": args.round, "code": code_id, **row}), flush=True)
    gm = math.exp(sum(math.log(t) for t in times) / len(times)) if times else None
    print(json.dumps({"round": args.round, "code": code_id, "cases": len(files), "correctness": bool(all_ok),
                      "performance": {"geomean_us": None if gm is None else round(gm, 3)}}), flush=True)
    return 0 if all_ok else 1


if __name__ == "__main__":
    sys.exit(main())
