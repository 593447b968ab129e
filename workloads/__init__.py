"""Seeded synthetic inputs for the three serving operators, shaped like LLM-serving layers.

This module serves both the tests/benchmark of the HIP library and the CPU oracle.  It holds none of
the operators' arithmetic: it only draws random numbers (numpy ``Generator(PCG64)``) and rounds them
to the 16-bit storage type with the library casts of numpy (fp16) and torch (bf16), both
round-to-nearest-even.  16-bit tensors are returned as ``uint16`` bit patterns, scores as ``float32``.
Storage type ``"f32"`` (a boundary convenience, no benchmark config uses it) returns the ``float32``
draws themselves.

Distribution readings (where a benchmark config says N(mu, v), v is the variance):
  fused_add_rmsnorm  x ~ N(0,1); r ~ N(0,1) or N(0,4) (sigma 2); w ~ N(1, 0.1) (sigma sqrt(0.1))
  silu_and_mul       N(0,1) over the whole [T, 2d] input, an independent 0.1 % of entries times 20
  merge              v_a, v_b ~ N(0,1); lse_a, lse_b ~ U[-5, 15) with an independent 1 % of each set to -inf
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

_CHUNK = 1 << 24  # elements drawn per call; fixed, so a case's stream does not depend on host memory


def _rng(config: int, case: int, seed: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, config, case])))


ELEM_BYTES = {"f16": 2, "bf16": 2, "f32": 4}


def to_bits(x: np.ndarray, dtype: str) -> np.ndarray:
    """float32 array -> uint16 bit patterns of `dtype` via a library cast (RNE); "f32" returns the array itself."""
    x = np.ascontiguousarray(x, np.float32)
    if dtype == "f32":
        return x
    if dtype == "f16":
        return x.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        import torch

        return torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    raise ValueError(dtype)


def _normal_bits(rng, n: int, dtype: str, mean: float = 0.0, std: float = 1.0, outlier_p: float = 0.0,
                 outlier_scale: float = 1.0) -> np.ndarray:
    out = np.empty(n, np.float32 if dtype == "f32" else np.uint16)
    for lo in range(0, n, _CHUNK):
        m = min(_CHUNK, n - lo)
        z = rng.standard_normal(m, dtype=np.float32)
        if outlier_p > 0.0:
            mask = rng.random(m, dtype=np.float32) < np.float32(outlier_p)
            z[mask] *= np.float32(outlier_scale)
        if std != 1.0:
            z *= np.float32(std)
        if mean != 0.0:
            z += np.float32(mean)
        out[lo:lo + m] = to_bits(z, dtype)
    return out


def rmsnorm_inputs(T: int, H: int, dtype: str, rng, r_std: float = 1.0):
    """(x [T,H], r [T,H], w [H]) as uint16 bit patterns."""
    x = _normal_bits(rng, T * H, dtype).reshape(T, H)
    r = _normal_bits(rng, T * H, dtype, std=r_std).reshape(T, H)
    w = _normal_bits(rng, H, dtype, mean=1.0, std=float(np.sqrt(0.1)))
    return x, r, w


def silu_inputs(T: int, d: int, dtype: str, rng):
    """input [T, 2d] as uint16 bit patterns: N(0,1), 0.1 % of entries scaled by 20."""
    return _normal_bits(rng, T * 2 * d, dtype, outlier_p=1e-3, outlier_scale=20.0).reshape(T, 2 * d)


def merge_inputs(T: int, NH: int, D: int, dtype: str, rng, empty_p: float = 0.01):
    """(v_a [T,NH,D] u16, lse_a [T,NH] f32, v_b, lse_b)."""
    va = _normal_bits(rng, T * NH * D, dtype).reshape(T, NH, D)
    vb = _normal_bits(rng, T * NH * D, dtype).reshape(T, NH, D)
    lse = []
    for _ in range(2):
        s = rng.uniform(-5.0, 15.0, size=(T, NH)).astype(np.float32)
        s[rng.random((T, NH)) < empty_p] = -np.inf
        lse.append(s)
    return va, lse[0], vb, lse[1]


@dataclass(frozen=True)
class Case:
    """One synthetic workload.  `config` is the index into the benchmark's config list."""
    name: str
    kernel: str  # "rmsnorm" | "silu" | "merge"
    config: int
    case: int
    dtype: str
    shape: dict = field(default_factory=dict)
    eps: float = 0.0
    r_std: float = 1.0

    def rng(self):
        return _rng(self.config, self.case)

    def generate(self):
        g = self.rng()
        s = self.shape
        if self.kernel == "rmsnorm":
            return rmsnorm_inputs(s["T"], s["H"], self.dtype, g, r_std=self.r_std)
        if self.kernel == "silu":
            return (silu_inputs(s["T"], s["d"], self.dtype, g),)
        if self.kernel == "merge":
            return merge_inputs(s["T"], s["NH"], s["D"], self.dtype, g)
        raise ValueError(self.kernel)

    def algorithmic_bytes(self) -> int:
        """Bytes the operator itself must move in one pass (elements of the storage type, float32 scores)."""
        s = self.shape
        e = ELEM_BYTES[self.dtype]
        if self.kernel == "rmsnorm":
            return 4 * s["T"] * s["H"] * e + s["H"] * e
        if self.kernel == "silu":
            return 3 * s["T"] * s["d"] * e
        return 3 * s["T"] * s["NH"] * s["D"] * e + 3 * s["T"] * s["NH"] * 4

    def tokens(self) -> int:
        return self.shape["T"]


def _cases():
    out = []
    # config 0: decode-sized rmsnorm
    out.append(Case("c0_rmsnorm_T16_H4096_bf16", "rmsnorm", 0, 0, "bf16", {"T": 16, "H": 4096}, eps=1e-6))
    # config 1: SwiGLU gate at a 70B-class intermediate size
    out.append(Case("c1_silu_T4096_d14336_bf16", "silu", 1, 0, "bf16", {"T": 4096, "d": 14336}))
    # config 2: merge of two partial attention states
    out.append(Case("c2_merge_T4096_NH32_D128_bf16", "merge", 2, 0, "bf16", {"T": 4096, "NH": 32, "D": 128}))
    # config 3: rmsnorm sweep, H = 8192
    k = 0
    for T in (1, 8, 64, 512, 8192, 32768):
        for dt in ("bf16", "f16"):
            out.append(Case(f"c3_rmsnorm_T{T}_H8192_{dt}", "rmsnorm", 3, k, dt, {"T": T, "H": 8192}, eps=1e-5,
                            r_std=2.0))
            k += 1
    # config 4: odd shapes, fp16
    k = 0
    for T in (1, 3, 257, 4099):
        for H in (5120, 7168):
            out.append(Case(f"c4_rmsnorm_T{T}_H{H}_f16", "rmsnorm", 4, k, "f16", {"T": T, "H": H}, eps=1e-5,
                            r_std=2.0))
            k += 1
        for d in (11008, 1408):
            out.append(Case(f"c4_silu_T{T}_d{d}_f16", "silu", 4, k, "f16", {"T": T, "d": d}))
            k += 1
        for D in (64, 256):
            out.append(Case(f"c4_merge_T{T}_NH40_D{D}_f16", "merge", 4, k, "f16", {"T": T, "NH": 40, "D": D}))
            k += 1
    return out


def _paper_shape_cases():
    """The twelve shapes of the paper's Table 4 (Section 6.1): [seq_len, heads, head_dim] for the merge,
    [batch, hidden] for the other two (for silu_and_mul `hidden` is read as the output width d).  fp16,
    the only storage type the paper's listings show; value recipes as in the benchmark configs."""
    out = []
    k = 0
    for T, NH, D in ((512, 32, 256), (512, 40, 128), (768, 32, 256), (512, 64, 128)):
        out.append(Case(f"p4_merge_T{T}_NH{NH}_D{D}_f16", "merge", 5, k, "f16", {"T": T, "NH": NH, "D": D}))
        k += 1
    for T, H in ((256, 4096), (1024, 4096), (128, 11008), (512, 14336)):
        out.append(Case(f"p4_rmsnorm_T{T}_H{H}_f16", "rmsnorm", 5, k, "f16", {"T": T, "H": H}, eps=1e-6))
        k += 1
    for T, d in ((16, 4096), (32, 5120), (64, 8192), (16, 12288)):
        out.append(Case(f"p4_silu_T{T}_d{d}_f16", "silu", 5, k, "f16", {"T": T, "d": d}))
        k += 1
    return out


def _f32_cases():
    """Bandwidth-regime shapes with binary32 storage (not benchmark configs: they exist to measure the
    boundary's convenience storage type); value recipes as in the 16-bit configs of the same operator."""
    return [
        Case("f32_rmsnorm_T16384_H8192", "rmsnorm", 6, 0, "f32", {"T": 16384, "H": 8192}, eps=1e-5, r_std=2.0),
        Case("f32_rmsnorm_T32768_H4096", "rmsnorm", 6, 1, "f32", {"T": 32768, "H": 4096}, eps=1e-5, r_std=2.0),
        Case("f32_silu_T4096_d14336", "silu", 6, 2, "f32", {"T": 4096, "d": 14336}),
        Case("f32_merge_T4096_NH32_D128", "merge", 6, 3, "f32", {"T": 4096, "NH": 32, "D": 128}),
    ]


def _prefill_cases():
    """Prefill-chunk shapes (some hundreds to a few thousand tokens) at the dimensions of the models the paper names
    for its shape selection (Section 6.1: LLaMA-7B, 13B and 70B): hidden 4096 / 5120 / 8192, intermediate 11008 /
    13824 / 28672, 32 / 40 / 64 heads of 128.  Not benchmark configs: they exist to measure the grids of one to a
    few rounds of resident workgroups; value recipes as in the benchmark configs of the same operator."""
    out = []
    k = 0
    for H in (4096, 5120, 8192):
        for T in (512, 1024, 2048, 4096):
            out.append(Case(f"pf_rmsnorm_T{T}_H{H}_bf16", "rmsnorm", 7, k, "bf16", {"T": T, "H": H}, eps=1e-5, r_std=2.0))
            k += 1
    for d in (11008, 13824, 28672):
        for T in (512, 2048):
            out.append(Case(f"pf_silu_T{T}_d{d}_bf16", "silu", 7, k, "bf16", {"T": T, "d": d}))
            k += 1
    for NH in (32, 40, 64):
        for T in (512, 2048):
            out.append(Case(f"pf_merge_T{T}_NH{NH}_D128_bf16", "merge", 7, k, "bf16", {"T": T, "NH": NH, "D": 128}))
            k += 1
    return out


CASES = {c.name: c for c in _cases()}
PAPER_SHAPE_CASES = {c.name: c for c in _paper_shape_cases()}
F32_CASES = {c.name: c for c in _f32_cases()}
PREFILL_CASES = {c.name: c for c in _prefill_cases()}


def case(name: str) -> Case:
    for table in (CASES, PAPER_SHAPE_CASES, F32_CASES, PREFILL_CASES):
        if name in table:
            return table[name]
    raise KeyError(name)
