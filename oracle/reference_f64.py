"""Float64 statement of the three operators (arxiv 2509.07506, Table 1), numpy only.

TEST INFRASTRUCTURE ONLY.  Outputs are real-valued float64 arrays (no rounding to the storage type),
so a caller compares a 16-bit result against them with a tolerance.  The one place where binary32 is
part of the operator's definition is the residual sum of Kernel 2: the stored residual is the
binary32 sum of the two 16-bit operands rounded once to the storage type, and the normalisation is
taken over that binary32 sum.  Everything else is float64.

Each formula is written exactly as Table 1 prints it, with the max-shift that keeps the exponentials
of Kernel 1 finite.
"""
from __future__ import annotations

import numpy as np


def widen(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Stored values -> float64 (exact): uint16 bit patterns for "f16"/"bf16", float32 arrays for "f32"."""
    bits = np.ascontiguousarray(bits)
    if dtype == "f32":
        assert bits.dtype == np.float32
        return bits.astype(np.float64)
    assert bits.dtype == np.uint16
    if dtype == "bf16":
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if dtype == "f16":
        return bits.view(np.float16).astype(np.float64)
    raise ValueError(dtype)


def fused_add_rmsnorm(x_bits, r_bits, w_bits, eps: float, dtype: str):
    """Kernel 2.  Returns (y, s): y = s / sqrt(mean(s^2) + eps) * w in float64, s = binary32(x + r)."""
    x = widen(x_bits, dtype).astype(np.float32)
    r = widen(r_bits, dtype).astype(np.float32)
    w = widen(w_bits, dtype)
    s = (x + r).astype(np.float64)  # float32 add, then exact widening
    ms = np.mean(s * s, axis=-1, keepdims=True)
    y = s / np.sqrt(ms + np.float64(np.float32(eps))) * w
    return y, s


def silu(z: np.ndarray) -> np.ndarray:
    """SiLU(z) = z / (1 + e^-z); e^-z may overflow to inf for very negative z, giving -0."""
    z = np.asarray(z, np.float64)
    with np.errstate(over="ignore"):
        return z / (1.0 + np.exp(-z))


def silu_and_mul(in_bits, dtype: str) -> np.ndarray:
    """Kernel 3.  in [T, 2d]: first half activated, second half gates.  Returns float64 [T, d]."""
    a = widen(in_bits, dtype)
    d = a.shape[-1] // 2
    return silu(a[..., :d]) * a[..., d:]


def merge_attn_states_lse(va_bits, lse_a, vb_bits, lse_b, dtype: str):
    """Kernel 1.  Returns (v_out float64 [T,NH,D], lse_out float64 [T,NH]).

    Both scores -inf: v_out = 0, lse_out = -inf.  A side whose weight is exactly zero (an empty partition) is left
    out of the blend whatever its values are.
    """
    va = widen(va_bits, dtype)
    vb = widen(vb_bits, dtype)
    sa = np.asarray(lse_a, np.float64)
    sb = np.asarray(lse_b, np.float64)
    m = np.maximum(sa, sb)
    empty = np.isneginf(m)
    m0 = np.where(empty, 0.0, m)
    ea = np.exp(sa - m0)
    eb = np.exp(sb - m0)
    den = ea + eb
    with np.errstate(divide="ignore", invalid="ignore"):
        a = np.where(empty, 0.0, ea / den)
        b = np.where(empty, 0.0, eb / den)
        s_out = np.where(empty, -np.inf, m0 + np.log(den))
    # a term whose weight is exactly zero is left out: its values are not looked at
    ta = a[..., None] * np.where(a[..., None] == 0.0, 0.0, va)
    tb = b[..., None] * np.where(b[..., None] == 0.0, 0.0, vb)
    return ta + tb, s_out


def merge_attn_states_lse_kway(v_parts_bits, lse_parts, dtype: str):
    """K-way merge in float64: softmax over the K scores weights the K partial outputs; S_out is their
    logsumexp.  v_parts [K,T,NH,D] uint16, lse_parts [K,T,NH].  All scores -inf: 0 and -inf."""
    v = widen(v_parts_bits, dtype)
    s = np.asarray(lse_parts, np.float64)
    m = np.max(s, axis=0)
    empty = np.isneginf(m)
    m0 = np.where(empty, 0.0, m)
    e = np.exp(s - m0)
    den = e.sum(axis=0)
    with np.errstate(divide="ignore", invalid="ignore"):
        a = np.where(empty, 0.0, e / den)
        s_out = np.where(empty, -np.inf, m0 + np.log(den))
    live = (a != 0.0)[..., None]  # zero-weight parts are left out, their values not looked at
    return (a[..., None] * np.where(live, v, 0.0)).sum(axis=0), s_out
