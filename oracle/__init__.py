"""CPU oracle for the three Astra serving operators (arxiv 2509.07506, Table 1).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this; only ``tests/``, the smoke
check and the benchmark's CPU-baseline leg do.  Two independent statements of each operator live here:

* ``astra_oracle.c``  -- plain scalar C in binary32, bit-defined outputs in the 16-bit storage type
  (loaded through ``ctypes`` by the functions below);
* ``reference_f64.py`` -- the same definitions in numpy float64 with real-valued (unrounded) outputs.

All arrays are host numpy arrays.  16-bit tensors travel as ``uint16`` bit patterns; ``dtype`` is
``"f16"`` or ``"bf16"``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "astra_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
# Test hook: tests/test_oracle_mutations.py points this at a deliberately broken build to show that the
# pins catch it.  When set, that library is loaded as is and nothing is compiled.
_OVERRIDE = os.environ.get("ASTRA_ORACLE_LIB")

DTYPES = {"f16": 0, "bf16": 1}

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc.  No FMA contraction, no fast-math."""
    if _OVERRIDE:
        return _OVERRIDE
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        i64, f32, i32 = ctypes.c_int64, ctypes.c_float, ctypes.c_int
        vp = ctypes.c_void_p
        L.oracle_widen_array.argtypes = [vp, vp, i64, i32]
        L.oracle_narrow_array.argtypes = [vp, vp, i64, i32]
        L.oracle_set_threads.argtypes = [i32]
        L.oracle_get_threads.restype = i32
        L.oracle_fused_add_rmsnorm_f32.argtypes = [vp, vp, vp, i64, i64, f32, vp, vp]
        L.oracle_fused_add_rmsnorm.argtypes = [vp, vp, vp, i64, i64, i32, f32]
        L.oracle_silu_f32.argtypes = [f32]
        L.oracle_silu_f32.restype = f32
        L.oracle_silu_and_mul.argtypes = [vp, vp, i64, i64, i32]
        L.oracle_silu_and_mul_f32.argtypes = [vp, vp, i64, i64]
        L.oracle_merge_weights_f32.argtypes = [f32, f32, vp, vp, vp]
        L.oracle_merge_attn_states_lse.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, i32]
        L.oracle_merge_attn_states_lse_f32.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64]
        L.oracle_merge_attn_states_lse_kway.argtypes = [vp, vp, vp, vp, i64, i64, i64, i32]
        L.oracle_merge_attn_states_lse_kway.restype = None
        L.oracle_merge_attn_states_lse_kway_f32.argtypes = [vp, vp, vp, vp, i64, i64, i64]
        L.oracle_merge_attn_states_lse_kway_f32.restype = None
        for name in ("oracle_widen_array", "oracle_narrow_array", "oracle_set_threads", "oracle_fused_add_rmsnorm_f32",
                     "oracle_fused_add_rmsnorm", "oracle_silu_and_mul", "oracle_silu_and_mul_f32",
                     "oracle_merge_weights_f32", "oracle_merge_attn_states_lse", "oracle_merge_attn_states_lse_f32"):
            getattr(L, name).restype = None
        _lib = L
    return _lib


def _ptr(a: np.ndarray) -> int:
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float32, a.dtype
    return a


def set_threads(n: int) -> int:
    """Number of OpenMP threads for the row loops; returns the number actually in use."""
    lib().oracle_set_threads(int(n))
    return int(lib().oracle_get_threads())


# ------------------------------------------------------------------------------------------------
# conversions

def widen(bits, dtype: str) -> np.ndarray:
    """16-bit patterns -> float32 (exact)."""
    bits = _u16(bits)
    out = np.empty(bits.shape, np.float32)
    lib().oracle_widen_array(_ptr(bits), _ptr(out), bits.size, DTYPES[dtype])
    return out


def narrow(x, dtype: str) -> np.ndarray:
    """float32 -> 16-bit patterns, round to nearest even."""
    x = _f32(x)
    out = np.empty(x.shape, np.uint16)
    lib().oracle_narrow_array(_ptr(x), _ptr(out), x.size, DTYPES[dtype])
    return out


# ------------------------------------------------------------------------------------------------
# Kernel 2

def fused_add_rmsnorm(x_bits, r_bits, w_bits, eps: float, dtype: str):
    """Returns (input_after, residual_after) as uint16 [T,H]; the arguments are not modified."""
    x = _u16(x_bits).copy()
    r = _u16(r_bits).copy()
    w = _u16(w_bits)
    T, H = x.shape
    assert r.shape == (T, H) and w.shape == (H,)
    lib().oracle_fused_add_rmsnorm(_ptr(x), _ptr(r), _ptr(w), T, H, DTYPES[dtype], float(eps))
    return x, r


def fused_add_rmsnorm_f32(x, r, w, eps: float):
    """All-float32 form: returns (s, y) with s = x + r."""
    x, r, w = _f32(x), _f32(r), _f32(w)
    T, H = x.shape
    s = np.empty((T, H), np.float32)
    y = np.empty((T, H), np.float32)
    lib().oracle_fused_add_rmsnorm_f32(_ptr(x), _ptr(r), _ptr(w), T, H, float(eps), _ptr(s), _ptr(y))
    return s, y


# ------------------------------------------------------------------------------------------------
# Kernel 3

def silu_f32(z: float) -> float:
    return float(lib().oracle_silu_f32(float(z)))


def silu_and_mul(in_bits, dtype: str) -> np.ndarray:
    """in [T, 2d] uint16 -> out [T, d] uint16; first half of a row is activated, second half gates."""
    a = _u16(in_bits)
    T, two_d = a.shape
    assert two_d % 2 == 0
    d = two_d // 2
    out = np.empty((T, d), np.uint16)
    lib().oracle_silu_and_mul(_ptr(out), _ptr(a), T, d, DTYPES[dtype])
    return out


def silu_and_mul_f32(a) -> np.ndarray:
    a = _f32(a)
    T, two_d = a.shape
    d = two_d // 2
    out = np.empty((T, d), np.float32)
    lib().oracle_silu_and_mul_f32(_ptr(out), _ptr(a), T, d)
    return out


# ------------------------------------------------------------------------------------------------
# Kernel 1

def merge_weights_f32(sa: float, sb: float):
    """(a, b, s_out) for one pair of scores, float32 arithmetic."""
    a = ctypes.c_float()
    b = ctypes.c_float()
    s = ctypes.c_float()
    lib().oracle_merge_weights_f32(float(sa), float(sb), ctypes.addressof(a), ctypes.addressof(b),
                                   ctypes.addressof(s))
    return a.value, b.value, s.value


def merge_attn_states_lse(va_bits, lse_a, vb_bits, lse_b, dtype: str):
    """v_* [T,NH,D] uint16, lse_* [T,NH] float32 -> (v_out uint16, lse_out float32)."""
    va, vb = _u16(va_bits), _u16(vb_bits)
    la, lb = _f32(lse_a), _f32(lse_b)
    T, NH, D = va.shape
    assert vb.shape == (T, NH, D) and la.shape == (T, NH) and lb.shape == (T, NH)
    vo = np.empty((T, NH, D), np.uint16)
    lo = np.empty((T, NH), np.float32)
    lib().oracle_merge_attn_states_lse(_ptr(vo), _ptr(lo), _ptr(va), _ptr(la), _ptr(vb), _ptr(lb), T, NH, D,
                                       DTYPES[dtype])
    return vo, lo


def merge_attn_states_lse_f32(va, lse_a, vb, lse_b):
    va, vb, la, lb = _f32(va), _f32(vb), _f32(lse_a), _f32(lse_b)
    T, NH, D = va.shape
    vo = np.empty((T, NH, D), np.float32)
    lo = np.empty((T, NH), np.float32)
    lib().oracle_merge_attn_states_lse_f32(_ptr(vo), _ptr(lo), _ptr(va), _ptr(la), _ptr(vb), _ptr(lb), T, NH, D)
    return vo, lo


def merge_attn_states_lse_kway(v_parts_bits, lse_parts, dtype: str):
    """K-way merge.  v_parts [K,T,NH,D] uint16, lse_parts [K,T,NH] float32 -> (v_out [T,NH,D], lse_out [T,NH])."""
    v, l = _u16(v_parts_bits), _f32(lse_parts)
    K, T, NH, D = v.shape
    assert l.shape == (K, T, NH)
    vo = np.empty((T, NH, D), np.uint16)
    lo = np.empty((T, NH), np.float32)
    lib().oracle_merge_attn_states_lse_kway(_ptr(vo), _ptr(lo), _ptr(v), _ptr(l), K, T * NH, D, DTYPES[dtype])
    return vo, lo


def merge_attn_states_lse_kway_f32(v_parts, lse_parts):
    """All-float32 K-way merge.  v_parts [K,T,NH,D] float32, lse_parts [K,T,NH] float32 -> (v_out, lse_out) float32."""
    v, l = _f32(v_parts), _f32(lse_parts)
    K, T, NH, D = v.shape
    assert l.shape == (K, T, NH)
    vo = np.empty((T, NH, D), np.float32)
    lo = np.empty((T, NH), np.float32)
    lib().oracle_merge_attn_states_lse_kway_f32(_ptr(vo), _ptr(lo), _ptr(v), _ptr(l), K, T * NH, D)
    return vo, lo
