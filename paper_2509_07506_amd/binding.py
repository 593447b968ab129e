"""ctypes binding of ``libastra_hip.so`` (declared in ``include/astra.h`` and ``include/astra_plan.h``).

Two layers, both argument marshalling only:

* ``astra_*`` -- the C entry points themselves: integer device addresses, sizes, dtype code, stream
  handle in, status code out.
* ``fused_add_rmsnorm`` / ``silu_and_mul`` / ``merge_attn_states_lse`` / ``stream_copy`` -- take torch
  tensors living on the GPU, check dtype / contiguity / shapes, pass ``data_ptr()`` and torch's current
  stream, and raise :class:`AstraError` on a non-zero status.

PyTorch is used for device memory and streams only.
"""
from __future__ import annotations

import ctypes
import os

ASTRA_F16 = 0
ASTRA_BF16 = 1
ASTRA_F32 = 2

# include/astra_ablation.h
ASTRA_VARIANT_TUNED = 0
ASTRA_VARIANT_SCALAR_LOADS = 1
ASTRA_VARIANT_LDS_TREE_REDUCTION = 2
ASTRA_VARIANT_UNHOISTED_WEIGHTS = 3
ASTRA_VARIANT_LIBM_EXP_DIVIDE = 4
ASTRA_VARIANT_ELEMENT_WISE = 5
ASTRA_VARIANT_PACE_NONE = 6
ASTRA_VARIANT_PACE_STORE_GAP = 7
ASTRA_VARIANT_PACE_X_BEFORE_R = 8
ASTRA_VARIANT_PACE_WEIGHT_X_R = 9
ASTRA_VARIANT_STORE_DEVICE_SCOPE_WHOLE_LINES = 10
ASTRA_VARIANT_STORE_DEVICE_SCOPE = 11
ASTRA_ERR_VARIANT = 8

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libastra_hip.so")
_lib = None


class AstraError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        super().__init__(f"{where}: status {int(status)} ({astra_status_string(status)})")


class LaunchInfo(ctypes.Structure):
    _fields_ = [("path", ctypes.c_int32), ("block", ctypes.c_int32), ("vectors_per_lane", ctypes.c_int32),
                ("log2_xcd_chunk", ctypes.c_int32), ("grid", ctypes.c_int64), ("pace", ctypes.c_int32),
                ("rows_per_block", ctypes.c_int32), ("access_bytes", ctypes.c_int32), ("non_temporal", ctypes.c_int32)]

    def as_dict(self):
        return {"path": {0: "none", 1: "vector", 2: "generic", 3: "ragged", 4: "phased"}[self.path], "block": self.block,
                "vectors_per_lane": self.vectors_per_lane, "log2_xcd_chunk": self.log2_xcd_chunk, "grid": self.grid,
                "pace": self.pace, **({"rows_per_block": self.rows_per_block} if self.rows_per_block else {}),
                **({"access_bytes": self.access_bytes} if self.access_bytes not in (0, 16) else {}),
                **({"non_temporal": 0} if self.path in (1, 3, 4) and not self.non_temporal else {})}


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Loads the built library.  Builds it first when none is built, or when the built one does not come from the
    sources as they are now (so that tests and benchmarks never check or time an outdated binary)."""
    global _lib
    if _lib is not None:
        return _lib
    from . import build as _build

    if _build.is_stale():
        try:
            _build.build()
        except Exception as e:  # no silent fallback: the product path needs the HIP library
            raise RuntimeError(f"astra HIP library is missing or older than its sources and building it failed: {e}") from e
    # PyTorch ships its own HIP runtime; load it first so that this library binds to the same runtime as
    # the streams and device buffers it is handed (two HIP runtimes in one process do not share streams).
    import torch  # noqa: F401

    L = ctypes.CDLL(_LIB_PATH)
    vp, i64, i32, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float
    L.astra_fused_add_rmsnorm.argtypes = [vp, vp, vp, i64, i64, i32, f32, vp]
    L.astra_silu_and_mul.argtypes = [vp, vp, i64, i64, i32, vp]
    L.astra_merge_attn_states_lse.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, i32, vp]
    L.astra_stream_copy.argtypes = [vp, vp, i64, vp]
    L.astra_stream_probe.argtypes = [vp, vp, vp, i64, i32, vp]
    L.astra_stream_probe.restype = i32
    L.astra_fused_add_rmsnorm_strided.argtypes = [vp, i64, vp, i64, vp, i64, vp, i64, vp, i64, i64, i32, f32, vp]
    L.astra_fused_add_rmsnorm_strided.restype = i32
    L.astra_silu_and_mul_strided.argtypes = [vp, i64, vp, i64, i64, i64, i32, vp]
    L.astra_silu_and_mul_strided.restype = i32
    L.astra_merge_attn_states_lse_strided.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, vp, i64, i64, vp, i64, i64, i64, i32, vp]
    L.astra_merge_attn_states_lse_strided.restype = i32
    L.astra_merge_attn_states_lse_kway.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i32, vp]
    L.astra_merge_attn_states_lse_kway.restype = i32
    L.astra_ablation_fused_add_rmsnorm.argtypes = [vp, vp, vp, i64, i64, i32, f32, i32, vp]
    L.astra_ablation_silu_and_mul.argtypes = [vp, vp, i64, i64, i32, i32, vp]
    L.astra_ablation_merge_attn_states_lse.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, i32, i32, vp]
    L.astra_status_string.argtypes = [i32]
    L.astra_status_string.restype = ctypes.c_char_p
    pinfo = ctypes.POINTER(LaunchInfo)
    L.astra_plan_fused_add_rmsnorm.argtypes = [i64, i64, i32, i32, pinfo]
    L.astra_plan_silu_and_mul.argtypes = [i64, i64, i32, i32, pinfo]
    L.astra_plan_merge_attn_states_lse.argtypes = [i64, i64, i64, i32, i32, pinfo]
    L.astra_device_memory_info.argtypes = [i32, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
    L.astra_device_memory_info.restype = i32
    L.astra_plan_xcd_chunked.argtypes = [ctypes.c_uint32, i32]
    L.astra_plan_xcd_chunked.restype = ctypes.c_uint32
    for n in ("astra_fused_add_rmsnorm", "astra_silu_and_mul", "astra_merge_attn_states_lse", "astra_stream_copy",
              "astra_ablation_fused_add_rmsnorm", "astra_ablation_silu_and_mul", "astra_ablation_merge_attn_states_lse",
              "astra_plan_fused_add_rmsnorm", "astra_plan_silu_and_mul", "astra_plan_merge_attn_states_lse"):
        getattr(L, n).restype = i32
    _lib = L
    return L


# ---------------------------------------------------------------------------------------------------
# the C entry points, one to one

def astra_status_string(status: int) -> str:
    return load_library().astra_status_string(int(status)).decode()


def astra_fused_add_rmsnorm(input_ptr, residual_ptr, weight_ptr, T, H, dtype, eps, stream=None) -> int:
    return load_library().astra_fused_add_rmsnorm(input_ptr, residual_ptr, weight_ptr, T, H, dtype, eps, stream)


def astra_silu_and_mul(out_ptr, input_ptr, T, d, dtype, stream=None) -> int:
    return load_library().astra_silu_and_mul(out_ptr, input_ptr, T, d, dtype, stream)


def astra_merge_attn_states_lse(v_out, lse_out, v_a, lse_a, v_b, lse_b, T, num_heads, head_dim, dtype,
                                stream=None) -> int:
    return load_library().astra_merge_attn_states_lse(v_out, lse_out, v_a, lse_a, v_b, lse_b, T, num_heads, head_dim,
                                                      dtype, stream)


def astra_stream_copy(dst, src, nbytes, stream=None) -> int:
    return load_library().astra_stream_copy(dst, src, nbytes, stream)


ASTRA_PROBE_COPY, ASTRA_PROBE_READ2, ASTRA_PROBE_WRITE1, ASTRA_PROBE_READ2_WRITE1, ASTRA_PROBE_UPDATE2 = range(5)


def astra_stream_probe(a, b, c, nbytes, mode, stream=None) -> int:
    return load_library().astra_stream_probe(a, b, c, nbytes, mode, stream)


def astra_fused_add_rmsnorm_strided(y_out, y_stride, r_out, r_out_stride, x, x_stride, r, r_stride, weight, T, H, dtype, eps,
                                    stream=None) -> int:
    return load_library().astra_fused_add_rmsnorm_strided(y_out, y_stride, r_out, r_out_stride, x, x_stride, r, r_stride,
                                                          weight, T, H, dtype, eps, stream)


def astra_silu_and_mul_strided(out, out_stride, input_ptr, in_stride, T, d, dtype, stream=None) -> int:
    return load_library().astra_silu_and_mul_strided(out, out_stride, input_ptr, in_stride, T, d, dtype, stream)


def astra_merge_attn_states_lse_strided(v_out, out_ts, out_hs, lse_out, v_a, a_ts, a_hs, lse_a, v_b, b_ts, b_hs, lse_b, T,
                                        num_heads, head_dim, dtype, stream=None) -> int:
    return load_library().astra_merge_attn_states_lse_strided(v_out, out_ts, out_hs, lse_out, v_a, a_ts, a_hs, lse_a, v_b,
                                                              b_ts, b_hs, lse_b, T, num_heads, head_dim, dtype, stream)


def astra_merge_attn_states_lse_kway(v_out, lse_out, v_parts, lse_parts, K, T, num_heads, head_dim, dtype, stream=None) -> int:
    return load_library().astra_merge_attn_states_lse_kway(v_out, lse_out, v_parts, lse_parts, K, T, num_heads, head_dim,
                                                           dtype, stream)


def astra_ablation_fused_add_rmsnorm(input_ptr, residual_ptr, weight_ptr, T, H, dtype, eps, variant, stream=None) -> int:
    return load_library().astra_ablation_fused_add_rmsnorm(input_ptr, residual_ptr, weight_ptr, T, H, dtype, eps, variant,
                                                           stream)


def astra_ablation_silu_and_mul(out_ptr, input_ptr, T, d, dtype, variant, stream=None) -> int:
    return load_library().astra_ablation_silu_and_mul(out_ptr, input_ptr, T, d, dtype, variant, stream)


def astra_ablation_merge_attn_states_lse(v_out, lse_out, v_a, lse_a, v_b, lse_b, T, num_heads, head_dim, dtype, variant,
                                         stream=None) -> int:
    return load_library().astra_ablation_merge_attn_states_lse(v_out, lse_out, v_a, lse_a, v_b, lse_b, T, num_heads,
                                                               head_dim, dtype, variant, stream)


def _plan(fn, *args):
    info = LaunchInfo()
    st = fn(*args, ctypes.byref(info))
    return st, info


def astra_plan_fused_add_rmsnorm(T, H, aligned16=True, dtype=ASTRA_BF16):
    return _plan(load_library().astra_plan_fused_add_rmsnorm, T, H, dtype, int(aligned16))


def astra_plan_silu_and_mul(T, d, aligned16=True, dtype=ASTRA_BF16):
    return _plan(load_library().astra_plan_silu_and_mul, T, d, dtype, int(aligned16))


def astra_plan_merge_attn_states_lse(T, num_heads, head_dim, aligned16=True, dtype=ASTRA_BF16):
    return _plan(load_library().astra_plan_merge_attn_states_lse, T, num_heads, head_dim, dtype, int(aligned16))


def astra_device_memory_info(device: int = 0):
    """(status, memory clock in kHz, bus width in bits) as the HIP runtime reports them."""
    clk, width = ctypes.c_int(0), ctypes.c_int(0)
    st = load_library().astra_device_memory_info(int(device), ctypes.byref(clk), ctypes.byref(width))
    return st, clk.value, width.value


def astra_plan_xcd_chunked(workgroup: int, log2_chunk: int) -> int:
    return int(load_library().astra_plan_xcd_chunked(workgroup, log2_chunk))


# ---------------------------------------------------------------------------------------------------
# torch-tensor convenience layer (marshalling only)

def _dtype_code(t) -> int:
    import torch

    if t.dtype == torch.bfloat16:
        return ASTRA_BF16
    if t.dtype == torch.float16:
        return ASTRA_F16
    if t.dtype == torch.float32:
        return ASTRA_F32
    raise TypeError(f"astra operators take float16, bfloat16 or float32 tensors, got {t.dtype}")


def _check_gpu(*tensors):
    for t in tensors:
        if not t.is_cuda:
            raise ValueError("astra operators run on GPU tensors only (there is no CPU path)")
        if not t.is_contiguous():
            raise ValueError("astra operators take dense row-major tensors")


def _stream(stream):
    import torch

    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def fused_add_rmsnorm(input, residual, weight, eps: float, stream=None) -> None:
    """In place: residual <- input + residual, input <- rmsnorm(input + residual) * weight."""
    _check_gpu(input, residual, weight)
    T, H = input.shape
    if residual.shape != (T, H) or weight.shape != (H,) or residual.dtype != input.dtype or weight.dtype != input.dtype:
        raise ValueError("fused_add_rmsnorm: input/residual [T,H] and weight [H] of one dtype expected")
    if T == 0:
        return  # an empty torch tensor has a null data_ptr(), which the C entry point rejects
    st = astra_fused_add_rmsnorm(input.data_ptr(), residual.data_ptr(), weight.data_ptr(), T, H, _dtype_code(input),
                                 float(eps), _stream(stream))
    if st:
        raise AstraError(st, "astra_fused_add_rmsnorm")


def silu_and_mul(out, input, stream=None) -> None:
    """out[T,d] <- silu(input[:, :d]) * input[:, d:]."""
    _check_gpu(out, input)
    T, two_d = input.shape
    if two_d % 2 or out.shape != (T, two_d // 2) or out.dtype != input.dtype:
        raise ValueError("silu_and_mul: input [T,2d] and out [T,d] of one dtype expected")
    if T == 0:
        return
    st = astra_silu_and_mul(out.data_ptr(), input.data_ptr(), T, two_d // 2, _dtype_code(input), _stream(stream))
    if st:
        raise AstraError(st, "astra_silu_and_mul")


def merge_attn_states_lse(v_out, lse_out, v_a, lse_a, v_b, lse_b, stream=None) -> None:
    """(v_out, lse_out) <- merge of the partial attention states (v_a, lse_a) and (v_b, lse_b)."""
    import torch

    _check_gpu(v_out, lse_out, v_a, lse_a, v_b, lse_b)
    T, NH, D = v_a.shape
    if v_b.shape != (T, NH, D) or v_out.shape != (T, NH, D) or v_b.dtype != v_a.dtype or v_out.dtype != v_a.dtype:
        raise ValueError("merge_attn_states_lse: v tensors [T,NH,D] of one dtype expected")
    for s in (lse_a, lse_b, lse_out):
        if s.shape != (T, NH) or s.dtype != torch.float32:
            raise ValueError("merge_attn_states_lse: lse tensors [T,NH] float32 expected")
    if T == 0:
        return
    st = astra_merge_attn_states_lse(v_out.data_ptr(), lse_out.data_ptr(), v_a.data_ptr(), lse_a.data_ptr(),
                                     v_b.data_ptr(), lse_b.data_ptr(), T, NH, D, _dtype_code(v_a), _stream(stream))
    if st:
        raise AstraError(st, "astra_merge_attn_states_lse")


def merge_attn_states_lse_kway(v_out, lse_out, v_parts, lse_parts, stream=None) -> None:
    """(v_out, lse_out) <- merge of the K stacked partial states v_parts [K,T,NH,D], lse_parts [K,T,NH]."""
    import torch

    _check_gpu(v_out, lse_out, v_parts, lse_parts)
    K, T, NH, D = v_parts.shape
    if v_out.shape != (T, NH, D) or v_out.dtype != v_parts.dtype or lse_parts.shape != (K, T, NH) or \
            lse_out.shape != (T, NH) or lse_parts.dtype != torch.float32 or lse_out.dtype != torch.float32:
        raise ValueError("merge_attn_states_lse_kway: v_parts [K,T,NH,D], lse_parts [K,T,NH] f32, v_out [T,NH,D], lse_out [T,NH] f32")
    if T == 0:
        return
    st = astra_merge_attn_states_lse_kway(v_out.data_ptr(), lse_out.data_ptr(), v_parts.data_ptr(), lse_parts.data_ptr(), K,
                                          T, NH, D, _dtype_code(v_parts), _stream(stream))
    if st:
        raise AstraError(st, "astra_merge_attn_states_lse_kway")


def fused_add_rmsnorm_strided(y_out, r_out, x, r, weight, eps: float, stream=None) -> None:
    """y_out <- rmsnorm(x + r) * weight, r_out <- x + r, for 2-D tensors whose rows are dense but may be strided views."""
    for t in (y_out, r_out, x, r, weight):
        if not t.is_cuda:
            raise ValueError("astra operators run on GPU tensors only (there is no CPU path)")
    T, H = x.shape
    for t in (y_out, r_out, x, r):
        if t.shape != (T, H) or t.dtype != x.dtype or (H > 1 and t.stride(1) != 1):
            raise ValueError("fused_add_rmsnorm_strided: [T,H] tensors of one dtype with unit column stride expected")
    if weight.shape != (H,) or weight.dtype != x.dtype or not weight.is_contiguous():
        raise ValueError("fused_add_rmsnorm_strided: weight [H], dense")
    if T == 0:
        return
    rs = lambda t: t.stride(0) if T > 1 else H
    st = astra_fused_add_rmsnorm_strided(y_out.data_ptr(), rs(y_out), r_out.data_ptr(), rs(r_out), x.data_ptr(), rs(x),
                                         r.data_ptr(), rs(r), weight.data_ptr(), T, H, _dtype_code(x), float(eps),
                                         _stream(stream))
    if st:
        raise AstraError(st, "astra_fused_add_rmsnorm_strided")


def silu_and_mul_strided(out, input, stream=None) -> None:
    """out[T,d] <- silu(input[:, :d]) * input[:, d:] for 2-D tensors whose rows are dense but may be strided views."""
    for t in (out, input):
        if not t.is_cuda:
            raise ValueError("astra operators run on GPU tensors only (there is no CPU path)")
    T, two_d = input.shape
    d = two_d // 2
    if two_d % 2 or out.shape != (T, d) or out.dtype != input.dtype or (two_d > 1 and input.stride(1) != 1) or \
            (d > 1 and out.stride(1) != 1):
        raise ValueError("silu_and_mul_strided: input [T,2d] and out [T,d] of one dtype with unit column stride expected")
    if T == 0:
        return
    st = astra_silu_and_mul_strided(out.data_ptr(), out.stride(0) if T > 1 else d, input.data_ptr(),
                                    input.stride(0) if T > 1 else two_d, T, d, _dtype_code(input), _stream(stream))
    if st:
        raise AstraError(st, "astra_silu_and_mul_strided")


def merge_attn_states_lse_strided(v_out, lse_out, v_a, lse_a, v_b, lse_b, stream=None) -> None:
    """Merge for value tensors [T,NH,D] that are strided views (dense along D); scores dense [T,NH] float32."""
    import torch

    for t in (v_out, lse_out, v_a, lse_a, v_b, lse_b):
        if not t.is_cuda:
            raise ValueError("astra operators run on GPU tensors only (there is no CPU path)")
    T, NH, D = v_a.shape
    for t in (v_out, v_a, v_b):
        if t.shape != (T, NH, D) or t.dtype != v_a.dtype or (D > 1 and t.stride(2) != 1):
            raise ValueError("merge_attn_states_lse_strided: v tensors [T,NH,D] of one dtype, dense along D, expected")
    for s in (lse_a, lse_b, lse_out):
        if s.shape != (T, NH) or s.dtype != torch.float32 or not s.is_contiguous():
            raise ValueError("merge_attn_states_lse_strided: lse tensors [T,NH] float32, dense, expected")
    if T == 0:
        return
    hs = lambda t: t.stride(1) if NH > 1 else D
    ts = lambda t: t.stride(0) if T > 1 else (NH - 1) * hs(t) + D
    st = astra_merge_attn_states_lse_strided(v_out.data_ptr(), ts(v_out), hs(v_out), lse_out.data_ptr(), v_a.data_ptr(),
                                             ts(v_a), hs(v_a), lse_a.data_ptr(), v_b.data_ptr(), ts(v_b), hs(v_b),
                                             lse_b.data_ptr(), T, NH, D, _dtype_code(v_a), _stream(stream))
    if st:
        raise AstraError(st, "astra_merge_attn_states_lse_strided")


def stream_copy(dst, src, stream=None) -> None:
    _check_gpu(dst, src)
    n = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != n:
        raise ValueError("stream_copy: sizes differ")
    st = astra_stream_copy(dst.data_ptr(), src.data_ptr(), n, _stream(stream))
    if st:
        raise AstraError(st, "astra_stream_copy")
