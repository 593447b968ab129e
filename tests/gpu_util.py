"""Host <-> device plumbing for the GPU parity tests (no operator arithmetic)."""
import numpy as np
import torch

from oracle import reference_f64
from tests.util import LSE_ATOL, TOL, assert_bits_equal, close_mask

TORCH_DT = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}
CANARY32 = 0x7BCD7BCD  # a finite binary32 pattern


def to_dev(bits: np.ndarray, dt: str) -> torch.Tensor:
    """Stored values (uint16 bit patterns, or float32 for "f32") -> GPU tensor of the storage type (bit-preserving)."""
    if dt == "f32":
        return torch.from_numpy(np.ascontiguousarray(bits, np.float32)).cuda()
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(TORCH_DT[dt]).cuda()


def to_bits(t: torch.Tensor) -> np.ndarray:
    """GPU tensor -> what to_dev took: uint16 bit patterns, or the float32 values of a float32 tensor."""
    if t.dtype == torch.float32:
        return t.detach().cpu().contiguous().numpy()
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def padded(bits: np.ndarray, dt: str, pad: int = 64, offset_elems: int = 0, canary: int = 0x7BCD):
    """Uploads `bits` into the middle of a larger canary-filled buffer.  Returns (view, whole).
    `offset_elems` shifts the view by that many elements to break 16-byte alignment."""
    n = bits.size
    if dt == "f32":
        whole = torch.full((pad + offset_elems + n + pad,), CANARY32, dtype=torch.int32).view(torch.float32).cuda()
        view = whole[pad + offset_elems: pad + offset_elems + n].view(bits.shape)
        view.copy_(torch.from_numpy(np.ascontiguousarray(bits, np.float32)))
        return view, whole
    whole = torch.full((pad + offset_elems + n + pad,), canary, dtype=torch.int16).view(TORCH_DT[dt]).cuda()
    view = whole[pad + offset_elems: pad + offset_elems + n].view(bits.shape)
    view.copy_(torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(TORCH_DT[dt]).view(bits.shape))
    return view, whole


def canaries_intact(whole: torch.Tensor, n: int, pad: int = 64, offset_elems: int = 0, canary: int = 0x7BCD) -> bool:
    if whole.dtype == torch.float32:
        w = whole.view(torch.int32).cpu().numpy().view(np.uint32)
        canary = CANARY32
    else:
        w = whole.view(torch.int16).cpu().numpy().view(np.uint16)
    lo = w[: pad + offset_elems]
    hi = w[pad + offset_elems + n:]
    return bool(np.all(lo == canary) and np.all(hi == canary))


def assert_storage_close(got_bits, ref_bits, dt, what, chunk=1 << 24):
    """Tolerance comparison of two stored tensors (uint16 bit patterns, or float32 arrays for "f32").  Elements
    with identical bits are equal by definition; only the differing ones are widened (numpy, float64) and compared."""
    rtol, atol = TOL[dt]
    g = np.asarray(got_bits).reshape(-1)
    r = np.asarray(ref_bits).reshape(-1)
    assert g.shape == r.shape and g.dtype == r.dtype, (what, g.shape, r.shape, g.dtype, r.dtype)
    nbad = 0
    ndiff = 0
    first = None
    for lo in range(0, g.size, chunk):
        gi, ri = g[lo:lo + chunk], r[lo:lo + chunk]
        idx = np.nonzero(gi != ri)[0]
        if idx.size == 0:
            continue
        ndiff += idx.size
        gv = reference_f64.widen(gi[idx], dt)
        rv = reference_f64.widen(ri[idx], dt)
        ok = close_mask(gv, rv, rtol, atol)
        # +0 and -0 compare equal; NaN only equals NaN (close_mask)
        if not ok.all():
            nbad += int((~ok).sum())
            if first is None:
                k = idx[np.nonzero(~ok)[0][0]]
                first = (lo + int(k), float(gv[np.nonzero(~ok)[0][0]]), float(rv[np.nonzero(~ok)[0][0]]))
    assert nbad == 0, f"{what}: {nbad} of {g.size} elements out of tolerance (rtol={rtol}, atol={atol}); first {first}"
    return ndiff


def assert_storage_close_to_real(got_bits, ref_real, dt, what):
    """16-bit result against a real-valued (float64) reference."""
    rtol, atol = TOL[dt]
    gv = reference_f64.widen(np.asarray(got_bits), dt)
    # a real value at or beyond (largest finite + half an ulp) of the storage type is stored as +-inf
    limit = {"f16": 65520.0, "bf16": float.fromhex("0x1.ffp127"), "f32": float.fromhex("0x1.ffffffp127")}[dt]
    ref_real = np.asarray(ref_real, np.float64)
    ref_real = np.where(np.abs(ref_real) >= limit, np.copysign(np.inf, ref_real), ref_real)
    ok = close_mask(gv, ref_real, rtol, atol)
    if not ok.all():
        bad = np.argwhere(~ok)
        i = tuple(bad[0])
        raise AssertionError(f"{what}: {len(bad)} of {ok.size} out of tolerance vs float64; first at {i}: "
                             f"got {gv[i]!r}, ref {np.asarray(ref_real)[i]!r}")


def assert_lse_close(got, ref, what):
    ok = close_mask(got, ref, 0.0, LSE_ATOL)
    if not ok.all():
        bad = np.argwhere(~ok)
        i = tuple(bad[0])
        raise AssertionError(f"{what}: {len(bad)} of {ok.size} lse values differ by more than {LSE_ATOL}; first at {i}: "
                             f"got {np.asarray(got)[i]!r}, ref {np.asarray(ref)[i]!r}")
