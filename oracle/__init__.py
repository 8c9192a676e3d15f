"""CPU oracle for the GranQ activation fake-quantizer: numpy front end.

TEST INFRASTRUCTURE ONLY.  The arithmetic lives in ``granq_oracle.c`` (plain
scalar C, written from the paper's Eq. 1, 2, 4, 5, 6 and Alg. 1); this module
only compiles it with gcc, loads it with ctypes and moves numpy arrays in and
out.  Nothing here is shared with, imported by or derived from the HIP library.
Callers: the tests, the smoke check and the benchmark's CPU-baseline leg.

Arrays: ``x`` is a C-contiguous array of shape (N, C, H, W) -- or any shape
(N, C, ...) -- of dtype float32, float16, or uint16 holding bfloat16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "granq_oracle.c")
_LIB = os.path.join(_HERE, "libgranq_oracle.so")

# -O1, every operation rounded on its own: no FMA contraction, no fast-math.
CFLAGS = ["-O1", "-std=c11", "-ffp-contract=off", "-fno-fast-math",
          "-fPIC", "-shared", "-Wall", "-Wextra"]


def build(out: str = _LIB, src: str = _SRC, extra_flags=()) -> str:
    """Compile the oracle with gcc.  Returns the path of the shared object."""
    cmd = ["gcc", *CFLAGS, *extra_flags, "-o", out, src, "-lm"]
    subprocess.run(cmd, check=True)
    return out


def _stale() -> bool:
    return (not os.path.exists(_LIB)
            or os.path.getmtime(_LIB) < os.path.getmtime(_SRC))


_lib = None

_i64 = ctypes.c_int64
_int = ctypes.c_int
_ptr = ctypes.c_void_p


def load(path: str | None = None) -> ctypes.CDLL:
    """Load the oracle library (building it first when missing or stale)."""
    global _lib
    if path is None:
        if _lib is not None:
            return _lib
        if _stale():
            build()
        lib = ctypes.CDLL(_LIB)
    else:
        lib = ctypes.CDLL(path)
    lib.granq_oracle_range_reduce.argtypes = [_ptr, _int, _i64, _i64, _i64, _ptr, _ptr]
    lib.granq_oracle_prescale.argtypes = [_ptr, _ptr, _i64, _int, _ptr, _ptr]
    lib.granq_oracle_fakequant_fwd.argtypes = [_ptr, _int, _i64, _i64, _i64, _ptr, _ptr,
                                               _int, _ptr, _ptr]
    lib.granq_oracle_fakequant_bwd.argtypes = [_ptr, _ptr, _int, _i64, _i64, _i64, _ptr, _ptr,
                                               _int, _ptr]
    lib.granq_oracle_gate_mask.argtypes = [_ptr, _int, _i64, _i64, _i64, _ptr, _ptr, _int, _ptr]
    lib.granq_oracle_bwd_from_mask.argtypes = [_ptr, _ptr, _int, _i64, _ptr]
    lib.granq_oracle_distortion.argtypes = [_ptr, _int, _i64, _i64, _i64, _ptr, _ptr, _int, _ptr, _ptr]
    lib.granq_oracle_fold_weights.argtypes = [_ptr, _ptr, _ptr, _i64, _i64, _ptr, _ptr, _ptr]
    lib.granq_oracle_conv1x1_int8.argtypes = [_ptr, _i64, _i64, _i64, _i64, _ptr, _ptr, _ptr, _ptr]
    lib.granq_oracle_conv1x1_float.argtypes = [_ptr, _int, _i64, _i64, _i64, _i64, _ptr, _ptr]
    lib.granq_oracle_pack4.argtypes = [_ptr, _i64, _ptr]
    lib.granq_oracle_unpack4.argtypes = [_ptr, _i64, _ptr]
    lib.granq_oracle_accumulate_inloop.argtypes = [_ptr, _i64, _i64, _i64, _ptr, _ptr, _ptr, _ptr]
    lib.granq_oracle_accumulate_prescaled.argtypes = [_ptr, _i64, _i64, _i64, _ptr, _ptr]
    lib.granq_oracle_f16_widen.argtypes = [_ptr, _i64, _ptr]
    lib.granq_oracle_f16_narrow.argtypes = [_ptr, _i64, _ptr]
    for name in ("f16_widen", "f16_narrow", "range_reduce", "prescale", "fakequant_fwd", "fakequant_bwd", "gate_mask", "bwd_from_mask", "distortion", "fold_weights", "conv1x1_int8",
                 "accumulate_inloop", "accumulate_prescaled"):
        getattr(lib, "granq_oracle_" + name).restype = None
    if path is None:
        _lib = lib
    return lib


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    if a.dtype == np.float16:
        return 2
    raise TypeError("oracle takes float32, float16, or uint16 holding bfloat16 bits; got %s" % a.dtype)


def _nchw(a: np.ndarray):
    if a.ndim < 2:
        raise ValueError("need at least (N, C) dimensions")
    if not a.flags["C_CONTIGUOUS"]:
        raise ValueError("oracle takes C-contiguous arrays")
    n, c = a.shape[0], a.shape[1]
    hw = 1
    for d in a.shape[2:]:
        hw *= d
    return n, c, hw


def _p(a: np.ndarray):
    return a.ctypes.data_as(_ptr)


def _f32vec(a, c: int) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    if a.shape != (c,):
        raise ValueError("per-channel vector must have shape (%d,)" % c)
    return a


def range_reduce(x: np.ndarray, lib=None):
    """Per-channel (min, max) over batch and space (Eq. 4 with Sec. 5.1's batch level)."""
    lib = lib or load()
    n, c, hw = _nchw(x)
    mn = np.empty(c, np.float32)
    mx = np.empty(c, np.float32)
    lib.granq_oracle_range_reduce(_p(x), _dtype_code(x), n, c, hw, _p(mn), _p(mx))
    return mn, mx


def prescale(ch_min, ch_max, bits: int, lib=None):
    """Per-channel (scale, zero_point) from the ranges (Eq. 5)."""
    lib = lib or load()
    ch_min = np.ascontiguousarray(ch_min, dtype=np.float32)
    c = ch_min.shape[0]
    ch_min = _f32vec(ch_min, c)
    ch_max = _f32vec(ch_max, c)
    s = np.empty(c, np.float32)
    z = np.empty(c, np.float32)
    lib.granq_oracle_prescale(_p(ch_min), _p(ch_max), c, int(bits), _p(s), _p(z))
    return s, z


def fakequant_fwd(x: np.ndarray, scale, zero_point, bits: int, lib=None):
    """Quantize, clamp, dequantize (Eq. 1 and Eq. 6).  Returns (x_hat, codes)."""
    lib = lib or load()
    n, c, hw = _nchw(x)
    s = _f32vec(scale, c)
    z = _f32vec(zero_point, c)
    x_hat = np.empty_like(x)
    codes = np.empty(x.shape, np.uint8)
    lib.granq_oracle_fakequant_fwd(_p(x), _dtype_code(x), n, c, hw, _p(s), _p(z), int(bits),
                                   _p(x_hat), _p(codes))
    return x_hat, codes


def fakequant_bwd(x: np.ndarray, dy: np.ndarray, scale, zero_point, bits: int, lib=None):
    """Straight-through-estimator backward: dy where the clamp was inactive, else 0."""
    lib = lib or load()
    n, c, hw = _nchw(x)
    if dy.shape != x.shape or dy.dtype != x.dtype or not dy.flags["C_CONTIGUOUS"]:
        raise ValueError("dy must match x in shape, dtype and layout")
    s = _f32vec(scale, c)
    z = _f32vec(zero_point, c)
    dx = np.empty_like(x)
    lib.granq_oracle_fakequant_bwd(_p(x), _p(dy), _dtype_code(x), n, c, hw, _p(s), _p(z),
                                   int(bits), _p(dx))
    return dx


def gate_mask(x: np.ndarray, scale, zero_point, bits: int, lib=None) -> np.ndarray:
    """Packed straight-through gate: bit (i & 7) of byte (i >> 3), 1 = clamp inactive."""
    lib = lib or load()
    n, c, hw = _nchw(x)
    s = _f32vec(scale, c)
    z = _f32vec(zero_point, c)
    mask = np.empty((x.size + 7) // 8, np.uint8)
    lib.granq_oracle_gate_mask(_p(x), _dtype_code(x), n, c, hw, _p(s), _p(z), int(bits), _p(mask))
    return mask


def bwd_from_mask(dy: np.ndarray, mask: np.ndarray, lib=None) -> np.ndarray:
    """dx = dy where the gate bit is set, else 0."""
    lib = lib or load()
    if not dy.flags["C_CONTIGUOUS"] or mask.dtype != np.uint8 or mask.size < (dy.size + 7) // 8:
        raise ValueError("dy must be contiguous and mask uint8 with ceil(size / 8) bytes")
    dx = np.empty_like(dy)
    lib.granq_oracle_bwd_from_mask(_p(dy), _p(np.ascontiguousarray(mask)), _dtype_code(dy), dy.size, _p(dx))
    return dx


def distortion(x: np.ndarray, scale, zero_point, bits: int, lib=None):
    """Table 2's figures.  Returns (ch_sums[C,4], layer[6]): per-channel sums x.q, x.x, q.q,
    (x-q).(x-q); layer = those sums over all channels, cosine similarity, relative error."""
    lib = lib or load()
    n, c, hw = _nchw(x)
    s = _f32vec(scale, c)
    z = _f32vec(zero_point, c)
    ch = np.empty((c, 4), np.float64)
    layer = np.empty(6, np.float64)
    lib.granq_oracle_distortion(_p(x), _dtype_code(x), n, c, hw, _p(s), _p(z), int(bits), _p(ch), _p(layer))
    return ch, layer


def fakequant(x: np.ndarray, bits: int, lib=None):
    """The whole forward path on one tensor.  Returns (x_hat, codes, scale, zero_point)."""
    mn, mx = range_reduce(x, lib)
    s, z = prescale(mn, mx, bits, lib)
    x_hat, codes = fakequant_fwd(x, s, z, bits, lib)
    return x_hat, codes, s, z


def fold_weights(w: np.ndarray, scale, zero_point, lib=None):
    """Eq. 3's w_c * s_c folded into int8 rows.  Returns (wq int8[O,C], corr int64[O], out_scale f32[O])."""
    lib = lib or load()
    w = np.ascontiguousarray(w, np.float32)
    o, c = w.shape
    s, z = _f32vec(scale, c), _f32vec(zero_point, c)
    wq = np.empty((o, c), np.int8)
    corr = np.empty(o, np.int64)
    a = np.empty(o, np.float32)
    lib.granq_oracle_fold_weights(_p(w), _p(s), _p(z), o, c, _p(wq), _p(corr), _p(a))
    return wq, corr, a


def conv1x1_int8(codes: np.ndarray, wq: np.ndarray, corr: np.ndarray, out_scale: np.ndarray, lib=None):
    """y[n,o,k] = out_scale[o] * (sum_c wq[o,c] * code[n,c,k] - corr[o])."""
    lib = lib or load()
    n, c, hw = _nchw(codes)
    if codes.dtype != np.uint8 or wq.dtype != np.int8 or wq.shape[1] != c:
        raise TypeError("codes must be uint8 (N,C,...), wq int8 (O,C)")
    o = wq.shape[0]
    wq = np.ascontiguousarray(wq)
    corr = np.ascontiguousarray(corr, np.int64)
    a = np.ascontiguousarray(out_scale, np.float32)
    y = np.empty((n, o) + codes.shape[2:], np.float32)
    lib.granq_oracle_conv1x1_int8(_p(codes), n, c, hw, o, _p(wq), _p(corr), _p(a), _p(y))
    return y


def conv1x1_float(x_hat: np.ndarray, w: np.ndarray, lib=None) -> np.ndarray:
    """1x1 convolution over the pre-scaled activations in floating point (Eq. 6's accumulation):
    y[n,o,...] = sum_c w[o,c] * x_hat[n,c,...], summed in binary64; returns float64.  w (O, C)
    has x_hat's storage type."""
    lib = lib or load()
    n, c, hw = _nchw(x_hat)
    if w.ndim != 2 or w.shape[1] != c or w.dtype != x_hat.dtype or not w.flags["C_CONTIGUOUS"]:
        raise ValueError("w must be a C-contiguous (O, %d) array of x_hat's type" % c)
    o = w.shape[0]
    y = np.empty((n, o) + x_hat.shape[2:], np.float64)
    lib.granq_oracle_conv1x1_float(_p(x_hat), _dtype_code(x_hat), n, c, hw, o, _p(w), _p(y))
    return y


def pack4(codes: np.ndarray, lib=None) -> np.ndarray:
    """Two codes (each below 16) per byte: element 2i in the low nibble of byte i."""
    lib = lib or load()
    codes = np.ascontiguousarray(codes, np.uint8)
    if codes.size and codes.max() > 15:
        raise ValueError("codes of more than four bits cannot be packed two per byte")
    out = np.empty((codes.size + 1) // 2, np.uint8)
    lib.granq_oracle_pack4(_p(codes), codes.size, _p(out))
    return out


def unpack4(packed: np.ndarray, total: int, lib=None) -> np.ndarray:
    lib = lib or load()
    packed = np.ascontiguousarray(packed, np.uint8)
    if packed.size != (total + 1) // 2:
        raise ValueError("packed codes of %d elements take %d bytes" % (total, (total + 1) // 2))
    out = np.empty(total, np.uint8)
    lib.granq_oracle_unpack4(_p(packed), int(total), _p(out))
    return out


def accumulate_inloop(codes: np.ndarray, scale, zero_point, weight, lib=None):
    """Weighted channel sum with the scale applied inside the loop (Eq. 3)."""
    lib = lib or load()
    n, c, hw = _nchw(codes)
    if codes.dtype != np.uint8:
        raise TypeError("codes must be uint8")
    s, z, w = _f32vec(scale, c), _f32vec(zero_point, c), _f32vec(weight, c)
    y = np.empty((n,) + codes.shape[2:], np.float32)
    lib.granq_oracle_accumulate_inloop(_p(codes), n, c, hw, _p(s), _p(z), _p(w), _p(y))
    return y


def accumulate_prescaled(x_hat: np.ndarray, weight, lib=None):
    """Weighted channel sum over pre-scaled activations (Eq. 6 / Alg. 1 output)."""
    lib = lib or load()
    n, c, hw = _nchw(x_hat)
    if x_hat.dtype != np.float32:
        raise TypeError("x_hat must be float32")
    w = _f32vec(weight, c)
    y = np.empty((n,) + x_hat.shape[2:], np.float32)
    lib.granq_oracle_accumulate_prescaled(_p(x_hat), n, c, hw, _p(w), _p(y))
    return y


def f16_widen(h: np.ndarray, lib=None) -> np.ndarray:
    """The oracle's own binary16 -> binary32 conversion on uint16 bit patterns (test hook)."""
    h = np.ascontiguousarray(h, np.uint16)
    out = np.empty(h.shape, np.float32)
    (lib or load()).granq_oracle_f16_widen(_p(h), h.size, _p(out))
    return out


def f16_narrow(f: np.ndarray, lib=None) -> np.ndarray:
    """The oracle's own binary32 -> binary16 conversion, as uint16 bit patterns (test hook)."""
    f = np.ascontiguousarray(f, np.float32)
    out = np.empty(f.shape, np.uint16)
    (lib or load()).granq_oracle_f16_narrow(_p(f), f.size, _p(out))
    return out


def bf16_bits_from_f32(a: np.ndarray) -> np.ndarray:
    """Truncation-free helper for tests: float32 values that are exactly
    bfloat16-representable -> their uint16 bit patterns.  Raises otherwise."""
    bits = np.ascontiguousarray(a, np.float32).view(np.uint32)
    if np.any(bits & 0xFFFF):
        raise ValueError("values are not bfloat16-representable")
    return (bits >> 16).astype(np.uint16)


def f32_from_bf16_bits(h: np.ndarray) -> np.ndarray:
    """uint16 bfloat16 bit patterns -> float32 values (exact)."""
    return (np.ascontiguousarray(h, np.uint16).astype(np.uint32) << 16).view(np.float32)
