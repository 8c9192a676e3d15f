"""ctypes binding of the GranQ C ABI (include/granq.h).

Argument marshalling only: every function here turns torch tensors into device
pointers plus a descriptor, calls the entry point of the same name in
``libgranq.so`` and raises on a non-zero status.  No arithmetic of the method is
done in Python and there is no CPU fallback: without the built library, or with
tensors that are not on a GPU, the calls fail.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

from . import build as _build

GRANQ_OK = 0
GRANQ_ERR_INVALID_ARG = 1
GRANQ_ERR_UNSUPPORTED = 2
GRANQ_ERR_WORKSPACE = 3
GRANQ_ERR_HIP = 4

GRANQ_F32 = 0
GRANQ_BF16 = 1
GRANQ_F16 = 2

EXPORTS = ("granq_status_string", "granq_version", "granq_workspace_bytes", "granq_plan_describe",
           "granq_range_reduce", "granq_range_reduce_noalloc",
           "granq_prescale", "granq_calibrate", "granq_calibrate_fakequant_fwd", "granq_resident_state_bytes", "granq_resident_state_init",
           "granq_calibrate_fakequant_fwd_resident", "granq_fakequant_fwd", "granq_fakequant_bwd", "granq_mask_bytes",
           "granq_fakequant_fwd_mask", "granq_fakequant_bwd_mask", "granq_rowwise_fakequant_multi",
           "granq_rowwise_fakequant_bwd_multi", "granq_distortion_workspace_bytes", "granq_distortion",
           "granq_fold_weights", "granq_conv1x1_int8", "granq_conv1x1_int8_as", "granq_packed4_bytes",
           "granq_fakequant_fwd_packed4", "granq_conv1x1_int8_packed4", "granq_conv1x1_float")
COMPARE_EXPORTS = ("granq_cmp_channel_loop_fwd", "granq_cmp_accumulate_inloop",
                   "granq_cmp_accumulate_prescaled")


class granq_desc_t(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int64), ("c", ctypes.c_int64), ("h", ctypes.c_int64),
                ("w", ctypes.c_int64), ("dtype", ctypes.c_int)]


class granq_rowq_item_t(ctypes.Structure):
    _fields_ = [("w", ctypes.c_void_p), ("w_hat", ctypes.c_void_p), ("scale", ctypes.c_void_p),
                ("zero_point", ctypes.c_void_p), ("rows", ctypes.c_int64), ("row_len", ctypes.c_int64)]


class granq_rowq_bwd_item_t(ctypes.Structure):
    _fields_ = [("w", ctypes.c_void_p), ("dy", ctypes.c_void_p), ("dw", ctypes.c_void_p),
                ("scale", ctypes.c_void_p), ("zero_point", ctypes.c_void_p),
                ("rows", ctypes.c_int64), ("row_len", ctypes.c_int64)]


class GranqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s" % (where, status_string(status)))


_lib: Optional[ctypes.CDLL] = None
_vp = ctypes.c_void_p


def library_path() -> str:
    return _build.LIB


def load(path: Optional[str] = None) -> ctypes.CDLL:
    """Load libgranq.so (building it with hipcc first if it has never been built)."""
    global _lib
    if path is None and _lib is not None:
        return _lib
    p = path or _build.LIB
    if path is None and not os.path.exists(p):
        _build.build()
    lib = ctypes.CDLL(p)
    dp = ctypes.POINTER(granq_desc_t)
    lib.granq_status_string.argtypes = [ctypes.c_int]
    lib.granq_status_string.restype = ctypes.c_char_p
    lib.granq_version.argtypes = []
    lib.granq_version.restype = ctypes.c_char_p
    lib.granq_workspace_bytes.argtypes = [dp, ctypes.POINTER(ctypes.c_size_t)]
    lib.granq_plan_describe.argtypes = [dp, ctypes.POINTER(ctypes.c_int64 * 24)]
    lib.granq_range_reduce.argtypes = [_vp, dp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
    lib.granq_range_reduce_noalloc.argtypes = [_vp, dp, _vp, _vp, _vp]
    lib.granq_prescale.argtypes = [_vp, _vp, ctypes.c_int64, ctypes.c_int, _vp, _vp, _vp]
    lib.granq_calibrate.argtypes = [_vp, dp, ctypes.c_int, _vp, _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
    lib.granq_calibrate_fakequant_fwd.argtypes = [_vp, dp, ctypes.c_int, _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                                                  ctypes.c_size_t, _vp]
    lib.granq_resident_state_bytes.argtypes = [dp, ctypes.POINTER(ctypes.c_size_t)]
    lib.granq_resident_state_init.argtypes = [_vp, ctypes.c_size_t, _vp]
    lib.granq_calibrate_fakequant_fwd_resident.argtypes = [_vp, dp, ctypes.c_int, _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                                                           ctypes.c_size_t, _vp]
    lib.granq_fakequant_fwd.argtypes = [_vp, dp, _vp, _vp, ctypes.c_int, _vp, _vp, _vp]
    lib.granq_fakequant_bwd.argtypes = [_vp, _vp, dp, _vp, _vp, ctypes.c_int, _vp, _vp]
    lib.granq_mask_bytes.argtypes = [dp, ctypes.POINTER(ctypes.c_size_t)]
    lib.granq_fakequant_fwd_mask.argtypes = [_vp, dp, _vp, _vp, ctypes.c_int, _vp, _vp, _vp]
    lib.granq_fakequant_bwd_mask.argtypes = [_vp, _vp, dp, _vp, _vp]
    lib.granq_rowwise_fakequant_multi.argtypes = [_vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, _vp]
    lib.granq_rowwise_fakequant_bwd_multi.argtypes = [_vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, _vp]
    lib.granq_fold_weights.argtypes = [_vp, _vp, _vp, ctypes.c_int64, ctypes.c_int64, _vp, _vp, _vp, _vp]
    lib.granq_conv1x1_int8.argtypes = [_vp, dp, ctypes.c_int64, _vp, _vp, _vp, ctypes.c_int, _vp, _vp]
    lib.granq_conv1x1_int8_as.argtypes = [_vp, dp, ctypes.c_int64, _vp, _vp, _vp, ctypes.c_int, ctypes.c_int, _vp, _vp]
    lib.granq_packed4_bytes.argtypes = [dp, ctypes.POINTER(ctypes.c_size_t)]
    lib.granq_fakequant_fwd_packed4.argtypes = [_vp, dp, _vp, _vp, ctypes.c_int, _vp, _vp, _vp]
    lib.granq_conv1x1_int8_packed4.argtypes = [_vp, dp, ctypes.c_int64, _vp, _vp, _vp, ctypes.c_int, ctypes.c_int, _vp, _vp]
    lib.granq_conv1x1_float.argtypes = [_vp, dp, ctypes.c_int64, _vp, _vp, _vp]
    lib.granq_distortion_workspace_bytes.argtypes = [dp, ctypes.POINTER(ctypes.c_size_t)]
    lib.granq_distortion.argtypes = [_vp, dp, _vp, _vp, ctypes.c_int, _vp, _vp, _vp, ctypes.c_size_t, _vp]
    lib.granq_cmp_channel_loop_fwd.argtypes = [_vp, dp, ctypes.c_int, _vp, _vp, _vp, _vp, _vp, _vp,
                                               ctypes.c_size_t, _vp]
    lib.granq_cmp_accumulate_inloop.argtypes = [_vp, dp, _vp, _vp, _vp, _vp, _vp]
    lib.granq_cmp_accumulate_prescaled.argtypes = [_vp, dp, _vp, _vp, _vp]
    for name in EXPORTS[2:] + COMPARE_EXPORTS:
        getattr(lib, name).restype = ctypes.c_int
    if path is None:
        _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().granq_status_string(int(status)).decode()


def version() -> str:
    return load().granq_version().decode()


def _check(status: int, where: str) -> None:
    if status != GRANQ_OK:
        raise GranqError(status, where)


def dtype_code(dtype: torch.dtype) -> int:
    """granq_dtype_t of a torch dtype."""
    try:
        return {torch.float32: GRANQ_F32, torch.bfloat16: GRANQ_BF16, torch.float16: GRANQ_F16}[dtype]
    except KeyError:
        raise TypeError("GranQ takes float32, bfloat16 or float16 tensors, got %s" % dtype) from None


def _dtype_code(t: torch.Tensor) -> int:
    return dtype_code(t.dtype)


def make_desc(n: int, c: int, h: int, w: int, dtype: int) -> granq_desc_t:
    return granq_desc_t(int(n), int(c), int(h), int(w), int(dtype))


def desc_of(x: torch.Tensor) -> granq_desc_t:
    """Descriptor of a contiguous (N, C, ...) tensor; trailing dims fold into H*W."""
    if x.dim() < 2:
        raise ValueError("need an (N, C, ...) tensor")
    if not x.is_contiguous():
        raise ValueError("GranQ takes dense contiguous NCHW tensors")
    hw = 1
    for d in x.shape[2:]:
        hw *= int(d)
    h = int(x.shape[2]) if x.dim() > 2 else 1
    return make_desc(x.shape[0], x.shape[1], h, hw // h if h else 0, _dtype_code(x))


def _desc_for(x: torch.Tensor, desc: Optional[granq_desc_t], name: str = "x", typed: bool = True) -> granq_desc_t:
    """The caller's descriptor, checked against the tensor it describes, or the tensor's own.

    The C ABI cannot know how large a buffer is: a descriptor naming more elements, or a wider
    element type, than the tensor holds would make the kernels run past the allocation."""
    if desc is None:
        return desc_of(x)
    want = int(desc.n) * int(desc.c) * int(desc.h) * int(desc.w)
    if min(int(desc.n), int(desc.c), int(desc.h), int(desc.w)) <= 0 or x.numel() != want:
        raise ValueError("desc {%d,%d,%d,%d} names %d elements, %s holds %d"
                         % (desc.n, desc.c, desc.h, desc.w, want, name, x.numel()))
    if typed and dtype_code(x.dtype) != int(desc.dtype):
        raise ValueError("desc.dtype is %d, %s is %s" % (desc.dtype, name, x.dtype))
    return desc


def _dev(t: torch.Tensor, name: str) -> int:
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU (the library takes device pointers)" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    return t.data_ptr()


def _vec(t: torch.Tensor, c: int, name: str) -> int:
    if t.dtype != torch.float32 or t.numel() != c:
        raise ValueError("%s must be float32 with %d entries" % (name, c))
    return _dev(t, name)


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def granq_workspace_bytes(desc: granq_desc_t) -> int:
    out = ctypes.c_size_t(0)
    _check(load().granq_workspace_bytes(ctypes.byref(desc), ctypes.byref(out)), "granq_workspace_bytes")
    return int(out.value)


def granq_plan_describe(desc: granq_desc_t) -> dict:
    out = (ctypes.c_int64 * 24)()
    _check(load().granq_plan_describe(ctypes.byref(desc), ctypes.byref(out)), "granq_plan_describe")
    keys = ("vector_path", "rows", "row_len", "hw", "span", "col_tiles", "row_groups",
            "rows_per_group", "kmax", "uniform", "div_m", "div_s1", "div_s2", "fwd_rows", "bwd_rows",
            "elem_span", "fold", "one_call_launches", "range_launches")
    return dict(zip(keys, [int(v) for v in out]))


def granq_range_reduce(x: torch.Tensor, ch_min: torch.Tensor, ch_max: torch.Tensor,
                       workspace: torch.Tensor, stream=None, desc: Optional[granq_desc_t] = None) -> None:
    d = _desc_for(x, desc)
    _check(load().granq_range_reduce(_dev(x, "x"), ctypes.byref(d), _vec(ch_min, d.c, "ch_min"),
                                     _vec(ch_max, d.c, "ch_max"), _dev(workspace, "workspace"),
                                     workspace.numel() * workspace.element_size(), _stream(stream)),
           "granq_range_reduce")


def granq_range_reduce_noalloc(x: torch.Tensor, ch_min: torch.Tensor, ch_max: torch.Tensor, stream=None,
                               desc: Optional[granq_desc_t] = None) -> None:
    """granq_range_reduce on the library's own static scratch (no workspace, no allocation)."""
    d = _desc_for(x, desc)
    _check(load().granq_range_reduce_noalloc(_dev(x, "x"), ctypes.byref(d), _vec(ch_min, d.c, "ch_min"),
                                             _vec(ch_max, d.c, "ch_max"), _stream(stream)),
           "granq_range_reduce_noalloc")


def granq_prescale(ch_min: torch.Tensor, ch_max: torch.Tensor, bits: int, scale: torch.Tensor,
                   zero_point: torch.Tensor, stream=None) -> None:
    c = ch_min.numel()
    _check(load().granq_prescale(_vec(ch_min, c, "ch_min"), _vec(ch_max, c, "ch_max"), c, int(bits),
                                 _vec(scale, c, "scale"), _vec(zero_point, c, "zero_point"),
                                 _stream(stream)), "granq_prescale")


def granq_calibrate(x: torch.Tensor, bits: int, ch_min: torch.Tensor, ch_max: torch.Tensor,
                    scale: torch.Tensor, zero_point: torch.Tensor, workspace: torch.Tensor,
                    stream=None, desc: Optional[granq_desc_t] = None) -> None:
    d = _desc_for(x, desc)
    _check(load().granq_calibrate(_dev(x, "x"), ctypes.byref(d), int(bits), _vec(ch_min, d.c, "ch_min"),
                                  _vec(ch_max, d.c, "ch_max"), _vec(scale, d.c, "scale"),
                                  _vec(zero_point, d.c, "zero_point"), _dev(workspace, "workspace"),
                                  workspace.numel() * workspace.element_size(), _stream(stream)),
           "granq_calibrate")


def granq_calibrate_fakequant_fwd(x: torch.Tensor, bits: int, ch_min: torch.Tensor, ch_max: torch.Tensor,
                                  scale: torch.Tensor, zero_point: torch.Tensor, x_hat: Optional[torch.Tensor],
                                  codes: Optional[torch.Tensor], workspace: torch.Tensor, stream=None,
                                  desc: Optional[granq_desc_t] = None) -> None:
    d = _desc_for(x, desc)
    if x_hat is None and codes is None:
        raise ValueError("x_hat and codes are both None: nothing to write")
    if x_hat is not None and (x_hat.dtype != x.dtype or x_hat.numel() != x.numel()):
        raise ValueError("x_hat must match x")
    if codes is not None and (codes.dtype != torch.uint8 or codes.numel() != x.numel()):
        raise ValueError("codes must be uint8 with one entry per element")
    _check(load().granq_calibrate_fakequant_fwd(
        _dev(x, "x"), ctypes.byref(d), int(bits), _vec(ch_min, d.c, "ch_min"), _vec(ch_max, d.c, "ch_max"),
        _vec(scale, d.c, "scale"), _vec(zero_point, d.c, "zero_point"),
        _dev(x_hat, "x_hat") if x_hat is not None else 0, _dev(codes, "codes") if codes is not None else 0,
        _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream(stream)),
        "granq_calibrate_fakequant_fwd")


def granq_resident_state_bytes(desc: granq_desc_t) -> int:
    """Bytes of state the single-launch forward needs; 0 if it does not take this descriptor."""
    out = ctypes.c_size_t(0)
    st = load().granq_resident_state_bytes(ctypes.byref(desc), ctypes.byref(out))
    if st == GRANQ_ERR_UNSUPPORTED:
        return 0
    _check(st, "granq_resident_state_bytes")
    return int(out.value)


def granq_resident_state_init(state: torch.Tensor, stream=None) -> None:
    _check(load().granq_resident_state_init(_dev(state, "state"), state.numel() * state.element_size(),
                                            _stream(stream)), "granq_resident_state_init")


def granq_calibrate_fakequant_fwd_resident(x: torch.Tensor, bits: int, ch_min: torch.Tensor, ch_max: torch.Tensor,
                                           scale: torch.Tensor, zero_point: torch.Tensor,
                                           x_hat: Optional[torch.Tensor], codes: Optional[torch.Tensor],
                                           state: torch.Tensor, stream=None,
                                           desc: Optional[granq_desc_t] = None) -> bool:
    """Ranges, parameters and forward in one launch.  Returns False, with nothing launched, when
    the library does not take this tensor in that form (the caller then uses
    granq_calibrate_fakequant_fwd)."""
    d = _desc_for(x, desc)
    if x_hat is None and codes is None:
        raise ValueError("x_hat and codes are both None: nothing to write")
    if x_hat is not None and (x_hat.dtype != x.dtype or x_hat.numel() != x.numel()):
        raise ValueError("x_hat must match x")
    if codes is not None and (codes.dtype != torch.uint8 or codes.numel() != x.numel()):
        raise ValueError("codes must be uint8 with one entry per element")
    st = load().granq_calibrate_fakequant_fwd_resident(
        _dev(x, "x"), ctypes.byref(d), int(bits), _vec(ch_min, d.c, "ch_min"), _vec(ch_max, d.c, "ch_max"),
        _vec(scale, d.c, "scale"), _vec(zero_point, d.c, "zero_point"),
        _dev(x_hat, "x_hat") if x_hat is not None else 0, _dev(codes, "codes") if codes is not None else 0,
        _dev(state, "state"), state.numel() * state.element_size(), _stream(stream))
    if st == GRANQ_ERR_UNSUPPORTED:
        return False
    _check(st, "granq_calibrate_fakequant_fwd_resident")
    return True


def granq_fakequant_fwd(x: torch.Tensor, scale: torch.Tensor, zero_point: torch.Tensor, bits: int,
                        x_hat: Optional[torch.Tensor], codes: Optional[torch.Tensor] = None, stream=None,
                        desc: Optional[granq_desc_t] = None) -> None:
    """x_hat None: only the codes are written (codes must then be given)."""
    d = _desc_for(x, desc)
    if x_hat is None and codes is None:
        raise ValueError("x_hat and codes are both None: nothing to write")
    if x_hat is not None and (x_hat.dtype != x.dtype or x_hat.numel() != x.numel()):
        raise ValueError("x_hat must match x")
    cp = 0
    if codes is not None:
        if codes.dtype != torch.uint8 or codes.numel() != x.numel():
            raise ValueError("codes must be uint8 with one entry per element")
        cp = _dev(codes, "codes")
    _check(load().granq_fakequant_fwd(_dev(x, "x"), ctypes.byref(d), _vec(scale, d.c, "scale"),
                                      _vec(zero_point, d.c, "zero_point"), int(bits),
                                      _dev(x_hat, "x_hat") if x_hat is not None else 0, cp,
                                      _stream(stream)),
           "granq_fakequant_fwd")


def granq_fakequant_bwd(x: torch.Tensor, dy: torch.Tensor, scale: torch.Tensor,
                        zero_point: torch.Tensor, bits: int, dx: torch.Tensor, stream=None,
                        desc: Optional[granq_desc_t] = None) -> None:
    d = _desc_for(x, desc)
    if dy.dtype != x.dtype or dx.dtype != x.dtype or dy.numel() != x.numel() or dx.numel() != x.numel():
        raise ValueError("dy and dx must match x")
    _check(load().granq_fakequant_bwd(_dev(x, "x"), _dev(dy, "dy"), ctypes.byref(d),
                                      _vec(scale, d.c, "scale"), _vec(zero_point, d.c, "zero_point"),
                                      int(bits), _dev(dx, "dx"), _stream(stream)),
           "granq_fakequant_bwd")


def granq_mask_bytes(desc: granq_desc_t) -> int:
    out = ctypes.c_size_t(0)
    _check(load().granq_mask_bytes(ctypes.byref(desc), ctypes.byref(out)), "granq_mask_bytes")
    return int(out.value)


def granq_fakequant_fwd_mask(x: torch.Tensor, scale: torch.Tensor, zero_point: torch.Tensor, bits: int,
                             x_hat: torch.Tensor, mask: torch.Tensor, stream=None,
                             desc: Optional[granq_desc_t] = None) -> None:
    d = _desc_for(x, desc)
    if x_hat.dtype != x.dtype or x_hat.numel() != x.numel():
        raise ValueError("x_hat must match x")
    if mask.dtype != torch.uint8 or mask.numel() < (x.numel() + 7) // 8:
        raise ValueError("mask must be uint8 with at least ceil(numel / 8) entries")
    _check(load().granq_fakequant_fwd_mask(_dev(x, "x"), ctypes.byref(d), _vec(scale, d.c, "scale"),
                                           _vec(zero_point, d.c, "zero_point"), int(bits),
                                           _dev(x_hat, "x_hat"), _dev(mask, "mask"), _stream(stream)),
           "granq_fakequant_fwd_mask")


def granq_fakequant_bwd_mask(dy: torch.Tensor, mask: torch.Tensor, dx: torch.Tensor, stream=None,
                             desc: Optional[granq_desc_t] = None) -> None:
    d = _desc_for(dy, desc, "dy")
    if dx.dtype != dy.dtype or dx.numel() != dy.numel():
        raise ValueError("dx must match dy")
    if mask.dtype != torch.uint8 or mask.numel() < (dy.numel() + 7) // 8:
        raise ValueError("mask must be uint8 with at least ceil(numel / 8) entries")
    _check(load().granq_fakequant_bwd_mask(_dev(dy, "dy"), _dev(mask, "mask"), ctypes.byref(d),
                                           _dev(dx, "dx"), _stream(stream)), "granq_fakequant_bwd_mask")


def _rows_of(t: torch.Tensor):
    if t.dim() < 2:
        raise ValueError("a weight needs at least (rows, ...) dimensions")
    return int(t.shape[0]), t.numel() // int(t.shape[0])


def rowwise_items(weights, outs, scales, zero_points):
    """Marshal lists of tensors into the host descriptor array (keep it to reuse it)."""
    n = len(weights)
    arr = (granq_rowq_item_t * n)()
    for i, (w, o, s, z) in enumerate(zip(weights, outs, scales, zero_points)):
        rows, row_len = _rows_of(w)
        if o.dtype != w.dtype or o.numel() != w.numel():
            raise ValueError("w_hat must match w")
        arr[i] = granq_rowq_item_t(_dev(w, "w"), _dev(o, "w_hat"), _vec(s, rows, "scale"),
                                   _vec(z, rows, "zero_point"), rows, row_len)
    return arr


def granq_rowwise_fakequant_multi(items, dtype: torch.dtype, bits: int, stream=None) -> None:
    code = dtype_code(dtype)
    _check(load().granq_rowwise_fakequant_multi(ctypes.cast(items, _vp), len(items), code, int(bits),
                                                _stream(stream)), "granq_rowwise_fakequant_multi")


def rowwise_bwd_items(weights, dys, dws, scales, zero_points):
    n = len(weights)
    arr = (granq_rowq_bwd_item_t * n)()
    for i, (w, g, o, s, z) in enumerate(zip(weights, dys, dws, scales, zero_points)):
        rows, row_len = _rows_of(w)
        arr[i] = granq_rowq_bwd_item_t(_dev(w, "w"), _dev(g, "dy"), _dev(o, "dw"), _vec(s, rows, "scale"),
                                       _vec(z, rows, "zero_point"), rows, row_len)
    return arr


def granq_rowwise_fakequant_bwd_multi(items, dtype: torch.dtype, bits: int, stream=None) -> None:
    code = dtype_code(dtype)
    _check(load().granq_rowwise_fakequant_bwd_multi(ctypes.cast(items, _vp), len(items), code, int(bits),
                                                    _stream(stream)), "granq_rowwise_fakequant_bwd_multi")


def granq_fold_weights(w: torch.Tensor, scale: torch.Tensor, zero_point: torch.Tensor, wq: torch.Tensor,
                       corr: torch.Tensor, out_scale: torch.Tensor, stream=None) -> None:
    o, c = int(w.shape[0]), w.numel() // int(w.shape[0])
    if w.dtype != torch.float32 or wq.dtype != torch.int8 or wq.numel() != o * c:
        raise ValueError("w must be float32 (O, C) and wq int8 of the same size")
    if corr.dtype != torch.int64 or corr.numel() != o:
        raise ValueError("corr must be int64 with O entries")
    _check(load().granq_fold_weights(_dev(w, "w"), _vec(scale, c, "scale"), _vec(zero_point, c, "zero_point"),
                                     o, c, _dev(wq, "wq"), _dev(corr, "corr"), _vec(out_scale, o, "out_scale"),
                                     _stream(stream)), "granq_fold_weights")


def granq_conv1x1_int8(codes: torch.Tensor, wq: torch.Tensor, corr: torch.Tensor, out_scale: torch.Tensor,
                       bits: int, y: torch.Tensor, stream=None) -> None:
    if codes.dtype != torch.uint8 or codes.dim() != 4:
        raise ValueError("codes must be a uint8 (N, C, H, W) tensor")
    n, c, h, w = (int(v) for v in codes.shape)
    o = int(wq.shape[0])
    if wq.dtype != torch.int8 or wq.numel() != o * c or corr.dtype != torch.int64 or corr.numel() != o:
        raise ValueError("wq must be int8 (O, C) and corr int64 (O)")
    if y.dtype != torch.float32 or y.numel() != n * o * h * w:
        raise ValueError("y must be float32 (N, O, H, W)")
    d = make_desc(n, c, h, w, GRANQ_F32)
    _check(load().granq_conv1x1_int8(_dev(codes, "codes"), ctypes.byref(d), o, _dev(wq, "wq"),
                                     _dev(corr, "corr"), _vec(out_scale, o, "out_scale"), int(bits),
                                     _dev(y, "y"), _stream(stream)), "granq_conv1x1_int8")


def granq_conv1x1_int8_as(codes: torch.Tensor, wq: torch.Tensor, corr: torch.Tensor, out_scale: torch.Tensor,
                          bits: int, y: torch.Tensor, stream=None) -> None:
    """granq_conv1x1_int8 with y stored in y's own dtype (float32, bfloat16 or float16)."""
    if codes.dtype != torch.uint8 or codes.dim() != 4:
        raise ValueError("codes must be a uint8 (N, C, H, W) tensor")
    n, c, h, w = (int(v) for v in codes.shape)
    o = int(wq.shape[0])
    if wq.dtype != torch.int8 or wq.numel() != o * c or corr.dtype != torch.int64 or corr.numel() != o:
        raise ValueError("wq must be int8 (O, C) and corr int64 (O)")
    if y.numel() != n * o * h * w:
        raise ValueError("y must have N*O*H*W elements")
    d = make_desc(n, c, h, w, GRANQ_F32)
    _check(load().granq_conv1x1_int8_as(_dev(codes, "codes"), ctypes.byref(d), o, _dev(wq, "wq"),
                                        _dev(corr, "corr"), _vec(out_scale, o, "out_scale"), int(bits),
                                        dtype_code(y.dtype), _dev(y, "y"), _stream(stream)),
           "granq_conv1x1_int8_as")


def granq_packed4_bytes(desc: granq_desc_t) -> int:
    out = ctypes.c_size_t(0)
    _check(load().granq_packed4_bytes(ctypes.byref(desc), ctypes.byref(out)), "granq_packed4_bytes")
    return int(out.value)


def granq_fakequant_fwd_packed4(x: torch.Tensor, scale: torch.Tensor, zero_point: torch.Tensor, bits: int,
                                x_hat: Optional[torch.Tensor], packed: torch.Tensor, stream=None,
                                desc: Optional[granq_desc_t] = None) -> None:
    """The forward with its codes stored two per byte (bits <= 4); x_hat None: codes only."""
    d = _desc_for(x, desc)
    if x_hat is not None and (x_hat.dtype != x.dtype or x_hat.numel() != x.numel()):
        raise ValueError("x_hat must match x")
    if packed.dtype != torch.uint8 or packed.numel() < (x.numel() + 1) // 2:
        raise ValueError("packed must be uint8 with at least ceil(numel / 2) entries")
    _check(load().granq_fakequant_fwd_packed4(_dev(x, "x"), ctypes.byref(d), _vec(scale, d.c, "scale"),
                                              _vec(zero_point, d.c, "zero_point"), int(bits),
                                              _dev(x_hat, "x_hat") if x_hat is not None else 0,
                                              _dev(packed, "packed"), _stream(stream)),
           "granq_fakequant_fwd_packed4")


def granq_conv1x1_int8_packed4(packed: torch.Tensor, shape, wq: torch.Tensor, corr: torch.Tensor,
                               out_scale: torch.Tensor, bits: int, y: torch.Tensor, stream=None) -> None:
    """granq_conv1x1_int8_as on codes stored two per byte; `shape` = (N, C, H, W) of the codes."""
    n, c, h, w = (int(v) for v in shape)
    o = int(wq.shape[0])
    if packed.dtype != torch.uint8 or packed.numel() < (n * c * h * w + 1) // 2:
        raise ValueError("packed must be uint8 with at least ceil(N*C*H*W / 2) entries")
    if wq.dtype != torch.int8 or wq.numel() != o * c or corr.dtype != torch.int64 or corr.numel() != o:
        raise ValueError("wq must be int8 (O, C) and corr int64 (O)")
    if y.numel() != n * o * h * w:
        raise ValueError("y must have N*O*H*W elements")
    d = make_desc(n, c, h, w, GRANQ_F32)
    _check(load().granq_conv1x1_int8_packed4(_dev(packed, "packed"), ctypes.byref(d), o, _dev(wq, "wq"),
                                             _dev(corr, "corr"), _vec(out_scale, o, "out_scale"), int(bits),
                                             dtype_code(y.dtype), _dev(y, "y"), _stream(stream)),
           "granq_conv1x1_int8_packed4")


def granq_conv1x1_float(x_hat: torch.Tensor, w: torch.Tensor, y: torch.Tensor, stream=None) -> None:
    """y[n,o] = sum_c w[o,c] * x_hat[n,c] over an (N, C, H, W) tensor; w (O, C) and y (N, O, H, W)
    have x_hat's dtype."""
    if x_hat.dim() != 4:
        raise ValueError("x_hat must be an (N, C, H, W) tensor")
    n, c, h, wd = (int(v) for v in x_hat.shape)
    o = int(w.shape[0])
    if w.dtype != x_hat.dtype or w.numel() != o * c:
        raise ValueError("w must be (O, C) of x_hat's dtype")
    if y.dtype != x_hat.dtype or y.numel() != n * o * h * wd:
        raise ValueError("y must be (N, O, H, W) of x_hat's dtype")
    d = make_desc(n, c, h, wd, dtype_code(x_hat.dtype))
    _check(load().granq_conv1x1_float(_dev(x_hat, "x_hat"), ctypes.byref(d), o, _dev(w, "w"), _dev(y, "y"),
                                      _stream(stream)), "granq_conv1x1_float")


def granq_distortion_workspace_bytes(desc: granq_desc_t) -> int:
    out = ctypes.c_size_t(0)
    _check(load().granq_distortion_workspace_bytes(ctypes.byref(desc), ctypes.byref(out)),
           "granq_distortion_workspace_bytes")
    return int(out.value)


def granq_distortion(x: torch.Tensor, scale: torch.Tensor, zero_point: torch.Tensor, bits: int,
                     ch_sums: torch.Tensor, layer: torch.Tensor, workspace: torch.Tensor, stream=None,
                     desc: Optional[granq_desc_t] = None) -> None:
    d = _desc_for(x, desc)
    if ch_sums.dtype != torch.float64 or ch_sums.numel() != 4 * d.c:
        raise ValueError("ch_sums must be float64 with 4*C entries")
    if layer.dtype != torch.float64 or layer.numel() != 6:
        raise ValueError("layer must be float64 with 6 entries")
    _check(load().granq_distortion(_dev(x, "x"), ctypes.byref(d), _vec(scale, d.c, "scale"),
                                   _vec(zero_point, d.c, "zero_point"), int(bits), _dev(ch_sums, "ch_sums"),
                                   _dev(layer, "layer"), _dev(workspace, "workspace"),
                                   workspace.numel() * workspace.element_size(), _stream(stream)),
           "granq_distortion")


# --- comparison points for the benchmark (include/granq_compare.h) ---------------------------

def granq_cmp_channel_loop_fwd(x: torch.Tensor, bits: int, ch_min: torch.Tensor, ch_max: torch.Tensor,
                               scale: torch.Tensor, zero_point: torch.Tensor, x_hat: torch.Tensor,
                               workspace: torch.Tensor, stream=None,
                               desc: Optional[granq_desc_t] = None) -> None:
    d = _desc_for(x, desc)
    if x_hat.dtype != x.dtype or x_hat.numel() != x.numel():
        raise ValueError("x_hat must match x")
    _check(load().granq_cmp_channel_loop_fwd(
        _dev(x, "x"), ctypes.byref(d), int(bits), _vec(ch_min, d.c, "ch_min"), _vec(ch_max, d.c, "ch_max"),
        _vec(scale, d.c, "scale"), _vec(zero_point, d.c, "zero_point"), _dev(x_hat, "x_hat"),
        _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream(stream)),
        "granq_cmp_channel_loop_fwd")


def granq_cmp_accumulate_inloop(codes: torch.Tensor, scale: torch.Tensor, zero_point: torch.Tensor,
                                weight: torch.Tensor, y: torch.Tensor, stream=None,
                                desc: Optional[granq_desc_t] = None) -> None:
    d = _desc_for(codes, desc, "codes", typed=False) if desc is not None else make_desc(
        codes.shape[0], codes.shape[1], codes.shape[2], codes.shape[3], GRANQ_F32)
    if codes.dtype != torch.uint8 or y.dtype != torch.float32 or y.numel() != d.n * d.h * d.w:
        raise ValueError("codes must be uint8 and y float32 with N*H*W entries")
    _check(load().granq_cmp_accumulate_inloop(
        _dev(codes, "codes"), ctypes.byref(d), _vec(scale, d.c, "scale"), _vec(zero_point, d.c, "zero_point"),
        _vec(weight, d.c, "weight"), _dev(y, "y"), _stream(stream)), "granq_cmp_accumulate_inloop")


def granq_cmp_accumulate_prescaled(x_hat: torch.Tensor, weight: torch.Tensor, y: torch.Tensor, stream=None,
                                   desc: Optional[granq_desc_t] = None) -> None:
    d = _desc_for(x_hat, desc, "x_hat")
    if x_hat.dtype != torch.float32 or y.dtype != torch.float32 or y.numel() != d.n * d.h * d.w:
        raise ValueError("x_hat and y must be float32, y with N*H*W entries")
    _check(load().granq_cmp_accumulate_prescaled(
        _dev(x_hat, "x_hat"), ctypes.byref(d), _vec(weight, d.c, "weight"), _dev(y, "y"), _stream(stream)),
        "granq_cmp_accumulate_prescaled")
