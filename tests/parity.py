"""Helpers for the GPU-vs-oracle parity tests: run the HIP library through its
C ABI, run the oracle on the same bits, compare element by element."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

import oracle
import paper_2503_18339_amd as G

WORKERS = 8


def to_numpy(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> host array the oracle takes (bf16 as uint16 bit patterns)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def bits_view(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.float32:
        return a.view(np.uint32)
    if a.dtype == np.float16:
        return a.view(np.uint16)
    return a


def values(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.uint16:
        return oracle.f32_from_bf16_bits(a)
    if a.dtype == np.float16:
        return a.astype(np.float32)
    return a


def _chunks(n, parts):
    step = max(1, -(-n // parts))
    return [(i, min(n, i + step)) for i in range(0, n, step)]


def oracle_fwd(x, s, z, bits, workers=WORKERS):
    """Oracle forward; large tensors are split over the batch across threads
    (the forward is element-wise once scale and zero-point are given)."""
    if x.size < (1 << 22) or x.shape[0] < 2:
        return oracle.fakequant_fwd(x, s, z, bits)
    xhat = np.empty_like(x)
    codes = np.empty(x.shape, np.uint8)

    def work(rng):
        a, b = rng
        xhat[a:b], codes[a:b] = oracle.fakequant_fwd(x[a:b], s, z, bits)

    with ThreadPoolExecutor(workers) as ex:
        list(ex.map(work, _chunks(x.shape[0], workers * 2)))
    return xhat, codes


def oracle_bwd(x, dy, s, z, bits, workers=WORKERS):
    if x.size < (1 << 22) or x.shape[0] < 2:
        return oracle.fakequant_bwd(x, dy, s, z, bits)
    dx = np.empty_like(x)

    def work(rng):
        a, b = rng
        dx[a:b] = oracle.fakequant_bwd(x[a:b], dy[a:b], s, z, bits)

    with ThreadPoolExecutor(workers) as ex:
        list(ex.map(work, _chunks(x.shape[0], workers * 2)))
    return dx


def gpu_path(x: torch.Tensor, bits: int, dy: torch.Tensor = None, want_codes=True, desc=None,
             scale=None, zero_point=None):
    """range_reduce -> prescale -> fwd (-> bwd) through the C ABI.  Returns host arrays."""
    d = desc or G.desc_of(x)
    c = d.c
    dev = x.device
    out = {}
    f32 = dict(dtype=torch.float32, device=dev)
    if scale is None:
        ch_min = torch.full((c,), float("nan"), **f32)
        ch_max = torch.full((c,), float("nan"), **f32)
        ws = torch.empty(max(16, G.granq_workspace_bytes(d)), dtype=torch.uint8, device=dev)
        s = torch.full((c,), float("nan"), **f32)
        z = torch.full((c,), float("nan"), **f32)
        G.granq_range_reduce(x, ch_min, ch_max, ws, desc=d)
        G.granq_prescale(ch_min, ch_max, bits, s, z)
        out["min"], out["max"] = ch_min.cpu().numpy(), ch_max.cpu().numpy()
        # the one-call form must write the same four vectors, bit for bit
        four = [torch.full((c,), float("nan"), **f32) for _ in range(4)]
        G.granq_calibrate(x, bits, four[0], four[1], four[2], four[3], ws, desc=d)
        for got, ref, name in zip(four, (ch_min, ch_max, s, z), ("min", "max", "scale", "zero_point")):
            assert torch.equal(got.view(torch.int32), ref.view(torch.int32)), "granq_calibrate: " + name
    else:
        s = torch.as_tensor(scale, **f32)
        z = torch.as_tensor(zero_point, **f32)
    x_hat = torch.empty_like(x)
    codes = torch.full(x.shape, 255, dtype=torch.uint8, device=dev) if want_codes else None
    G.granq_fakequant_fwd(x, s, z, bits, x_hat, codes, desc=d)
    out["scale"], out["zero_point"] = s.cpu().numpy(), z.cpu().numpy()
    out["xhat"] = to_numpy(x_hat)
    if scale is None and want_codes:
        # ranges, parameters and forward in ONE call (a single launch for small channels) must
        # write the same six results, bit for bit
        six = [torch.full((c,), float("nan"), **f32) for _ in range(4)]
        xh1 = torch.empty_like(x)
        cd1 = torch.full(x.shape, 253, dtype=torch.uint8, device=dev)
        G.granq_calibrate_fakequant_fwd(x, bits, six[0], six[1], six[2], six[3], xh1, cd1, ws, desc=d)
        for got1, ref, name in zip(six, (ch_min, ch_max, s, z), ("min", "max", "scale", "zero_point")):
            assert torch.equal(got1.view(torch.int32), ref.view(torch.int32)), "one-call forward: " + name
        assert torch.equal(cd1, codes), "one-call forward: codes"
        ib = torch.int32 if x.dtype == torch.float32 else torch.int16
        assert torch.equal(xh1.view(ib), x_hat.view(ib)), "one-call forward: x_hat"
    if want_codes:
        out["codes"] = codes.cpu().numpy()
        # the quantize step alone (no x_hat) must write the same codes
        only = torch.full(x.shape, 254, dtype=torch.uint8, device=dev)
        G.granq_fakequant_fwd(x, s, z, bits, None, only, desc=d)
        assert torch.equal(only, codes), "codes-only forward differs from the forward with x_hat"
    if dy is not None:
        dx = torch.empty_like(x)
        G.granq_fakequant_bwd(x, dy, s, z, bits, dx, desc=d)
        out["dx"] = to_numpy(dx)
    torch.cuda.synchronize()
    return out


def oracle_path(x_np: np.ndarray, bits: int, dy_np: np.ndarray = None, view_shape=None,
                scale=None, zero_point=None):
    xv = x_np.reshape(view_shape) if view_shape else x_np
    out = {}
    if scale is None:
        mn, mx = oracle.range_reduce(xv)
        s, z = oracle.prescale(mn, mx, bits)
        out["min"], out["max"] = mn, mx
    else:
        s, z = np.asarray(scale, np.float32), np.asarray(zero_point, np.float32)
    out["scale"], out["zero_point"] = s, z
    xhat, codes = oracle_fwd(xv, s, z, bits)
    out["xhat"], out["codes"] = xhat.reshape(x_np.shape), codes.reshape(x_np.shape)
    if dy_np is not None:
        dyv = dy_np.reshape(view_shape) if view_shape else dy_np
        out["dx"] = oracle_bwd(xv, dyv, s, z, bits).reshape(x_np.shape)
    return out


def first_mismatch(a, b):
    bad = np.nonzero(a.ravel() != b.ravel())[0]
    return None if bad.size == 0 else (int(bad[0]), bad.size)


def assert_parity(got: dict, want: dict, what=""):
    """The bar: ranges equal as values (+0 == -0), scale / zero-point bit-exact, codes
    bit-exact, x_hat equal as values and within 1e-6 relative, dx bit-exact."""
    for key in ("min", "max"):
        if key in want and key in got:
            assert np.array_equal(got[key], want[key]), "%s %s differs: %r" % (
                what, key, first_mismatch(got[key], want[key]))
    for key in ("scale", "zero_point"):
        assert np.array_equal(bits_view(got[key]), bits_view(want[key])), "%s %s not bit-exact: %r" % (
            what, key, first_mismatch(bits_view(got[key]), bits_view(want[key])))
    if "codes" in got:
        mm = first_mismatch(got["codes"], want["codes"])
        assert mm is None, "%s codes differ at flat index %d (%d in total)" % ((what,) + mm)
    gv, wv = values(got["xhat"]), values(want["xhat"])
    # tolerance for floating-point outputs: 1e-6 relative
    fin = np.isfinite(wv)                    # binary16 storage overflows to infinity above 65504
    tol = 1e-6 * np.abs(wv[fin])
    far = np.nonzero(np.abs(gv[fin].astype(np.float64) - wv[fin].astype(np.float64)) > tol)[0]
    assert far.size == 0, "%s xhat beyond 1e-6 relative at %d places, first (finite-flat index %d): got %r want %r" % (
        what, far.size, far[0], gv[fin][far[0]], wv[fin][far[0]])
    mm = first_mismatch(gv, wv)              # expectation: identical values (only +-0 may differ in bits)
    assert mm is None, "%s xhat differs at flat index %d (%d in total)" % ((what,) + mm)
    if got["xhat"].dtype in (np.uint16, np.float16):
        nz = wv != 0
        assert np.array_equal(bits_view(got["xhat"])[nz], bits_view(want["xhat"])[nz]), what + " 16-bit xhat bits differ"
    if "dx" in want and "dx" in got:
        g, w = got["dx"], want["dx"]
        mm = first_mismatch(bits_view(g), bits_view(w))
        assert mm is None, "%s dx not bit-exact at flat index %d (%d in total)" % ((what,) + mm)
