"""The benchmark's comparison points against the oracle and against the library (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_18339_amd as G
import workloads
from parity import gpu_path, to_numpy

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.mark.parametrize("shape,law,bits", [((8, 16, 32, 32), "relu", 3), ((5, 7, 9, 9), "linear", 4),
                                            ((3, 33, 7, 7), "laplace", 8), ((16, 64, 8, 8), "relu", 3)])
def test_channel_loop_equals_vectorized_path(shape, law, bits):
    """The channel-by-channel loop (Sec. 5.3.2 baseline) reaches exactly the library's results."""
    x = workloads.make_activation(shape, law, (0.05, 20.0), 1, DEV)
    c = shape[1]
    v = [torch.full((c,), float("nan"), device=DEV) for _ in range(4)]
    x_hat = torch.empty_like(x)
    ws = torch.empty(max(16, 2 * shape[0]), device=DEV)
    G.granq_cmp_channel_loop_fwd(x, bits, v[0], v[1], v[2], v[3], x_hat, ws)
    torch.cuda.synchronize()
    lib = gpu_path(x, bits)
    mn, mx = oracle.range_reduce(to_numpy(x))
    s, z = oracle.prescale(mn, mx, bits)
    want, _ = oracle.fakequant_fwd(to_numpy(x), s, z, bits)
    for got, ref, libv in zip(v, (mn, mx, s, z), (lib["min"], lib["max"], lib["scale"], lib["zero_point"])):
        assert np.array_equal(got.cpu().numpy(), ref) and np.array_equal(libv, ref)
    assert np.array_equal(x_hat.cpu().numpy(), want)
    assert np.array_equal(lib["xhat"], want)


@pytest.mark.parametrize("shape", [(4, 12, 6, 6), (3, 64, 14, 14), (2, 5, 1, 300)])
def test_accumulation_forms(shape):
    """Eq. 3 (scale inside the loop, from codes) and Eq. 6 (pre-scaled) on the GPU, bit for bit
    against the oracle's loops, and agreeing with each other to rounding."""
    x = workloads.make_activation(shape, "linear", (0.05, 20.0), 2, DEV)
    out = gpu_path(x, 4)
    n, c, h, w = shape
    g = torch.Generator(device=DEV).manual_seed(3)
    weight = torch.randn(c, generator=g, device=DEV)
    codes = torch.from_numpy(out["codes"]).to(DEV)
    x_hat = torch.from_numpy(out["xhat"]).to(DEV)
    s = torch.from_numpy(out["scale"]).to(DEV)
    z = torch.from_numpy(out["zero_point"]).to(DEV)
    y3 = torch.empty(n, h, w, device=DEV)
    y6 = torch.empty(n, h, w, device=DEV)
    G.granq_cmp_accumulate_inloop(codes, s, z, weight, y3)
    G.granq_cmp_accumulate_prescaled(x_hat, weight, y6)
    torch.cuda.synchronize()
    w_np = weight.cpu().numpy()
    want3 = oracle.accumulate_inloop(out["codes"], out["scale"], out["zero_point"], w_np)
    want6 = oracle.accumulate_prescaled(out["xhat"], w_np)
    assert np.array_equal(y3.cpu().numpy(), want3)
    assert np.array_equal(y6.cpu().numpy(), want6)
    scale = float(np.abs(w_np).astype(np.float64) @ np.abs(out["xhat"]).max(axis=(0, 2, 3)))
    assert np.max(np.abs(want3 - want6)) <= 1e-5 * scale


def test_compare_argument_checks():
    import ctypes
    lib = G.load()
    d = G.make_desc(2, 3, 4, 4, G.GRANQ_BF16)
    assert lib.granq_cmp_accumulate_prescaled(16, ctypes.byref(d), 16, 16, 0) == G.GRANQ_ERR_UNSUPPORTED
    d = G.make_desc(2, 3, 4, 4, G.GRANQ_F32)
    assert lib.granq_cmp_accumulate_prescaled(0, ctypes.byref(d), 16, 16, 0) == G.GRANQ_ERR_INVALID_ARG
    assert lib.granq_cmp_channel_loop_fwd(16, ctypes.byref(d), 4, 16, 16, 16, 16, 16, 16, 8, 0) == G.GRANQ_ERR_WORKSPACE
    assert lib.granq_cmp_channel_loop_fwd(16, ctypes.byref(d), 0, 16, 16, 16, 16, 16, 16, 64, 0) == G.GRANQ_ERR_INVALID_ARG
