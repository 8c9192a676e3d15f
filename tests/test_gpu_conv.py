"""Integer-domain 1x1 convolution on the codes (int8 MFMA) and the weight fold, bit for bit
against the oracle's integer loops (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_18339_amd as G
import workloads
from parity import bits_view, gpu_path, to_numpy

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _case(shape, o, bits, law="linear", seed=0):
    n, c, h, w = shape
    x = workloads.make_activation(shape, law, (0.05, 20.0), seed, DEV)
    out = gpu_path(x, bits)
    g = torch.Generator(device=DEV).manual_seed(seed + 5)
    wt = torch.randn(o, c, generator=g, device=DEV) * torch.exp(torch.randn(o, 1, generator=g, device=DEV))
    s = torch.from_numpy(out["scale"]).to(DEV)
    z = torch.from_numpy(out["zero_point"]).to(DEV)
    wq = torch.full((o, c), 99, dtype=torch.int8, device=DEV)
    corr = torch.full((o,), 12345, dtype=torch.int32, device=DEV)
    a = torch.full((o,), float("nan"), device=DEV)
    G.granq_fold_weights(wt, s, z, wq, corr, a)
    codes = torch.from_numpy(out["codes"]).to(DEV)
    y = torch.full((n, o, h, w), float("nan"), device=DEV)
    G.granq_conv1x1_int8(codes, wq, corr, a, bits, y)
    torch.cuda.synchronize()
    ewq, ecorr, ea = oracle.fold_weights(wt.cpu().numpy(), out["scale"], out["zero_point"])
    assert np.array_equal(wq.cpu().numpy(), ewq)
    assert np.array_equal(corr.cpu().numpy(), ecorr)
    assert np.array_equal(bits_view(a.cpu().numpy()), bits_view(ea))
    want = oracle.conv1x1_int8(out["codes"], ewq, ecorr, ea)
    got = y.cpu().numpy()
    bad = np.nonzero(bits_view(got).ravel() != bits_view(want).ravel())[0]
    assert bad.size == 0, "y differs at %d of %d, first flat index %d" % (bad.size, got.size, bad[0])
    return x, out, wt, got


# matrix-core path: C % 16 == 0, O % 32 == 0, H*W % 4 == 0, bits <= 7
@pytest.mark.parametrize("shape,o,bits", [
    ((2, 16, 8, 8), 32, 4), ((3, 64, 14, 14), 64, 4), ((2, 32, 7, 12), 96, 3), ((1, 128, 28, 28), 160, 5),
    ((4, 48, 2, 2), 32, 7), ((2, 64, 56, 56), 64, 4), ((1, 256, 1, 4), 64, 4), ((2, 16, 23, 12), 128, 2),
    # more channels than one LDS chunk of weights (512), with a 16-channel tail; many samples per wavefront
    ((2, 1040, 2, 4), 96, 4), ((1, 528, 4, 4), 64, 6), ((70, 32, 1, 4), 32, 4), ((3, 1024, 14, 14), 256, 4),
])
def test_conv_mfma_path(shape, o, bits):
    _case(shape, o, bits)


# plain integer path: any other shape, and 8-bit codes
@pytest.mark.parametrize("shape,o,bits", [
    ((2, 7, 5, 5), 3, 4), ((1, 16, 7, 7), 32, 4), ((2, 24, 4, 4), 32, 4), ((2, 16, 4, 4), 40, 4),
    ((2, 16, 8, 8), 32, 8), ((1, 1, 1, 1), 1, 1),
])
def test_conv_plain_path(shape, o, bits):
    _case(shape, o, bits)


@pytest.mark.parametrize("ydtype", [torch.bfloat16, torch.float16], ids=["bf16", "f16"])
@pytest.mark.parametrize("shape,o,bits", [((3, 64, 14, 14), 64, 4), ((2, 528, 4, 4), 96, 6), ((2, 7, 5, 5), 3, 4),
                                          ((2, 16, 8, 8), 32, 8)])
def test_conv_output_in_16_bits(shape, o, bits, ydtype):
    """y stored as bfloat16 / binary16: the oracle's binary32 result narrowed with round to nearest
    even (torch's conversion for bfloat16, the oracle's own for binary16), bit for bit; both kernels."""
    n, c, h, w = shape
    x = workloads.make_activation(shape, "linear", (0.05, 20.0), 1, DEV)
    out = gpu_path(x, bits)
    g = torch.Generator(device=DEV).manual_seed(9)
    wt = torch.randn(o, c, generator=g, device=DEV) * torch.exp(torch.randn(o, 1, generator=g, device=DEV))
    s = torch.from_numpy(out["scale"]).to(DEV)
    z = torch.from_numpy(out["zero_point"]).to(DEV)
    wq = torch.empty((o, c), dtype=torch.int8, device=DEV)
    corr = torch.empty((o,), dtype=torch.int32, device=DEV)
    a = torch.empty((o,), device=DEV)
    G.granq_fold_weights(wt, s, z, wq, corr, a)
    codes = torch.from_numpy(out["codes"]).to(DEV)
    y = torch.full((n, o, h, w), float("nan"), dtype=ydtype, device=DEV)
    G.granq_conv1x1_int8_as(codes, wq, corr, a, bits, y)
    torch.cuda.synchronize()
    want32 = oracle.conv1x1_int8(out["codes"], wq.cpu().numpy(), corr.cpu().numpy(), a.cpu().numpy())
    if ydtype == torch.float16:
        want = oracle.f16_narrow(want32)
    else:
        want = torch.from_numpy(want32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = y.view(torch.int16).cpu().numpy().view(np.uint16)
    bad = np.nonzero(got.ravel() != want.ravel())[0]
    assert bad.size == 0, "y differs at %d of %d" % (bad.size, got.size)
    # float32 through the same entry point is the plain call
    y32 = torch.empty((n, o, h, w), device=DEV)
    G.granq_conv1x1_int8_as(codes, wq, corr, a, bits, y32)
    torch.cuda.synchronize()
    assert np.array_equal(bits_view(y32.cpu().numpy()), bits_view(want32))


def test_conv_approximates_the_float_convolution():
    """Eq. 3 folded into integers against Eq. 6 in binary64: within the rounding of the folded weights."""
    shape, o = (2, 64, 14, 14), 64
    x, out, wt, y = _case(shape, o, 4, seed=3)
    ref = np.einsum("oc,nchw->nohw", wt.cpu().numpy().astype(np.float64), out["xhat"].astype(np.float64))
    wq, corr, a = oracle.fold_weights(wt.cpu().numpy(), out["scale"], out["zero_point"])
    bound = 0.5 * a.astype(np.float64).reshape(1, -1, 1, 1) * np.abs(
        out["codes"].astype(np.float64) - out["zero_point"].reshape(1, -1, 1, 1)).sum(axis=1, keepdims=True)
    assert np.all(np.abs(y - ref) <= bound * (1 + 1e-4) + 1e-5 * np.abs(ref).max())
    rel = np.linalg.norm(y - ref) / np.linalg.norm(ref)
    assert rel < 0.02


def test_conv_argument_checks():
    import ctypes
    lib = G.load()
    d = G.make_desc(2, 16, 4, 4, 0)
    assert lib.granq_conv1x1_int8(16, ctypes.byref(d), 32, 16, 16, 16, 9, 16, 0) == G.GRANQ_ERR_INVALID_ARG
    assert lib.granq_conv1x1_int8(16, ctypes.byref(d), 0, 16, 16, 16, 4, 16, 0) == G.GRANQ_ERR_INVALID_ARG
    assert lib.granq_conv1x1_int8(0, ctypes.byref(d), 32, 16, 16, 16, 4, 16, 0) == G.GRANQ_ERR_INVALID_ARG
    assert lib.granq_conv1x1_int8(16, ctypes.byref(d), 32, 16, 18, 16, 4, 16, 0) == G.GRANQ_ERR_UNSUPPORTED
    assert lib.granq_fold_weights(16, 16, 16, 0, 4, 16, 16, 16, 0) == G.GRANQ_ERR_INVALID_ARG
    assert lib.granq_fold_weights(16, 16, 0, 4, 4, 16, 16, 16, 0) == G.GRANQ_ERR_INVALID_ARG
