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
    corr = torch.full((o,), 12345, dtype=torch.int64, device=DEV)
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
    # many output and input channels: the variant whose four wavefronts share a pixel tile (a 16-channel
    # tail, output channels that are no multiple of 64 or 256, two groups of 256, many samples per tile)
    ((2, 128, 4, 4), 192, 4), ((1, 144, 2, 6), 224, 5), ((5, 272, 1, 4), 320, 3), ((40, 160, 1, 4), 512, 7),
    ((2, 2048, 7, 8), 512, 4), ((1, 256, 3, 4), 1024, 4),
])
def test_conv_mfma_path(shape, o, bits):
    _case(shape, o, bits)


# matrix-core path with H*W no multiple of 4 (7 x 7 maps): a sample's last pixel group holds one, two or
# three pixels and every access is aligned to one element only; both kernels (the second from 192 output
# and 128 input channels on), tiles that span several samples, a ragged last tile
@pytest.mark.parametrize("shape,o,bits", [
    ((1, 16, 7, 7), 32, 4), ((3, 64, 7, 7), 64, 4), ((2, 64, 5, 5), 96, 3), ((1, 32, 3, 2), 32, 7),
    ((2, 16, 9, 7), 64, 5), ((37, 48, 1, 5), 32, 4), ((2, 2048, 7, 7), 512, 4), ((5, 512, 7, 7), 2048, 4),
    ((4, 128, 1, 5), 224, 6), ((3, 272, 3, 3), 320, 2), ((70, 160, 1, 7), 192, 4),
])
def test_conv_mfma_path_ragged_maps(shape, o, bits):
    _case(shape, o, bits)


def test_conv_ragged_maps_from_unaligned_pointers():
    """With H*W no multiple of 4 the codes and y need the alignment of one element only."""
    shape, o, bits = (3, 64, 7, 7), 64, 4
    n, c, h, w = shape
    x = workloads.make_activation(shape, "linear", (0.05, 20.0), 2, DEV)
    out = gpu_path(x, bits)
    g = torch.Generator(device=DEV).manual_seed(11)
    wt = torch.randn(o, c, generator=g, device=DEV)
    s = torch.from_numpy(out["scale"]).to(DEV)
    z = torch.from_numpy(out["zero_point"]).to(DEV)
    wq = torch.empty((o, c), dtype=torch.int8, device=DEV)
    corr = torch.empty((o,), dtype=torch.int64, device=DEV)
    a = torch.empty((o,), device=DEV)
    G.granq_fold_weights(wt, s, z, wq, corr, a)
    want = oracle.conv1x1_int8(out["codes"], wq.cpu().numpy(), corr.cpu().numpy(), a.cpu().numpy())
    for shift in (1, 2, 3):
        cbuf = torch.zeros(n * c * h * w + 8, dtype=torch.uint8, device=DEV)
        codes = cbuf[shift:shift + n * c * h * w].view(shape)
        codes.copy_(torch.from_numpy(out["codes"]).to(DEV))
        ybuf = torch.full((n * o * h * w + 8,), float("nan"), device=DEV)
        y = ybuf[shift:shift + n * o * h * w].view(n, o, h, w)
        G.granq_conv1x1_int8(codes, wq, corr, a, bits, y)
        torch.cuda.synchronize()
        assert np.array_equal(bits_view(y.cpu().numpy()), bits_view(want)), shift
        assert torch.isnan(ybuf[:shift]).all() and torch.isnan(ybuf[shift + n * o * h * w:]).all()


# plain integer path: any other shape, and 8-bit codes
@pytest.mark.parametrize("shape,o,bits", [
    ((2, 7, 5, 5), 3, 4), ((1, 16, 1, 3), 32, 4), ((2, 24, 4, 4), 32, 4), ((2, 16, 4, 4), 40, 4),
    ((2, 16, 8, 8), 32, 8), ((1, 1, 1, 1), 1, 1), ((2, 16, 7, 7), 32, 8),
])
def test_conv_plain_path(shape, o, bits):
    _case(shape, o, bits)


@pytest.mark.parametrize("ydtype", [torch.bfloat16, torch.float16], ids=["bf16", "f16"])
@pytest.mark.parametrize("shape,o,bits", [((3, 64, 14, 14), 64, 4), ((2, 528, 4, 4), 96, 6), ((2, 7, 5, 5), 3, 4),
                                          ((2, 16, 8, 8), 32, 8), ((3, 64, 7, 7), 64, 4), ((2, 160, 5, 3), 256, 5)])
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
    corr = torch.empty((o,), dtype=torch.int64, device=DEV)
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


def test_zero_point_term_beyond_32_bits():
    """A range far from zero on every channel ([1000, 1001] at 4 bits: z = -15000) over 2048
    channels: the zero-point term of Eq. 3 needs more than 32 bits; fold and both kernels exact."""
    n, c, h, w, o = 2, 2048, 2, 4, 32
    g = torch.Generator(device=DEV).manual_seed(3)
    x = 1000.0 + torch.rand((n, c, h, w), generator=g, device=DEV)
    x[0, :, 0, 0] = 1000.0
    x[1, :, 1, 3] = 1001.0
    out = gpu_path(x, 4)
    assert np.all(out["zero_point"] <= -14000)
    wt = torch.ones(o, c, device=DEV)
    wt[1::2] = -1.0
    s = torch.from_numpy(out["scale"]).to(DEV)
    z = torch.from_numpy(out["zero_point"]).to(DEV)
    wq = torch.empty((o, c), dtype=torch.int8, device=DEV)
    corr = torch.empty((o,), dtype=torch.int64, device=DEV)
    a = torch.empty((o,), device=DEV)
    G.granq_fold_weights(wt, s, z, wq, corr, a)
    codes = torch.from_numpy(out["codes"]).to(DEV)
    ewq, ecorr, ea = oracle.fold_weights(wt.cpu().numpy(), out["scale"], out["zero_point"])
    torch.cuda.synchronize()
    assert np.array_equal(corr.cpu().numpy(), ecorr) and np.abs(ecorr).max() > 2 ** 31
    want = oracle.conv1x1_int8(out["codes"], ewq, ecorr, ea)
    for shape_ok in (True, False):                     # matrix-core kernel, then the plain one (misaligned y)
        ybuf = torch.full((n * o * h * w + 4,), float("nan"), device=DEV)
        y = (ybuf[:-4] if shape_ok else ybuf[1:-3]).view(n, o, h, w)
        G.granq_conv1x1_int8(codes, wq, corr, a, 4, y)
        torch.cuda.synchronize()
        assert np.array_equal(bits_view(y.cpu().numpy()), bits_view(want))


PACKED_SHAPES = [
    ((2, 16, 8, 8), 32), ((3, 64, 14, 14), 64), ((2, 32, 7, 12), 96), ((2, 1040, 2, 4), 96), ((70, 32, 1, 4), 32),
    ((3, 1024, 14, 14), 256), ((1, 144, 2, 6), 224), ((5, 272, 1, 4), 320),        # matrix cores
    ((2, 7, 5, 5), 3), ((1, 16, 7, 7), 32), ((1, 3, 3, 3), 2), ((1, 1, 1, 1), 1),     # plain kernel, odd counts
]


@pytest.mark.parametrize("bits", [1, 2, 3, 4])
@pytest.mark.parametrize("shape,o", PACKED_SHAPES, ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_packed_codes_forward_and_convolution(shape, o, bits):
    """Codes two per byte: the forward's packed output against the oracle's packing of the
    oracle's codes (with and without x_hat), and the convolution on them against the
    oracle's convolution on the unpacked codes, bit for bit, float32 and bfloat16 outputs."""
    n, c, h, w = shape
    x = workloads.make_activation(shape, "linear", (0.05, 20.0), 11, DEV)
    out = gpu_path(x, bits)
    s = torch.from_numpy(out["scale"]).to(DEV)
    z = torch.from_numpy(out["zero_point"]).to(DEV)
    nbytes = G.granq_packed4_bytes(G.desc_of(x))
    assert nbytes == (x.numel() + 1) // 2
    want_packed = oracle.pack4(out["codes"])
    for with_xhat in (True, False):
        packed = torch.full((nbytes,), 0xEE, dtype=torch.uint8, device=DEV)
        xh = torch.empty_like(x) if with_xhat else None
        G.granq_fakequant_fwd_packed4(x, s, z, bits, xh, packed)
        torch.cuda.synchronize()
        assert np.array_equal(packed.cpu().numpy(), want_packed), "packed codes differ (x_hat %s)" % with_xhat
        if with_xhat:
            assert np.array_equal(xh.cpu().numpy(), out["xhat"])
    g = torch.Generator(device=DEV).manual_seed(5)
    wt = torch.randn(o, c, generator=g, device=DEV)
    wq = torch.empty((o, c), dtype=torch.int8, device=DEV)
    corr = torch.empty((o,), dtype=torch.int64, device=DEV)
    a = torch.empty((o,), device=DEV)
    G.granq_fold_weights(wt, s, z, wq, corr, a)
    torch.cuda.synchronize()
    codes_again = oracle.unpack4(want_packed, x.numel()).reshape(shape)
    assert np.array_equal(codes_again, out["codes"])
    want = oracle.conv1x1_int8(codes_again, wq.cpu().numpy(), corr.cpu().numpy(), a.cpu().numpy())
    y = torch.full((n, o, h, w), float("nan"), device=DEV)
    G.granq_conv1x1_int8_packed4(packed, shape, wq, corr, a, bits, y)
    y16 = torch.empty((n, o, h, w), dtype=torch.bfloat16, device=DEV)
    G.granq_conv1x1_int8_packed4(packed, shape, wq, corr, a, bits, y16)
    torch.cuda.synchronize()
    assert np.array_equal(bits_view(y.cpu().numpy()), bits_view(want))
    want16 = torch.from_numpy(want).to(torch.bfloat16)
    assert torch.equal(y16.cpu().view(torch.int16), want16.view(torch.int16))


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16], ids=["bf16", "f16"])
def test_packed_codes_from_16_bit_tensors(dtype):
    for shape in [(4, 24, 14, 14), (3, 10, 7, 7), (2, 3, 3, 3)]:
        x = workloads.make_activation(shape, "relu", (0.05, 20.0), 2, DEV, dtype)
        out = gpu_path(x, 3)
        s = torch.from_numpy(out["scale"]).to(DEV)
        z = torch.from_numpy(out["zero_point"]).to(DEV)
        packed = torch.full(((x.numel() + 1) // 2,), 0xEE, dtype=torch.uint8, device=DEV)
        xh = torch.empty_like(x)
        G.granq_fakequant_fwd_packed4(x, s, z, 3, xh, packed)
        torch.cuda.synchronize()
        assert np.array_equal(packed.cpu().numpy(), oracle.pack4(out["codes"]))
        assert np.array_equal(to_numpy(xh), out["xhat"])


def test_packed_codes_argument_checks():
    import ctypes
    lib = G.load()
    d = G.make_desc(2, 16, 4, 4, 0)
    assert lib.granq_fakequant_fwd_packed4(16, ctypes.byref(d), 16, 16, 5, 16, 16, 0) == G.GRANQ_ERR_INVALID_ARG
    assert lib.granq_fakequant_fwd_packed4(16, ctypes.byref(d), 16, 16, 4, 16, 0, 0) == G.GRANQ_ERR_INVALID_ARG
    assert lib.granq_conv1x1_int8_packed4(16, ctypes.byref(d), 32, 16, 16, 16, 5, 0, 16, 0) == G.GRANQ_ERR_INVALID_ARG
    assert G.granq_packed4_bytes(G.make_desc(1, 1, 1, 9, 0)) == 5


@pytest.mark.parametrize("c,o,hw", [(1024, 256, 14), (2048, 512, 7), (64, 256, 56)])
def test_conv_at_benchmark_size_on_sampled_outputs(c, o, hw):
    """The shapes and the batch that bench.py times (a launch of the same configuration): 4096 sampled
    outputs, each recomputed from the definition in exact integer arithmetic (the oracle's expression,
    one output at a time), must match bit for bit; the packed form must give the same tensor."""
    n, bits = 256, 4
    g = torch.Generator(device=DEV).manual_seed(c + o)
    codes = torch.randint(0, 1 << bits, (n, c, hw, hw), dtype=torch.uint8, generator=g, device=DEV)
    wq = torch.randint(-127, 128, (o, c), dtype=torch.int8, generator=g, device=DEV)
    corr = torch.randint(-(1 << 20), 1 << 20, (o,), dtype=torch.int64, generator=g, device=DEV)
    a = torch.rand(o, generator=g, device=DEV) * 0.01 + 1e-4
    y = torch.full((n, o, hw, hw), float("nan"), device=DEV)
    G.granq_conv1x1_int8(codes, wq, corr, a, bits, y)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    idx_n = rng.integers(0, n, 4096)
    idx_o = rng.integers(0, o, 4096)
    idx_k = rng.integers(0, hw * hw, 4096)
    # always among the samples: the corners and a sample's last pixel (the ragged group of a 7 x 7 map)
    idx_n[:4], idx_o[:4], idx_k[:4] = [0, n - 1, 0, n - 1], [0, o - 1, o - 1, 0], [0, hw * hw - 1, hw * hw - 1, 0]
    cn = codes.view(n, c, hw * hw)[torch.from_numpy(idx_n).to(DEV), :, torch.from_numpy(idx_k).to(DEV)].cpu().numpy().astype(np.int64)
    wn = wq.cpu().numpy().astype(np.int64)[idx_o]
    acc = (cn * wn).sum(axis=1) - corr.cpu().numpy()[idx_o]
    want = a.cpu().numpy()[idx_o] * acc.astype(np.float32)          # one conversion, one product: as the oracle
    got = y.view(n, o, hw * hw).cpu().numpy()[idx_n, idx_o, idx_k]
    assert np.array_equal(bits_view(got), bits_view(want.astype(np.float32)))
    assert not torch.isnan(y).any()
    if (hw * hw) % 4 == 0:
        packed = torch.from_numpy(oracle.pack4(codes.cpu().numpy())).to(DEV)
        y2 = torch.full((n, o, hw, hw), float("nan"), device=DEV)
        G.granq_conv1x1_int8_packed4(packed, (n, c, hw, hw), wq, corr, a, bits, y2)
        torch.cuda.synchronize()
        assert torch.equal(y, y2)
