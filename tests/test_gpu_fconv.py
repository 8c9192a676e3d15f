"""Floating-point 1x1 convolution over the pre-scaled activations (Eq. 6's accumulation with a
full weight matrix) against the oracle's binary64 sums (needs an MI355X).

Tolerance, from the arithmetic: the kernels form binary32 products and add them in binary32 in
an order of their own, so |y - exact| <= (C + 2) * 2^-24 * sum_c |w x_hat| (C - 1 additions and
one product rounding per term, first order); a 16-bit result is rounded once more, by half a unit
in the last place of its type.  Operands here are far from the ends of the binary32 range.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_18339_amd as G
import workloads
from parity import gpu_path, to_numpy, values

pytestmark = pytest.mark.gpu
DEV = "cuda"
TORCH = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}
HALF_ULP = {"f32": 0.0, "bf16": 2.0 ** -8, "f16": 2.0 ** -11}   # half a unit in the last place, relative, at most


def _weights(o, c, dtype, seed):
    g = torch.Generator(device=DEV).manual_seed(seed)
    w = torch.randn(o, c, generator=g, device=DEV) * torch.exp(0.5 * torch.randn(o, 1, generator=g, device=DEV))
    return w.to(dtype).contiguous()


def _check(xh: torch.Tensor, w: torch.Tensor, name: str):
    n, c, h, wd = xh.shape
    o = w.shape[0]
    y = torch.full((n, o, h, wd), float("nan"), dtype=xh.dtype, device=DEV)
    G.granq_conv1x1_float(xh, w, y)
    torch.cuda.synchronize()
    xa, wa = to_numpy(xh), to_numpy(w)
    want = oracle.conv1x1_float(xa, wa)
    mag = np.einsum("oc,nchw->nohw", np.abs(values(wa)).astype(np.float64), np.abs(values(xa)).astype(np.float64))
    got = values(to_numpy(y)).astype(np.float64)
    assert np.all(np.isfinite(got))
    tol = (c + 2) * 2.0 ** -24 * mag + HALF_ULP[name] * 1.0001 * np.abs(want) + 2.0 ** -100
    if name == "f16":
        tol = tol + 2.0 ** -25                      # half a step of the subnormal range
    bad = np.nonzero((np.abs(got - want) > tol).ravel())[0]
    assert bad.size == 0, "y off at %d of %d, first flat index %d: got %r want %r" % (
        bad.size, got.size, bad[0], got.ravel()[bad[0]], want.ravel()[bad[0]])
    return got, want, mag


def _xhat(shape, bits, name, seed=0):
    """Pre-scaled activations as the library's own forward leaves them."""
    x = workloads.make_activation(shape, "linear", (0.05, 20.0), seed, DEV).to(TORCH[name])
    q = G.ActivationQuantizer(shape, TORCH[name], bits, DEV)
    xh = torch.empty_like(x)
    q.forward(x, xh, None, torch.cuda.current_stream())
    torch.cuda.synchronize()
    return xh


# matrix-core path: C % 8 == 0, O % 32 == 0; several tiles, a ragged last tile, tiles that span
# samples, a second row tile past O, many sweeps of output channels
MFMA_SHAPES = [
    ((2, 16, 8, 8), 32), ((3, 64, 14, 14), 64), ((2, 32, 7, 12), 96), ((1, 128, 28, 28), 160),
    ((4, 48, 2, 2), 32), ((70, 8, 1, 4), 32), ((2, 256, 14, 14), 256), ((1, 24, 23, 12), 320),
]
# the same with H*W no multiple of 4: element-aligned accesses, short last group per sample
RAGGED_SHAPES = [
    ((1, 16, 7, 7), 32), ((3, 64, 7, 7), 64), ((2, 64, 5, 5), 96), ((1, 32, 3, 2), 32),
    ((2, 16, 9, 7), 64), ((37, 48, 1, 5), 32), ((2, 512, 7, 7), 128),
]
# anything else: one thread per output
PLAIN_SHAPES = [((2, 7, 5, 5), 3), ((1, 16, 1, 3), 32), ((2, 24, 4, 4), 40), ((2, 20, 4, 4), 32), ((1, 1, 1, 1), 1)]


@pytest.mark.parametrize("name", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("shape,o", MFMA_SHAPES + RAGGED_SHAPES + PLAIN_SHAPES)
def test_float_conv_against_the_oracle(shape, o, name):
    xh = _xhat(shape, 4, name, seed=len(shape) + o)
    w = _weights(o, shape[1], TORCH[name], seed=o)
    _check(xh, w, name)


def test_float_conv_exact_cases():
    """Identity and permutation weights return the channels themselves, bit for bit; small integers
    and powers of two give sums without any rounding."""
    shape = (3, 32, 6, 6)
    xh = _xhat(shape, 4, "f32", seed=7)
    eye = torch.eye(32, device=DEV)
    y = torch.empty_like(xh)
    G.granq_conv1x1_float(xh, eye, y)
    torch.cuda.synchronize()
    assert torch.equal(y, xh)
    perm = torch.randperm(32, generator=torch.Generator().manual_seed(1)).to(DEV)
    G.granq_conv1x1_float(xh, eye[perm].contiguous(), y)
    torch.cuda.synchronize()
    assert torch.equal(y, xh[:, perm])
    g = torch.Generator(device=DEV).manual_seed(3)
    xi = torch.randint(-64, 64, (2, 40, 4, 8), generator=g, device=DEV).float() / 8
    wi = torch.randint(-32, 32, (64, 40), generator=g, device=DEV).float() / 4
    yi = torch.empty(2, 64, 4, 8, device=DEV)
    G.granq_conv1x1_float(xi, wi, yi)
    torch.cuda.synchronize()
    want = oracle.conv1x1_float(xi.cpu().numpy(), wi.cpu().numpy())
    assert np.array_equal(yi.cpu().numpy().astype(np.float64), want)


def test_float_conv_beside_the_integer_form():
    """Eq. 6 in floating point and Eq. 3 folded into integers on the same tensor: they differ by
    the rounding of the folded weights only."""
    shape, o, bits = (2, 64, 14, 14), 64, 4
    x = workloads.make_activation(shape, "linear", (0.05, 20.0), 3, DEV)
    out = gpu_path(x, bits)
    xh = torch.from_numpy(out["xhat"]).to(DEV)
    w = _weights(o, 64, torch.float32, seed=5)
    yf, want, mag = _check(xh, w, "f32")
    s = torch.from_numpy(out["scale"]).to(DEV)
    z = torch.from_numpy(out["zero_point"]).to(DEV)
    wq = torch.empty((o, 64), dtype=torch.int8, device=DEV)
    corr = torch.empty((o,), dtype=torch.int64, device=DEV)
    a = torch.empty((o,), device=DEV)
    G.granq_fold_weights(w, s, z, wq, corr, a)
    yi = torch.empty(2, o, 14, 14, device=DEV)
    G.granq_conv1x1_int8(torch.from_numpy(out["codes"]).to(DEV), wq, corr, a, bits, yi)
    torch.cuda.synchronize()
    bound = 0.5 * a.cpu().numpy().astype(np.float64).reshape(1, -1, 1, 1) * np.abs(
        out["codes"].astype(np.float64) - out["zero_point"].reshape(1, -1, 1, 1)).sum(axis=1, keepdims=True)
    assert np.all(np.abs(yi.cpu().numpy() - yf) <= bound * (1 + 1e-4) + 1e-5 * np.abs(yf).max())


def test_float_conv_unaligned_pointers_and_argument_checks():
    import ctypes
    shape, o = (3, 16, 7, 7), 32
    xh = _xhat(shape, 4, "f32", seed=2)
    w = _weights(o, 16, torch.float32, seed=2)
    want = oracle.conv1x1_float(xh.cpu().numpy(), w.cpu().numpy())
    n, c, h, wd = shape
    for shift in (1, 3):
        xbuf = torch.zeros(xh.numel() + 8, device=DEV)
        xs = xbuf[shift:shift + xh.numel()].view(shape)
        xs.copy_(xh)
        ybuf = torch.full((n * o * h * wd + 8,), float("nan"), device=DEV)
        y = ybuf[shift:shift + n * o * h * wd].view(n, o, h, wd)
        G.granq_conv1x1_float(xs, w, y)
        torch.cuda.synchronize()
        mag = np.einsum("oc,nchw->nohw", np.abs(w.cpu().numpy()).astype(np.float64), np.abs(xh.cpu().numpy()).astype(np.float64))
        assert np.all(np.abs(y.cpu().numpy() - want) <= (c + 2) * 2.0 ** -24 * mag + 2.0 ** -100)
        assert torch.isnan(ybuf[:shift]).all() and torch.isnan(ybuf[shift + n * o * h * wd:]).all()
    lib = G.load()
    d = G.make_desc(2, 16, 4, 4, 0)
    assert lib.granq_conv1x1_float(0, ctypes.byref(d), 32, 16, 16, 0) == G.GRANQ_ERR_INVALID_ARG
    assert lib.granq_conv1x1_float(16, ctypes.byref(d), 0, 16, 16, 0) == G.GRANQ_ERR_INVALID_ARG
    assert lib.granq_conv1x1_float(18, ctypes.byref(d), 32, 16, 16, 0) == G.GRANQ_ERR_UNSUPPORTED
    bad = G.make_desc(2, 16, 4, 4, 7)
    assert lib.granq_conv1x1_float(16, ctypes.byref(bad), 32, 16, 16, 0) == G.GRANQ_ERR_INVALID_ARG


@pytest.mark.parametrize("name", ["f32", "bf16"])
@pytest.mark.parametrize("c,o,hw", [(1024, 256, 14), (2048, 512, 7), (64, 64, 56)])
def test_float_conv_at_benchmark_size_on_sampled_outputs(c, o, hw, name):
    """The shapes and the batch that bench.py times: 4096 sampled outputs, each recomputed from the
    definition in binary64, within the bound of this file's header."""
    n = 256
    g = torch.Generator(device=DEV).manual_seed(c + o + 1)
    xh = (torch.randn(n, c, hw, hw, generator=g, device=DEV) * 3).to(TORCH[name])
    w = _weights(o, c, TORCH[name], seed=c)
    y = torch.full((n, o, hw, hw), float("nan"), dtype=TORCH[name], device=DEV)
    G.granq_conv1x1_float(xh, w, y)
    torch.cuda.synchronize()
    rng = np.random.default_rng(6)
    idx_n, idx_o, idx_k = rng.integers(0, n, 4096), rng.integers(0, o, 4096), rng.integers(0, hw * hw, 4096)
    idx_n[:4], idx_o[:4], idx_k[:4] = [0, n - 1, 0, n - 1], [0, o - 1, o - 1, 0], [0, hw * hw - 1, hw * hw - 1, 0]
    tn, tk, to = (torch.from_numpy(v).to(DEV) for v in (idx_n, idx_k, idx_o))
    xs = xh.view(n, c, hw * hw)[tn, :, tk].double().cpu().numpy()
    ws = w[to].double().cpu().numpy()
    want = (xs * ws).sum(axis=1)
    mag = (np.abs(xs) * np.abs(ws)).sum(axis=1)
    got = y.view(n, o, hw * hw)[tn, to, tk].double().cpu().numpy()
    tol = (c + 2) * 2.0 ** -24 * mag + HALF_ULP[name] * 1.0001 * np.abs(want) + 2.0 ** -100
    assert np.all(np.abs(got - want) <= tol)
    assert not torch.isnan(y.float()).any()
