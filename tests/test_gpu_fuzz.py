"""Seeded random shapes, dtypes, bit-widths, value laws and pointer offsets through every entry
point of the four-call path and the gate-bit pair, element by element against the oracle
(needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_18339_amd as G
import workloads
from parity import assert_parity, bits_view, gpu_path, oracle_path, to_numpy

pytestmark = pytest.mark.gpu
DEV = "cuda"
LAWS = ("relu", "relu6", "linear", "laplace")


def _cases(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        kind = rng.integers(0, 4)
        if kind == 0:        # many channels, tiny maps
            shape = (int(rng.integers(1, 40)), int(rng.integers(1, 300)), int(rng.integers(1, 4)), int(rng.integers(1, 4)))
        elif kind == 1:      # few channels, larger maps
            shape = (int(rng.integers(1, 12)), int(rng.integers(1, 9)), int(rng.integers(1, 40)), int(rng.integers(1, 40)))
        elif kind == 2:      # multiples of the vector width
            shape = (int(rng.integers(1, 20)), int(rng.integers(1, 64)), int(rng.integers(1, 8)) * 2, int(rng.integers(1, 8)) * 4)
        else:                # anything
            shape = tuple(int(v) for v in rng.integers(1, 24, size=4))
        out.append((shape, LAWS[int(rng.integers(0, 4))], int(rng.integers(1, 9)),
                    (torch.float32, torch.bfloat16, torch.float16)[int(rng.integers(0, 3))], int(rng.integers(0, 3))))
    return out


@pytest.mark.parametrize("chunk", range(6))
def test_random_cases(chunk):
    for i, (shape, law, bits, dtype, offset) in enumerate(_cases(1000 + chunk, 30)):
        n_el = int(np.prod(shape))
                # offset 0: aligned allocation; 1, 2: start `offset` elements into a larger buffer
        buf = torch.zeros(n_el + 16, dtype=dtype, device=DEV)
        gbuf = torch.zeros(n_el + 16, dtype=dtype, device=DEV)
        x = buf[offset:offset + n_el].view(shape)
        dy = gbuf[offset:offset + n_el].view(shape)
        x.copy_(workloads.make_activation(shape, law, (0.05, 20.0), seed=chunk * 100 + i, device=DEV, dtype=dtype))
        dy.copy_(workloads.make_grad(shape, chunk * 100 + i, DEV, dtype))
        what = "%s %s b%d %s +%d" % (shape, law, bits, str(dtype)[6:], offset)
        got = gpu_path(x, bits, dy)
        x_np, dy_np = to_numpy(x), to_numpy(dy)
        want = oracle_path(x_np, bits, dy_np)
        assert_parity(got, want, what)
        # gate-bit pair with the same parameters
        s = torch.from_numpy(got["scale"]).to(DEV)
        z = torch.from_numpy(got["zero_point"]).to(DEV)
        mask = torch.full(((n_el + 7) // 8,), 0x5A, dtype=torch.uint8, device=DEV)
        xh = torch.empty_like(x)
        dx = torch.empty_like(x)
        G.granq_fakequant_fwd_mask(x, s, z, bits, xh, mask)
        G.granq_fakequant_bwd_mask(dy, mask, dx)
        torch.cuda.synchronize()
        assert np.array_equal(mask.cpu().numpy(), oracle.gate_mask(x_np, got["scale"], got["zero_point"], bits)), what
        assert np.array_equal(bits_view(to_numpy(dx)), bits_view(want["dx"])), what
        assert np.array_equal(bits_view(to_numpy(xh)), bits_view(got["xhat"])), what


def _conv_cases(seed, count):
    """Random consumer shapes: channel counts that hit and miss the matrix-core conditions (C % 16,
    C % 8, O % 32), maps that are and are not multiples of 4, the many-channel variant, pointer offsets."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        c = int(rng.choice([8, 16, 24, 48, 64, 128, 144, 272, 7, 20]))
        o = int(rng.choice([32, 64, 96, 192, 224, 320, 3, 40]))
        h, w = int(rng.integers(1, 9)), int(rng.integers(1, 9))
        n = int(rng.integers(1, 12))
        out.append(((n, c, h, w), o, int(rng.integers(1, 8)), int(rng.integers(0, 4)),
                    (torch.float32, torch.bfloat16, torch.float16)[int(rng.integers(0, 3))]))
    return out


@pytest.mark.parametrize("chunk", range(3))
def test_random_consumer_cases(chunk):
    """The integer convolution (bit for bit), its packed form and the float convolution (within its
    bound) on seeded random shapes."""
    for i, (shape, o, bits, offset, ydtype) in enumerate(_conv_cases(2000 + chunk, 24)):
        n, c, h, w = shape
        what = "%s -> %d b%d +%d %s" % (shape, o, bits, offset, str(ydtype)[6:])
        x = workloads.make_activation(shape, LAWS[i % 4], (0.05, 20.0), seed=chunk * 50 + i, device=DEV)
        got = gpu_path(x, bits)
        g = torch.Generator(device=DEV).manual_seed(chunk * 50 + i)
        wt = torch.randn(o, c, generator=g, device=DEV) * torch.exp(torch.randn(o, 1, generator=g, device=DEV))
        s = torch.from_numpy(got["scale"]).to(DEV)
        z = torch.from_numpy(got["zero_point"]).to(DEV)
        wq = torch.empty((o, c), dtype=torch.int8, device=DEV)
        corr = torch.empty((o,), dtype=torch.int64, device=DEV)
        a = torch.empty((o,), device=DEV)
        G.granq_fold_weights(wt, s, z, wq, corr, a)
        n_el, n_out = n * c * h * w, n * o * h * w
        cbuf = torch.zeros(n_el + 8, dtype=torch.uint8, device=DEV)
        codes = cbuf[offset:offset + n_el].view(shape)
        codes.copy_(torch.from_numpy(got["codes"]).to(DEV))
        ybuf = torch.full((n_out + 8,), float("nan"), device=DEV)
        y = ybuf[offset:offset + n_out].view(n, o, h, w)
        G.granq_conv1x1_int8(codes, wq, corr, a, bits, y)
        torch.cuda.synchronize()
        want = oracle.conv1x1_int8(got["codes"], wq.cpu().numpy(), corr.cpu().numpy(), a.cpu().numpy())
        assert np.array_equal(bits_view(y.cpu().numpy()), bits_view(want)), what
        assert torch.isnan(ybuf[:offset]).all() and torch.isnan(ybuf[offset + n_out:]).all(), what
        if bits <= 4:
            packed = torch.from_numpy(oracle.pack4(got["codes"])).to(DEV)
            y2 = torch.full((n, o, h, w), float("nan"), device=DEV)
            G.granq_conv1x1_int8_packed4(packed, shape, wq, corr, a, bits, y2)
            torch.cuda.synchronize()
            assert np.array_equal(bits_view(y2.cpu().numpy()), bits_view(want)), what
        # the float form on x_hat in a random storage type
        xh = torch.from_numpy(got["xhat"]).to(DEV).to(ydtype)
        wf = wt.to(ydtype)
        yf = torch.full((n, o, h, w), float("nan"), dtype=ydtype, device=DEV)
        G.granq_conv1x1_float(xh, wf, yf)
        torch.cuda.synchronize()
        xa, wa = to_numpy(xh), to_numpy(wf)
        exact = oracle.conv1x1_float(xa, wa)
        from parity import values
        mag = np.einsum("oc,nchw->nohw", np.abs(values(wa)).astype(np.float64), np.abs(values(xa)).astype(np.float64))
        half_ulp = {torch.float32: 0.0, torch.bfloat16: 2.0 ** -8, torch.float16: 2.0 ** -11}[ydtype]
        tol = (c + 2) * 2.0 ** -24 * mag + half_ulp * 1.0001 * np.abs(exact) + 2.0 ** -25
        gotf = values(to_numpy(yf)).astype(np.float64)
        assert np.all(np.abs(gotf - exact) <= tol), what
