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
