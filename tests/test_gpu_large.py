"""Tensors with more than 2^31 elements, and rows of 2^31 elements or more: 64-bit indexing in
every kernel family, against the oracle on every element (needs an MI355X and ~40 GB of host RAM)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_18339_amd as G
from parity import assert_parity, gpu_path, oracle_path, to_numpy

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _fill(shape, dtype, seed):
    """|N(0, sigma_c)| with a few planted extremes far from the start of the tensor."""
    g = torch.Generator(device=DEV).manual_seed(seed)
    x = torch.empty(shape, dtype=dtype, device=DEV)
    c = shape[1]
    sig = torch.exp(torch.rand(c, generator=g, device=DEV) * 6 - 3).view(1, c, 1, 1)
    for n in range(shape[0]):
        x[n:n + 1] = (torch.randn((1,) + tuple(shape[1:]), generator=g, device=DEV).abs_() * sig).to(dtype)
    return x


def _check_all(x, dy, bits, what):
    """Ranges, scale and zero-point, then x_hat / codes / dx of every element (the oracle's
    element-wise passes are split over the batch across host threads)."""
    got = gpu_path(x, bits, dy)
    x_np = to_numpy(x)
    mn, mx = oracle.range_reduce(x_np)
    s, z = oracle.prescale(mn, mx, bits)
    assert np.array_equal(got["min"], mn) and np.array_equal(got["max"], mx), what
    assert np.array_equal(got["scale"], s) and np.array_equal(got["zero_point"], z), what
    want = oracle_path(x_np, bits, to_numpy(dy), scale=s, zero_point=z)
    assert_parity({k: got[k] for k in ("scale", "zero_point", "xhat", "codes", "dx")}, want, what)


def test_more_than_2_to_31_elements_bf16():
    shape = (33, 16, 2048, 2048)                       # 2.21e9 elements, 4.4 GB per tensor
    assert np.prod(shape) > 2 ** 31
    x = _fill(shape, torch.bfloat16, 1)
    x[32, 15, 2047, 2040:] = 77.0                      # the maximum of the last channel sits at the very end
    x[32, 0, 2047, 2047] = 0.0
    dy = torch.empty_like(x)
    g = torch.Generator(device=DEV).manual_seed(2)
    for n in range(shape[0]):
        dy[n:n + 1] = torch.randn((1,) + shape[1:], generator=g, device=DEV).to(torch.bfloat16)
    _check_all(x, dy, 4, "2.2e9 elements bf16")


def test_rows_longer_than_2_to_31_take_the_elementwise_kernels():
    hw = 2 ** 30 + 8
    shape = (1, 2, 1, hw)                              # C*H*W = 2^31 + 16 elements per row
    pl = G.granq_plan_describe(G.make_desc(*shape, G.GRANQ_BF16))
    assert not pl["vector_path"]
    x = _fill(shape, torch.bfloat16, 3)
    x[0, 1, 0, hw - 1] = 55.0
    dy = torch.ones_like(x)
    _check_all(x, dy, 3, "row of 2^31+16 elements")
