"""Fused distortion metrics (cosine similarity, relative error: the paper's Table 2)
against the binary64 oracle (needs an MI355X).

Tolerance: both sides form every product and difference in binary64 from the same
binary32 values; only the order of the binary64 additions differs.  With at most
n = 3.3e6 non-negative terms per channel the worst-case relative error of either
summation is n * 2^-53 = 3.7e-10, so sums must agree to 1e-9 relative (observed:
about 1e-14); x.q may have mixed signs, so it is compared against the scale
sqrt(x.x * q.q)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_18339_amd as G
import workloads
from parity import to_numpy

pytestmark = pytest.mark.gpu
DEV = "cuda"
RTOL = 1e-9


def _gpu_distortion(x, s, z, bits, desc=None):
    d = desc or G.desc_of(x)
    ch = torch.full((d.c, 4), float("nan"), dtype=torch.float64, device=DEV)
    layer = torch.full((6,), float("nan"), dtype=torch.float64, device=DEV)
    ws = torch.empty(max(16, G.granq_distortion_workspace_bytes(d)), dtype=torch.uint8, device=DEV)
    G.granq_distortion(x, s, z, bits, ch, layer, ws, desc=d)
    torch.cuda.synchronize()
    return ch.cpu().numpy(), layer.cpu().numpy()


def _compare(ch, layer, want_ch, want_layer):
    scale = np.sqrt(want_ch[:, 1] * want_ch[:, 2])
    assert np.all(np.abs(ch[:, 0] - want_ch[:, 0]) <= RTOL * np.maximum(scale, 1e-300))
    for j in (1, 2, 3):
        assert np.all(np.abs(ch[:, j] - want_ch[:, j]) <= RTOL * want_ch[:, j])
    lscale = np.sqrt(want_layer[1] * want_layer[2])
    assert abs(layer[0] - want_layer[0]) <= RTOL * lscale
    for j in (1, 2, 3):
        assert abs(layer[j] - want_layer[j]) <= RTOL * want_layer[j]
    assert abs(layer[4] - want_layer[4]) <= 2 * RTOL
    assert abs(layer[5] - want_layer[5]) <= 2 * RTOL * max(want_layer[5], 1e-300)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16], ids=["f32", "bf16", "f16"])
@pytest.mark.parametrize("shape,law,bits", [((8, 16, 32, 32), "relu", 3), ((5, 37, 9, 8), "linear", 4),
                                            ((6, 100, 7, 7), "laplace", 5), ((3, 40, 1, 1), "linear", 8),
                                            ((2, 3, 7, 7), "relu", 3), ((64, 64, 56, 56), "relu", 4),
                                            ((1, 1, 1, 5), "linear", 2)])
def test_distortion_matches_oracle(shape, law, bits, dtype):
    x = workloads.make_activation(shape, law, (0.05, 20.0), 3, DEV, dtype)
    q = G.ActivationQuantizer(shape, dtype, bits, DEV)
    q.calibrate(x)
    ch, layer = _gpu_distortion(x, q.scale, q.zero_point, bits)
    want_ch, want_layer = oracle.distortion(to_numpy(x), q.scale.cpu().numpy(), q.zero_point.cpu().numpy(), bits)
    _compare(ch, layer, want_ch, want_layer)
    assert 0 <= layer[5] < 1.5 and layer[4] <= 1 + 1e-12
    # deterministic: a second run gives the same bits
    ch2, layer2 = _gpu_distortion(x, q.scale, q.zero_point, bits)
    assert np.array_equal(ch, ch2) and np.array_equal(layer, layer2)


def test_channelwise_distorts_less_than_layerwise():
    """Direction of Table 2 on a tensor with very different channel spreads."""
    shape = (64, 64, 56, 56)
    x = workloads.make_activation(shape, "relu", (0.05, 20.0), 1, DEV)
    qc = G.ActivationQuantizer(shape, torch.float32, 3, DEV, view="channel")
    ql = G.ActivationQuantizer(shape, torch.float32, 3, DEV, view="layer")
    qc.calibrate(x)
    ql.calibrate(x)
    _, lay_c = _gpu_distortion(x, qc.scale, qc.zero_point, 3, qc.desc)
    _, lay_l = _gpu_distortion(x, ql.scale, ql.zero_point, 3, ql.desc)
    assert lay_c[4] > lay_l[4] and lay_c[5] < lay_l[5]


def test_distortion_argument_checks():
    import ctypes
    lib = G.load()
    d = G.make_desc(2, 3, 4, 4, G.GRANQ_F32)
    need = G.granq_distortion_workspace_bytes(d)
    assert need >= 3 * 4 * 8
    assert lib.granq_distortion(16, ctypes.byref(d), 16, 16, 4, 16, 16, 16, need - 1, 0) == G.GRANQ_ERR_WORKSPACE
    assert lib.granq_distortion(16, ctypes.byref(d), 16, 16, 0, 16, 16, 16, need, 0) == G.GRANQ_ERR_INVALID_ARG
    assert lib.granq_distortion(16, ctypes.byref(d), 16, 16, 4, 0, 16, 16, need, 0) == G.GRANQ_ERR_INVALID_ARG
    assert lib.granq_distortion(16, ctypes.byref(d), 16, 16, 4, 12, 16, 16, need, 0) == G.GRANQ_ERR_UNSUPPORTED
