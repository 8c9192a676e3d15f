"""Gate-bit forward / backward pair against the oracle and against the x-based pair (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_18339_amd as G
import workloads
from parity import bits_view, gpu_path, to_numpy

pytestmark = pytest.mark.gpu
DEV = "cuda"

SHAPES = [
    (8, 16, 32, 32), (5, 37, 9, 8), (6, 104, 7, 7), (3, 40, 1, 1), (9, 24, 14, 14), (4, 3000, 1, 1),
    (1, 1, 1, 16384), (1, 64, 1, 1152), (140001, 2, 2, 2), (1, 2048, 7, 7), (17, 520, 2, 2), (4, 4, 64, 66), (1, 8, 1, 1),
    # rows that are not a multiple of eight elements, or no 16-byte structure: byte-wise kernels
    (6, 100, 7, 7), (4, 9, 2, 2), (2, 3, 7, 7), (5, 7, 3, 3), (1, 1, 1, 5), (1, 1, 1, 1), (3, 1, 7, 3),
    (1, 1, 1, 4), (2, 1, 5, 4),
]


def _run_mask_pair(x, dy, s, z, bits, desc=None):
    d = desc or G.desc_of(x)
    nbytes = G.granq_mask_bytes(d)
    assert nbytes == (x.numel() + 7) // 8
    mask = torch.full((nbytes,), 0xA5, dtype=torch.uint8, device=x.device)
    x_hat = torch.empty_like(x)
    dx = torch.empty_like(x)
    G.granq_fakequant_fwd_mask(x, s, z, bits, x_hat, mask, desc=d)
    G.granq_fakequant_bwd_mask(dy, mask, dx, desc=d)
    torch.cuda.synchronize()
    return to_numpy(x_hat), mask.cpu().numpy(), to_numpy(dx)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16], ids=["f32", "bf16", "f16"])
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_mask_pair_small_shapes(shape, dtype):
    for i, (law, bits) in enumerate([("linear", 4), ("relu", 3)]):
        x = workloads.make_activation(shape, law, (0.05, 20.0), seed=i, device=DEV, dtype=dtype)
        dy = workloads.make_grad(shape, i, DEV, dtype)
        ref = gpu_path(x, bits, dy)                         # x-based pair (itself checked elsewhere)
        # stale ranges from a narrower tensor so that both clamp sides occur
        s_np = ref["scale"] * np.float32(0.5 if law == "linear" else 1.0)
        s = torch.from_numpy(s_np).to(DEV)
        z = torch.from_numpy(ref["zero_point"]).to(DEV)
        x_hat, mask, dx = _run_mask_pair(x, dy, s, z, bits)
        x_np, dy_np = to_numpy(x), to_numpy(dy)
        want_hat, _ = oracle.fakequant_fwd(x_np, s_np, ref["zero_point"], bits)
        want_mask = oracle.gate_mask(x_np, s_np, ref["zero_point"], bits)
        want_dx = oracle.fakequant_bwd(x_np, dy_np, s_np, ref["zero_point"], bits)
        assert np.array_equal(mask, want_mask), "gate bits differ %s" % (shape,)
        from parity import values
        assert np.array_equal(values(x_hat), values(want_hat))
        assert np.array_equal(bits_view(dx), bits_view(want_dx))
        assert np.array_equal(bits_view(oracle.bwd_from_mask(dy_np, want_mask)), bits_view(want_dx))
        if law == "linear" and x.numel() > 64:
            assert 0 < np.unpackbits(mask, bitorder="little")[:x.numel()].mean() < 1


def test_mask_pair_in_place_and_unaligned():
    shape = (4, 16, 14, 14)
    x = workloads.make_activation(shape, "linear", (0.05, 20.0), seed=3, device=DEV)
    dy = workloads.make_grad(shape, 3, DEV)
    ref = gpu_path(x, 4, dy)
    s = torch.from_numpy(ref["scale"]).to(DEV)
    z = torch.from_numpy(ref["zero_point"]).to(DEV)
    mask = torch.zeros(G.granq_mask_bytes(G.desc_of(x)), dtype=torch.uint8, device=DEV)
    x2, dy2 = x.clone(), dy.clone()
    G.granq_fakequant_fwd_mask(x2, s, z, 4, x2, mask)      # x_hat aliases x
    G.granq_fakequant_bwd_mask(dy2, mask, dy2)             # dx aliases dy
    torch.cuda.synchronize()
    assert np.array_equal(x2.cpu().numpy(), ref["xhat"])
    assert np.array_equal(dy2.cpu().numpy(), ref["dx"])
    # tensors that start 4 bytes into an allocation take the byte-wise kernels
    n = x.numel()
    xb = torch.zeros(n + 8, device=DEV)
    gb = torch.zeros(n + 8, device=DEV)
    xo, go = xb[1:1 + n].view(shape), gb[1:1 + n].view(shape)
    xo.copy_(x)
    go.copy_(dy)
    x_hat, m2, dx = _run_mask_pair(xo, go, s, z, 4)
    assert np.array_equal(x_hat, ref["xhat"]) and np.array_equal(dx, ref["dx"])
    assert np.array_equal(m2, mask.cpu().numpy())


@pytest.mark.parametrize("idx,dtype", [(0, "f32"), (0, "bf16"), (3, "bf16"), (4, "f32")])
def test_mask_pair_full_size(idx, dtype):
    wl = workloads.resnet18_imagenet()
    a = wl.acts[idx]
    shape = a.shape(wl.batch)
    x = workloads.make_activation(shape, a.law, wl.sigma, idx, DEV, workloads.torch_dtype(dtype))
    dy = workloads.make_grad(shape, idx, DEV, x.dtype)
    q = G.ActivationQuantizer(shape, x.dtype, 4, DEV)
    q.calibrate(x)
    x_hat, mask, dx = _run_mask_pair(x, dy, q.scale, q.zero_point, 4)
    # every element of every output against the oracle (its element-wise passes split over the
    # batch across host threads; a sample holds a whole number of mask bytes)
    from concurrent.futures import ThreadPoolExecutor
    from parity import oracle_bwd, oracle_fwd, values
    s_np, z_np = q.scale.cpu().numpy(), q.zero_point.cpu().numpy()
    x_np, dy_np = to_numpy(x), to_numpy(dy)
    mn, mx = oracle.range_reduce(x_np)
    ws, wz = oracle.prescale(mn, mx, 4)
    assert np.array_equal(bits_view(s_np), bits_view(ws)) and np.array_equal(bits_view(z_np), bits_view(wz))
    want_hat, _ = oracle_fwd(x_np, s_np, z_np, 4)
    assert np.array_equal(values(x_hat), values(want_hat))
    del want_hat
    want_dx = oracle_bwd(x_np, dy_np, s_np, z_np, 4)
    assert np.array_equal(bits_view(dx), bits_view(want_dx))
    del want_dx
    per_sample = x_np[0].size
    assert per_sample % 8 == 0
    cuts = [(i, min(shape[0], i + 16)) for i in range(0, shape[0], 16)]
    with ThreadPoolExecutor(8) as ex:
        parts = list(ex.map(lambda ab: oracle.gate_mask(x_np[ab[0]:ab[1]], s_np, z_np, 4), cuts))
    assert np.array_equal(mask, np.concatenate(parts)), "gate bits differ from the oracle's"


def test_mask_argument_checks():
    import ctypes
    lib = G.load()
    d = G.make_desc(2, 3, 4, 4, G.GRANQ_F32)
    assert lib.granq_fakequant_fwd_mask(16, ctypes.byref(d), 16, 16, 4, 16, 0, 0) == G.GRANQ_ERR_INVALID_ARG
    assert lib.granq_fakequant_fwd_mask(16, ctypes.byref(d), 16, 16, 9, 16, 16, 0) == G.GRANQ_ERR_INVALID_ARG
    assert lib.granq_fakequant_bwd_mask(0, 16, ctypes.byref(d), 16, 0) == G.GRANQ_ERR_INVALID_ARG
    assert lib.granq_fakequant_bwd_mask(18, 16, ctypes.byref(d), 16, 0) == G.GRANQ_ERR_UNSUPPORTED
    assert G.granq_mask_bytes(G.make_desc(1, 1, 1, 9, 0)) == 2
