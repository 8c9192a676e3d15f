"""Multi-tensor row-wise (channel-wise weight) fake-quant against the oracle on the
{1, O, 1, I*kh*kw} view of every tensor (needs an MI355X)."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2503_18339_amd as G
import workloads
from parity import bits_view, to_numpy, values

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _oracle_rows(w_np, bits, dy_np=None):
    o = w_np.shape[0]
    view = w_np.reshape(1, o, 1, -1)
    mn, mx = oracle.range_reduce(view)
    s, z = oracle.prescale(mn, mx, bits)
    w_hat, _ = oracle.fakequant_fwd(view, s, z, bits)
    dw = None
    if dy_np is not None:
        dw = oracle.fakequant_bwd(view, dy_np.reshape(view.shape), s, z, bits).reshape(w_np.shape)
    return s, z, w_hat.reshape(w_np.shape), dw


def _run(shapes, dtype, bits):
    ws = [workloads.make_weight(s, i, DEV, dtype) for i, s in enumerate(shapes)]
    outs = [torch.empty_like(w) for w in ws]
    sc = [torch.full((s[0],), float("nan"), device=DEV) for s in shapes]
    zp = [torch.full((s[0],), float("nan"), device=DEV) for s in shapes]
    items = G.rowwise_items(ws, outs, sc, zp)
    G.granq_rowwise_fakequant_multi(items, dtype, bits)
    dys = [workloads.make_grad(s, i, DEV, dtype) for i, s in enumerate(shapes)]
    dws = [torch.empty_like(w) for w in ws]
    G.granq_rowwise_fakequant_bwd_multi(G.rowwise_bwd_items(ws, dys, dws, sc, zp), dtype, bits)
    torch.cuda.synchronize()
    for w, o, s, z, g, dw in zip(ws, outs, sc, zp, dys, dws):
        es, ez, ew, edw = _oracle_rows(to_numpy(w), bits, to_numpy(g))
        assert np.array_equal(bits_view(s.cpu().numpy()), bits_view(es)), w.shape
        assert np.array_equal(bits_view(z.cpu().numpy()), bits_view(ez)), w.shape
        assert np.array_equal(values(to_numpy(o)), values(ew)), w.shape
        assert np.array_equal(bits_view(to_numpy(dw)), bits_view(edw)), w.shape
    return ws, outs, sc, zp


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16], ids=["f32", "bf16", "f16"])
@pytest.mark.parametrize("bits", [3, 4, 8])
def test_resnet18_weights_one_launch(dtype, bits):
    _run(workloads.resnet18_weight_shapes(), dtype, bits)


def test_more_items_than_one_launch_holds_and_odd_rows():
    shapes = [(3 + i % 5, 1 + i % 7, 1 + i % 3, 1 + i % 2) for i in range(71)] + [(2, 5000), (1, 1), (300, 1)]
    _run(shapes, torch.float32, 4)


def test_matches_the_four_call_path_on_the_weight_view():
    shape = (128, 64, 3, 3)
    ws, outs, sc, zp = _run([shape], torch.float32, 4)
    w = ws[0]
    d = G.make_desc(1, 128, 1, 64 * 9, G.GRANQ_F32)
    q = G.ActivationQuantizer((1, 128, 1, 576), torch.float32, 4, DEV)
    ref = torch.empty_like(w)
    q.forward(w, ref)
    torch.cuda.synchronize()
    assert torch.equal(ref, outs[0]) and torch.equal(q.scale, sc[0]) and torch.equal(q.zero_point, zp[0])


def test_in_place_and_dead_rows():
    w = workloads.make_weight((16, 8, 3, 3), 1, DEV)
    w[3] = 0.0
    w[5] = 0.25
    ref = w.clone()
    s = torch.empty(16, device=DEV)
    z = torch.empty(16, device=DEV)
    G.granq_rowwise_fakequant_multi(G.rowwise_items([w], [w], [s], [z]), torch.float32, 4)
    torch.cuda.synchronize()
    es, ez, ew, _ = _oracle_rows(ref.cpu().numpy(), 4)
    assert np.array_equal(w.cpu().numpy(), ew) and np.array_equal(s.cpu().numpy(), es)
    assert s[3].item() == 1.0 and torch.all(w[3] == 0)


def test_argument_checks():
    lib = G.load()
    item = G.binding.granq_rowq_item_t(16, 16, 16, 16, 4, 4)
    arr = (G.binding.granq_rowq_item_t * 1)(item)
    p = ctypes.cast(arr, ctypes.c_void_p)
    assert lib.granq_rowwise_fakequant_multi(p, 1, 0, 9, 0) == G.GRANQ_ERR_INVALID_ARG
    assert lib.granq_rowwise_fakequant_multi(p, 0, 0, 4, 0) == G.GRANQ_ERR_INVALID_ARG
    assert lib.granq_rowwise_fakequant_multi(p, 1, 5, 4, 0) == G.GRANQ_ERR_UNSUPPORTED
    arr[0].rows = 0
    assert lib.granq_rowwise_fakequant_multi(p, 1, 0, 4, 0) == G.GRANQ_ERR_INVALID_ARG
    arr[0].rows = 4
    arr[0].w = 0
    assert lib.granq_rowwise_fakequant_multi(p, 1, 0, 4, 0) == G.GRANQ_ERR_INVALID_ARG
    arr[0].w = 18
    assert lib.granq_rowwise_fakequant_multi(p, 1, 0, 4, 0) == G.GRANQ_ERR_UNSUPPORTED
