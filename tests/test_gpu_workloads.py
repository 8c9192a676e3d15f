"""Full-size parity on the five workloads, in the launch configuration the
benchmark times, every element compared with the oracle (needs an MI355X).

Tensors are the synthetic stand-ins described in workloads/__init__.py.  One
tensor is resident at a time; the oracle's element-wise passes are split over
the batch across host threads."""
import numpy as np
import pytest
import torch

import paper_2503_18339_amd as G
import workloads
from parity import assert_parity, gpu_path, oracle_path, to_numpy

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _distinct(wl):
    seen, out = set(), []
    for a in wl.acts:
        key = (a.c, a.hw, a.law)
        if key not in seen:
            seen.add(key)
            out.append(a)
    return out


def _run(wl, act, bits, dtype, seed):
    shape = act.shape(wl.batch)
    x = workloads.make_activation(shape, act.law, wl.sigma, seed, DEV, workloads.torch_dtype(dtype))
    dy = workloads.make_grad(shape, seed, DEV, x.dtype)
    got = gpu_path(x, bits, dy)
    x_np, dy_np = to_numpy(x), to_numpy(dy)
    del x, dy
    torch.cuda.empty_cache()
    want = oracle_path(x_np, bits, dy_np)
    assert_parity(got, want, "%s %s b%d %s" % (wl.name, act.name, bits, dtype))
    return got


CFG2 = workloads.resnet20_cifar()
CFG3 = workloads.resnet18_imagenet()
CFG4 = workloads.mobilenetv2_imagenet()
CFG5 = workloads.resnet50_imagenet()


@pytest.mark.parametrize("bits", CFG2.bits)
@pytest.mark.parametrize("idx", range(len(CFG2.tensors())))
def test_config2_resnet20_cifar(idx, bits):
    _run(CFG2, CFG2.tensors()[idx], bits, "f32", seed=idx)


@pytest.mark.parametrize("dtype,bits", [("f32", 4), ("bf16", 4), ("f32", 5), ("bf16", 5), ("f16", 4)])
@pytest.mark.parametrize("idx", range(len(CFG3.acts)))
def test_config3_resnet18_imagenet(idx, dtype, bits):
    got = _run(CFG3, CFG3.acts[idx], bits, dtype, seed=idx)
    assert np.all(got["zero_point"] == 0)          # post-ReLU: min 0
    assert got["codes"].max() == 2 ** bits - 1


@pytest.mark.parametrize("idx", range(len(CFG4.acts)))
def test_config4_mobilenetv2(idx):
    got = _run(CFG4, CFG4.acts[idx], 4, "f32", seed=idx)
    if CFG4.acts[idx].law == "linear":
        assert np.any(got["zero_point"] != 0)      # signed data: non-zero zero-points


@pytest.mark.parametrize("idx", range(len(_distinct(CFG5))))
def test_config5_resnet50_distinct_shapes(idx):
    _run(CFG5, _distinct(CFG5)[idx], 3, "f32", seed=idx)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_channels_last_view_full_size(dtype):
    """(256,56,56,64) channels-last = the view {256*56*56, 64, 1, 1}: rows of 64 elements, glued by
    the plans; full size, against the oracle on the same view."""
    wl = workloads.Workload("channels_last", 256 * 56 * 56, (workloads.Act(64, 1, "linear", 1, "nhwc"),),
                            (0.05, 20.0), (4,), (dtype,))
    got = _run(wl, wl.acts[0], 4, dtype, seed=3)
    assert np.any(got["zero_point"] != 0)


def test_config5_pass_back_to_back_on_one_stream():
    """The ResNet-50 pass as the benchmark issues it -- all 49 forwards (ranges, parameters and
    forward in one call each) in network order, then all 49 backwards in reverse order, one
    stream, no host synchronisation in between -- at batch 16, every tensor checked afterwards."""
    wl = CFG5
    batch = 16
    st = torch.cuda.Stream()
    layers = []
    for i, a in enumerate(wl.tensors()):
        shape = a.shape(batch)
        x = workloads.make_activation(shape, a.law, wl.sigma, i, DEV)
        dy = workloads.make_grad(shape, i, DEV)
        layers.append((x, dy, torch.empty_like(x), torch.empty_like(x), G.ActivationQuantizer(shape, x.dtype, 3, DEV)))
    assert len(layers) == 49
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        for rep in range(2):                               # the second pass reuses every workspace
            for x, dy, xh, dx, q in layers:
                q.forward(x, xh, None, st)
            for x, dy, xh, dx, q in reversed(layers):
                q.backward(x, dy, dx, st)
    st.synchronize()
    for i, (x, dy, xh, dx, q) in enumerate(layers):
        got = {"min": q.ch_min.cpu().numpy(), "max": q.ch_max.cpu().numpy(), "scale": q.scale.cpu().numpy(),
               "zero_point": q.zero_point.cpu().numpy(), "xhat": to_numpy(xh), "dx": to_numpy(dx)}
        want = oracle_path(to_numpy(x), 3, to_numpy(dy))
        assert_parity(got, want, "ResNet-50 pass, tensor %d %s" % (i, tuple(x.shape)))
