"""The four calls, the one-call forms and the gate-bit pair captured into a HIP graph and
replayed: every replay must reproduce the eager result, with eager work and synchronisations
in between (needs an MI355X)."""
import numpy as np
import pytest
import torch

import paper_2503_18339_amd as G
import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda"


# the last two shapes are small enough for the one-launch path of the one-call forward
@pytest.mark.parametrize("shape,dtype", [((16, 64, 28, 28), torch.float32), ((8, 96, 7, 7), torch.bfloat16),
                                         ((16, 16, 32, 32), torch.float32), ((5, 33, 3, 3), torch.float16)])
def test_graph_replays_match_eager(shape, dtype):
    bits = 4
    x = workloads.make_activation(shape, "linear", (0.05, 20.0), 1, DEV, dtype)
    dy = workloads.make_grad(shape, 1, DEV, dtype)
    q = G.ActivationQuantizer(shape, dtype, bits, DEV)
    x_hat = torch.empty_like(x)
    dx = torch.empty_like(x)
    mask = torch.empty(G.granq_mask_bytes(q.desc), dtype=torch.uint8, device=DEV)
    dx_m = torch.empty_like(x)
    x_hat1 = torch.empty_like(x)

    def step(stream):
        q.forward(x, x_hat1, None, stream)       # ranges, parameters and forward in one call
        q.calibrate(x, stream)
        G.granq_fakequant_fwd_mask(x, q.scale, q.zero_point, bits, x_hat, mask, stream, q.desc)
        G.granq_fakequant_bwd(x, dy, q.scale, q.zero_point, bits, dx, stream, q.desc)
        G.granq_fakequant_bwd_mask(dy, mask, dx_m, stream, q.desc)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (x_hat, x_hat1, dx, dx_m, q.scale, q.zero_point, q.ch_min, q.ch_max)]

    def check(ref):
        for a, b in zip(snapshot(), ref):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(side)
    torch.cuda.current_stream().wait_stream(side)
    want1 = snapshot()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(torch.cuda.current_stream())
    x2 = workloads.make_activation(shape, "relu", (0.05, 20.0), 2, DEV, dtype)
    x1 = x.clone()
    for rep in range(4):
        src = x1 if rep % 2 == 0 else x2
        x.copy_(src)                       # eager work between replays: new input in the captured buffer
        for t in (x_hat, x_hat1, dx, dx_m):
            t.fill_(7)                      # clobber the outputs
        step(torch.cuda.current_stream())   # eager reference for this input
        ref = snapshot()
        for t in (x_hat, x_hat1, dx, dx_m, q.scale, q.zero_point):
            t.fill_(3)
        torch.cuda.synchronize()
        graph.replay()
        check(ref)
        if rep == 0:
            check(want1)


@pytest.mark.parametrize("shape,o", [((4, 256, 14, 14), 256), ((3, 64, 7, 7), 64)])
def test_graph_replays_of_the_consumers_match_eager(shape, o):
    """Codes-only forward, weight fold, the integer and the float convolution captured in one graph:
    the shared-tile integer kernel (which asks for more LDS through a function attribute) and the
    ragged 7 x 7 variants included."""
    bits = 4
    n, c, h, w = shape
    x = workloads.make_activation(shape, "linear", (0.05, 20.0), 1, DEV)
    q = G.ActivationQuantizer(shape, torch.float32, bits, DEV)
    x_hat = torch.empty_like(x)
    codes = torch.empty(shape, dtype=torch.uint8, device=DEV)
    wt = workloads.make_weight((o, c, 1, 1), 3, DEV).view(o, c).contiguous()
    wq = torch.empty(o, c, dtype=torch.int8, device=DEV)
    corr = torch.empty(o, dtype=torch.int64, device=DEV)
    a = torch.empty(o, device=DEV)
    y_int = torch.empty(n, o, h, w, device=DEV)
    y_flt = torch.empty(n, o, h, w, device=DEV)

    def step(stream):
        q.forward(x, x_hat, codes, stream)
        G.granq_fold_weights(wt, q.scale, q.zero_point, wq, corr, a, stream)
        G.granq_conv1x1_int8(codes, wq, corr, a, bits, y_int, stream)
        G.granq_conv1x1_float(x_hat, wt, y_flt, stream)

    outs = (x_hat, codes, wq, corr, a, y_int, y_flt)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in outs]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(side)                          # warm-up outside the capture (first use of each kernel)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(torch.cuda.current_stream())
    x2 = workloads.make_activation(shape, "relu", (0.05, 20.0), 2, DEV)
    x1 = x.clone()
    for rep in range(4):
        x.copy_(x1 if rep % 2 == 0 else x2)
        step(torch.cuda.current_stream())
        ref = snapshot()
        for t in outs:
            t.fill_(3)
        torch.cuda.synchronize()
        graph.replay()
        for got, want in zip(snapshot(), ref):
            assert torch.equal(got.view(torch.uint8), want.view(torch.uint8))
