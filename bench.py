#!/usr/bin/env python3
"""Benchmark of the GranQ activation fake-quantizer on one MI355X.

One step = one pass of the whole quantizer path over the batch-256 ResNet-18
ImageNet activation set (five tensors, synthetic stand-ins, resident in HBM):
for every tensor, in network order, the per-channel ranges (Eq. 4), scale and
zero-point (Eq. 5) and the quantize-clamp-dequantize forward (Eq. 1, 6) -- one
granq_calibrate_fakequant_fwd call -- then granq_fakequant_bwd for every tensor
in reverse order, all on one stream with no host synchronisation in between.
Throughput is algorithmic bytes per second: 24 bytes per float32 element and
step (x read by the reduction, x read and x_hat written by the forward, x and
dy read and dx written by the backward).  The same step issued as the four
separate calls (range_reduce, prescale, forward, backward) is timed beside it,
and so are the other four workloads (extra.workloads).

Prints ONE JSON line.  `python bench.py --gpus 1 --steps K --warmup W`.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import paper_2503_18339_amd as G  # noqa: E402
import workloads  # noqa: E402

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
# algorithmic bytes per element: (reduce, forward, backward) x element size
BYTES_PER_ELEM = {"reduce": 1, "fwd": 2, "bwd": 3}


class Layer:
    """Device buffers of one activation tensor and its quantizer state."""

    def __init__(self, act, batch, sigma, dtype, bits, seed, device):
        shape = act.shape(batch)
        self.name = act.name
        self.shape = shape
        self.numel = act.numel(batch)
        self.esize = 4 if dtype == torch.float32 else 2
        self.x = workloads.make_activation(shape, act.law, sigma, seed, device, dtype)
        self.dy = workloads.make_grad(shape, seed, device, dtype)
        self.x_hat = torch.empty_like(self.x)
        self.dx = torch.empty_like(self.x)
        self.q = G.ActivationQuantizer(shape, dtype, bits, device)
        # the dominant kernel is the backward on tensors whose 16-byte vectors stay inside
        # one channel (a separate template instance handles the others)
        self.dominant = bool(G.granq_plan_describe(self.q.desc)["uniform"])

    def bytes(self, kind):
        return self.numel * self.esize * BYTES_PER_ELEM[kind]


def build_layers(wl, dtype, bits, device):
    return [Layer(a, wl.batch, wl.sigma, dtype, bits, i, device) for i, a in enumerate(wl.tensors())]


FORMS = ("one_call", "calibrate", "four_calls")


def run_step(layers, stream, ev=None, form="one_call"):
    """One pass of the hot path.  form: "one_call" = granq_calibrate_fakequant_fwd per tensor
    (ranges, parameters and forward; one to three launches), "calibrate" = granq_calibrate +
    granq_fakequant_fwd, "four_calls" = range_reduce, prescale, forward; the backward follows for
    every tensor in reverse order.  Same results in every form.  `ev`, if given, collects one
    (start, end, bytes, launches) record per step around the consecutive backward launches of the
    dominant kernel (the layers are ordered so that those launches are adjacent)."""
    for L in layers:
        if form == "one_call":
            L.q.forward(L.x, L.x_hat, None, stream)
            continue
        if form == "calibrate":
            L.q.calibrate(L.x, stream)
        else:
            G.granq_range_reduce(L.x, L.q.ch_min, L.q.ch_max, L.q.workspace, stream, L.q.desc)
            G.granq_prescale(L.q.ch_min, L.q.ch_max, L.q.bits, L.q.scale, L.q.zero_point, stream)
        G.granq_fakequant_fwd(L.x, L.q.scale, L.q.zero_point, L.q.bits, L.x_hat, None, stream, L.q.desc)
    rev = list(reversed(layers))
    # the longest run of adjacent launches of the dominant kernel in the backward sweep
    first = last = None
    i = 0
    while i < len(rev):
        if rev[i].dominant:
            j = i
            while j + 1 < len(rev) and rev[j + 1].dominant:
                j += 1
            if first is None or sum(M.numel for M in rev[i:j + 1]) > sum(M.numel for M in rev[first:last + 1]):
                first, last = i, j
            i = j + 1
        else:
            i += 1
    a = b = None
    for i, L in enumerate(rev):
        if ev is not None and i == first:
            a = torch.cuda.Event(enable_timing=True)
            a.record(stream)
        G.granq_fakequant_bwd(L.x, L.dy, L.q.scale, L.q.zero_point, L.q.bits, L.dx, stream, L.q.desc)
        if ev is not None and i == last:
            b = torch.cuda.Event(enable_timing=True)
            b.record(stream)
            doms = [M for M in rev[first:last + 1]]
            assert all(M.dominant for M in doms)
            ev.append((a, b, sum(M.bytes("bwd") for M in doms), len(doms)))


def time_steps(layers, steps, warmup, with_events, form="one_call"):
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        run_step(layers, stream, None, form)
    ev = [] if with_events else None
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        # the dominant kernel's event pair on every fourth step: each pair costs about 1 us of the step
        run_step(layers, stream, ev if k % 4 == 0 else None, form)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    return dt, ev


def time_graph_steps(layers, steps, warmup, form="one_call"):
    """The same step captured once into a HIP graph and replayed (no per-kernel events)."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run_step(layers, side, None, form)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run_step(layers, torch.cuda.current_stream(), None, form)
    for _ in range(warmup):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def kernel_breakdown(layers, reps=10):
    """Per tensor and kernel: average device time over `reps` launches (HIP events)."""
    stream = torch.cuda.current_stream()
    rows = []
    for L in layers:
        calls = {
            "reduce": lambda: G.granq_range_reduce(L.x, L.q.ch_min, L.q.ch_max, L.q.workspace, stream, L.q.desc),
            "prescale": lambda: G.granq_prescale(L.q.ch_min, L.q.ch_max, L.q.bits, L.q.scale, L.q.zero_point, stream),
            "fwd": lambda: G.granq_fakequant_fwd(L.x, L.q.scale, L.q.zero_point, L.q.bits, L.x_hat, None, stream, L.q.desc),
            "bwd": lambda: G.granq_fakequant_bwd(L.x, L.dy, L.q.scale, L.q.zero_point, L.q.bits, L.dx, stream, L.q.desc),
        }
        row = {"tensor": "%s %s" % (L.name, "x".join(map(str, L.shape)))}
        for kind, fn in calls.items():
            fn()
            a = torch.cuda.Event(enable_timing=True)
            b = torch.cuda.Event(enable_timing=True)
            a.record(stream)
            for _ in range(reps):
                fn()
            b.record(stream)
            b.synchronize()
            us = a.elapsed_time(b) * 1e3 / reps
            row[kind + "_us"] = round(us, 2)
            if kind != "prescale":
                row[kind + "_GBs"] = round(L.bytes(kind) / us / 1e3, 1)
        rows.append(row)
    return rows


def _timeit(fn, reps=10):
    stream = torch.cuda.current_stream()
    fn()
    a = torch.cuda.Event(enable_timing=True)
    b = torch.cuda.Event(enable_timing=True)
    a.record(stream)
    for _ in range(reps):
        fn()
    b.record(stream)
    b.synchronize()
    return a.elapsed_time(b) * 1e3 / reps


def comparison_points(wl, bits, device):
    """The comparison points the paper itself uses, timed with the same library:
    layer-wise fake-quant (one range per tensor), the channel-by-channel loop of the
    Table 5 baseline, and the two accumulation forms (Eq. 3 vs Eq. 6)."""
    out = {}
    stream = torch.cuda.current_stream()

    # (1) layer-wise vs channel-wise, forward path (reduce + prescale + forward), benchmark tensors
    rows = []
    for i, a in enumerate(wl.tensors()):
        shape = a.shape(wl.batch)
        x = workloads.make_activation(shape, a.law, wl.sigma, i, device)
        xh = torch.empty_like(x)
        qc = G.ActivationQuantizer(shape, torch.float32, bits, device, view="channel")
        ql = G.ActivationQuantizer(shape, torch.float32, bits, device, view="layer")
        rows.append({"tensor": "x".join(map(str, shape)),
                     "channelwise_us": round(_timeit(lambda: qc.forward(x, xh, stream=stream)), 2),
                     "layerwise_us": round(_timeit(lambda: ql.forward(x, xh, stream=stream)), 2)})
        del x, xh
    out["layerwise_vs_channelwise_fwd_path"] = rows

    # (2) the paper's Table 5 setting: ResNet-20 on CIFAR, 3-bit, batch 16, all 19 activation
    # tensors; "quantization latency" = the whole forward path summed over the layers
    r20 = workloads.resnet20_cifar()
    acts = r20.tensors()
    tens = [workloads.make_activation(a.shape(16), a.law, r20.sigma, i, device) for i, a in enumerate(acts)]
    outs = [torch.empty_like(t) for t in tens]
    qc = [G.ActivationQuantizer(t.shape, torch.float32, 3, device, view="channel") for t in tens]
    ql = [G.ActivationQuantizer(t.shape, torch.float32, 3, device, view="layer") for t in tens]
    vecs = [[torch.empty(t.shape[1], device=device) for _ in range(4)] for t in tens]
    ws = torch.empty(64, device=device)

    def vectorized():
        for q, t, o in zip(qc, tens, outs):
            q.forward(t, o, stream=stream)

    def layerwise():
        for q, t, o in zip(ql, tens, outs):
            q.forward(t, o, stream=stream)

    def channel_loop():
        for t, o, v in zip(tens, outs, vecs):
            G.granq_cmp_channel_loop_fwd(t, 3, v[0], v[1], v[2], v[3], o, ws, stream)

    # the same 19 calls captured once in a HIP graph and replayed: without the host's per-call cost
    vectorized()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(stream)
    with torch.cuda.stream(side):
        for q, t, o in zip(qc, tens, outs):
            q.forward(t, o, stream=side)
    stream.wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        cur = torch.cuda.current_stream()
        for q, t, o in zip(qc, tens, outs):
            q.forward(t, o, stream=cur)
    t_graph = _timeit(graph.replay)

    out["table5_setting_resnet20_cifar_b16_3bit"] = {
        "granq_vectorized_graph_replay_ms": round(t_graph / 1e3, 4),
        "layerwise_ms": round(_timeit(layerwise) / 1e3, 4),
        "channel_loop_baseline_ms": round(_timeit(channel_loop, 3) / 1e3, 4),
        "granq_vectorized_ms": round(_timeit(vectorized) / 1e3, 4),
        "paper_table5_ms_unknown_hardware": {"layerwise": 0.227, "channel_loop_baseline": 103.671, "granq": 0.236},
        "note": "19 tensors; granq_calibrate_fakequant_fwd takes ONE launch per tensor here (a block per "
                "channel: a channel holds at most 64 KB at batch 16), the layer-wise view three, the "
                "channel loop four per channel; launch-latency-bound at this size",
    }
    del tens, outs

    # (3) accumulation forms on 256x64x56x56: scale inside the loop from 8-bit codes (Eq. 3)
    # vs accumulation of pre-scaled activations (Eq. 6)
    shape = (wl.batch, 64, 56, 56)
    x = workloads.make_activation(shape, "relu", wl.sigma, 1, device)
    q = G.ActivationQuantizer(shape, torch.float32, bits, device)
    xh = torch.empty_like(x)
    codes = torch.empty(shape, dtype=torch.uint8, device=device)
    q.forward(x, xh, codes, stream)
    weight = torch.randn(64, device=device)
    y = torch.empty(shape[0], 56, 56, device=device)
    t3 = _timeit(lambda: G.granq_cmp_accumulate_inloop(codes, q.scale, q.zero_point, weight, y, stream))
    t6 = _timeit(lambda: G.granq_cmp_accumulate_prescaled(xh, weight, y, stream))
    e = x.numel()
    out["accumulation_256x64x56x56"] = {
        "inloop_scaling_from_codes_us": round(t3, 2), "inloop_GBs": round((e + y.numel() * 4) / t3 / 1e3, 1),
        "prescaled_us": round(t6, 2), "prescaled_GBs": round((e * 4 + y.numel() * 4) / t6 / 1e3, 1),
        "note": "one weight per channel; in-loop reads 1 byte per activation, pre-scaled reads 4",
    }
    return out


def channels_last_view(bits, device):
    """A channels-last activation (N,H,W,C) = (256,56,56,64), float32, through the same four calls
    on the view {N*H*W, C, 1, 1}: rows of 64 elements, which the plans glue into rows of a block's span."""
    shape = (256 * 56 * 56, 64, 1, 1)
    x = workloads.make_activation(shape, "relu", (0.05, 20.0), 2, device)
    dy = workloads.make_grad(shape, 2, device)
    q = G.ActivationQuantizer(shape, torch.float32, bits, device)
    xh, dx = torch.empty_like(x), torch.empty_like(x)
    st = torch.cuda.current_stream()
    e = x.numel()
    t_r = _timeit(lambda: G.granq_range_reduce(x, q.ch_min, q.ch_max, q.workspace, st, q.desc))
    G.granq_prescale(q.ch_min, q.ch_max, bits, q.scale, q.zero_point, st)
    t_f = _timeit(lambda: G.granq_fakequant_fwd(x, q.scale, q.zero_point, bits, xh, None, st, q.desc))
    t_b = _timeit(lambda: G.granq_fakequant_bwd(x, dy, q.scale, q.zero_point, bits, dx, st, q.desc))
    pl = G.granq_plan_describe(q.desc)
    return {"rows_glued": pl["fold"], "reduce_us": round(t_r, 1), "reduce_GBs": round(e * 4 / t_r / 1e3, 1),
            "fwd_us": round(t_f, 1), "fwd_GBs": round(e * 8 / t_f / 1e3, 1),
            "bwd_us": round(t_b, 1), "bwd_GBs": round(e * 12 / t_b / 1e3, 1),
            "same_tensor_nchw_us": "see per_kernel, layer1 256x64x56x56"}


def single_launch_form(bits, device):
    """Ranges, parameters and forward in ONE launch with the tensor resident in registers
    (granq_calibrate_fakequant_fwd_resident) against granq_calibrate_fakequant_fwd (one block per
    channel, or two launches) on tensors that take both: device time per call, relaunched on the
    same buffers."""
    stream = torch.cuda.current_stream()
    rows = []
    for shape in ((256, 16, 32, 32), (256, 32, 16, 16), (256, 64, 8, 8), (256, 512, 7, 7), (256, 256, 14, 14)):
        x = workloads.make_activation(shape, "relu", (0.05, 20.0), 0, device)
        xh = torch.empty_like(x)
        q = G.ActivationQuantizer(shape, torch.float32, bits, device)
        qs = G.ActivationQuantizer(shape, torch.float32, bits, device, single_launch=True)
        assert qs.state is not None
        t_one = _timeit(lambda: q.forward(x, xh, None, stream), 20)
        t_res = _timeit(lambda: qs.forward(x, xh, None, stream), 20)
        rows.append({"tensor": "x".join(map(str, shape)), "MB": round(x.numel() * 4 / 1e6, 1),
                     "one_call_launches": int(G.granq_plan_describe(q.desc)["one_call_launches"]),
                     "one_call_us": round(t_one, 2), "single_launch_resident_us": round(t_res, 2)})
        del x, xh
    return {"rows": rows,
            "note": "the resident form reads x once and has no kernel boundary inside, but its blocks meet "
                    "through device-scope atomics and loads (arrival counters, partials, parameter slots), "
                    "each a round trip to memory on this multi-die chip"}


def gate_bit_variant(wl, dtype, bits, device, steps, warmup):
    """The same step with the forward emitting one gate bit per element and the backward reading
    dy + bits instead of x + dy (granq_fakequant_fwd_mask / granq_fakequant_bwd_mask)."""
    layers = build_layers(wl, dtype, bits, device)
    for L in layers:
        L.mask = torch.empty(G.granq_mask_bytes(L.q.desc), dtype=torch.uint8, device=device)
    stream = torch.cuda.current_stream()

    def step():
        for L in layers:
            L.q.calibrate(L.x, stream)
            G.granq_fakequant_fwd_mask(L.x, L.q.scale, L.q.zero_point, L.q.bits, L.x_hat, L.mask, stream, L.q.desc)
        for L in reversed(layers):
            G.granq_fakequant_bwd_mask(L.dy, L.mask, L.dx, stream, L.q.desc)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    elems = sum(L.numel for L in layers)
    e = layers[0].esize
    moved = elems * (5 * e + 0.25)          # reduce e, fwd 2e + 1/8, bwd 2e + 1/8
    return {"ms_per_step": round(dt * 1e3, 4), "bytes_moved_per_step": int(moved),
            "GBs_on_bytes_moved": round(moved / dt / 1e9, 1),
            "speedup_vs_x_based_step": None,
            "note": "same results as the four-call step; %.3f instead of %d bytes per element" % (5 * e + 0.25, 6 * e)}


def weight_quantization(bits, device):
    """Channel-wise weight fake-quant of all ResNet-18 weights (Sec. 5.1): one multi-tensor
    launch against the four-call path applied tensor by tensor on the {1,O,1,I*kh*kw} view."""
    shapes = workloads.resnet18_weight_shapes()
    ws = [workloads.make_weight(s, i, device) for i, s in enumerate(shapes)]
    outs = [torch.empty_like(w) for w in ws]
    sc = [torch.empty(s[0], device=device) for s in shapes]
    zp = [torch.empty(s[0], device=device) for s in shapes]
    items = G.rowwise_items(ws, outs, sc, zp)
    stream = torch.cuda.current_stream()
    qs = [G.ActivationQuantizer((1, s[0], 1, w.numel() // s[0]), torch.float32, bits, device)
          for s, w in zip(shapes, ws)]

    def four_call():
        for q, w, o in zip(qs, ws, outs):
            q.forward(w, o, stream=stream)

    t_multi = _timeit(lambda: G.granq_rowwise_fakequant_multi(items, torch.float32, bits, stream))
    t_four = _timeit(four_call)
    params = sum(w.numel() for w in ws)
    return {"tensors": len(ws), "parameters": params, "multi_tensor_launch_us": round(t_multi, 2),
            "multi_GBs": round(params * 8 / t_multi / 1e3, 1),
            "four_call_per_tensor_us": round(t_four, 2)}


def distortion_table(wl, device):
    """The paper's Table 2 on the synthetic benchmark tensors (3-bit): average over the layers of
    cosine similarity and relative error, one range per layer against one range per channel;
    also the kernel time of the fused metric on the largest tensor."""
    rows = {"layerwise": [], "channelwise": []}
    stream = torch.cuda.current_stream()
    t_big = None
    for i, a in enumerate(wl.tensors()):
        shape = a.shape(wl.batch)
        x = workloads.make_activation(shape, a.law, wl.sigma, i, device)
        for view in ("layer", "channel"):
            q = G.ActivationQuantizer(shape, torch.float32, 3, device, view=view)
            q.calibrate(x, stream)
            ch = torch.empty(q.desc.c, 4, dtype=torch.float64, device=device)
            layer = torch.empty(6, dtype=torch.float64, device=device)
            ws = torch.empty(max(16, G.granq_distortion_workspace_bytes(q.desc)), dtype=torch.uint8, device=device)
            fn = lambda: G.granq_distortion(x, q.scale, q.zero_point, 3, ch, layer, ws, stream, q.desc)
            fn()
            if i == 0 and view == "channel":
                t_big = _timeit(fn, 5)
            rows[view + "wise"].append(layer.cpu().tolist()[4:])
        del x
    avg = {k: [round(sum(r[j] for r in v) / len(v), 4) for j in (0, 1)] for k, v in rows.items()}
    big = wl.tensors()[0].numel(wl.batch)
    return {"avg_cosine_similarity": {k: v[0] for k, v in avg.items()},
            "avg_relative_error": {k: v[1] for k, v in avg.items()},
            "paper_table2_resnet20_cifar100_trained": {"avg_cosine_similarity": {"layerwise": 0.5111, "channelwise": 0.6835},
                                                        "avg_relative_error": {"layerwise": 0.3129, "channelwise": 0.1063}},
            "fused_metric_kernel_us_256x64x112x112": round(t_big, 1),
            "fused_metric_GBs": round(big * 4 / t_big / 1e3, 1),
            "note": "synthetic tensors, not the paper's trained network: only the direction is comparable"}


def integer_accumulation(wl, bits, device):
    """The 1x1 convolution that consumes the quantized activations, on ResNet bottleneck shapes
    at batch 256: from the integer codes on the int8 matrix cores (Eq. 3, scale folded into the
    weights) against torch's float32 and bfloat16 convolutions on x_hat (Eq. 6)."""
    stream = torch.cuda.current_stream()
    rows = {}
    for c, o, hw in ((64, 64, 56), (64, 256, 56), (256, 64, 56), (1024, 256, 14), (512, 2048, 7), (2048, 512, 7)):
        shape = (wl.batch, c, hw, hw)
        x = workloads.make_activation(shape, "relu", wl.sigma, 1, device)
        q = G.ActivationQuantizer(shape, torch.float32, bits, device)
        xh = torch.empty_like(x)
        codes = torch.empty(shape, dtype=torch.uint8, device=device)
        q.forward(x, xh, codes, stream)
        t_q = _timeit(lambda: G.granq_fakequant_fwd(x, q.scale, q.zero_point, bits, None, codes, stream, q.desc))
        x_keep = x
        del x
        wt = workloads.make_weight((o, c, 1, 1), 3, device)
        wq = torch.empty(o, c, dtype=torch.int8, device=device)
        corr = torch.empty(o, dtype=torch.int64, device=device)
        a = torch.empty(o, device=device)
        y = torch.empty(shape[0], o, hw, hw, device=device)
        t_fold = _timeit(lambda: G.granq_fold_weights(wt, q.scale, q.zero_point, wq, corr, a, stream))
        t_int = _timeit(lambda: G.granq_conv1x1_int8(codes, wq, corr, a, bits, y, stream))
        y16 = torch.empty(shape[0], o, hw, hw, dtype=torch.bfloat16, device=device)
        t_int16 = _timeit(lambda: G.granq_conv1x1_int8_as(codes, wq, corr, a, bits, y16, stream))
        del y16
        # codes two per byte (4-bit and below): half a byte per element written and read
        packed = torch.empty(G.granq_packed4_bytes(q.desc), dtype=torch.uint8, device=device)
        t_qp = t_intp = None
        if bits <= 4 and (hw * hw) % 4 == 0:       # two codes per byte on the matrix cores: H*W a multiple of 4
            t_qp = _timeit(lambda: G.granq_fakequant_fwd_packed4(x_keep, q.scale, q.zero_point, bits, None, packed, stream, q.desc))
            t_intp = _timeit(lambda: G.granq_conv1x1_int8_packed4(packed, shape, wq, corr, a, bits, y, stream))
            G.granq_conv1x1_int8(codes, wq, corr, a, bits, y, stream)
        del x_keep, packed
        # Eq. 6's accumulation in floating point: this library's kernel and torch's convolution
        w2 = wt.view(o, c).contiguous()
        yf = torch.empty_like(y)
        t_own32 = _timeit(lambda: G.granq_conv1x1_float(xh, w2, yf, stream))
        rel = float((y - yf).norm() / yf.norm())
        t_f32 = _timeit(lambda: torch.nn.functional.conv2d(xh, wt))
        ref = torch.nn.functional.conv2d(xh, wt)
        rel_own = float((yf - ref).norm() / ref.norm())
        del ref, yf
        xh16, wt16 = xh.to(torch.bfloat16), wt.to(torch.bfloat16)
        w216 = wt16.view(o, c).contiguous()
        y16 = torch.empty(shape[0], o, hw, hw, dtype=torch.bfloat16, device=device)
        t_own16 = _timeit(lambda: G.granq_conv1x1_float(xh16, w216, y16, stream))
        del y16
        t_b16 = _timeit(lambda: torch.nn.functional.conv2d(xh16, wt16))
        e = codes.numel()
        ops = 2.0 * o * c * shape[0] * hw * hw
        rows["%d->%d@%dx%d" % (c, o, hw, hw)] = {
            "int8_mfma_from_codes_us": round(t_int, 1), "int8_GBs": round((e + y.numel() * 4) / t_int / 1e3, 1),
            "int8_TOPs": round(ops / t_int / 1e6, 2), "int8_mfma_bf16_output_us": round(t_int16, 1),
            "fold_weights_us": round(t_fold, 1),
            "quantize_to_codes_only_us": round(t_q, 1), "quantize_GBs": round(e * 5 / t_q / 1e3, 1),
            "quantize_to_packed_codes_only_us": round(t_qp, 1) if t_qp else None,
            "int8_mfma_from_packed_codes_us": round(t_intp, 1) if t_intp else None,
            "float_conv_on_x_hat_us": round(t_own32, 1), "float_conv_TFLOPs": round(ops / t_own32 / 1e6, 1),
            "float_conv_on_bf16_x_hat_us": round(t_own16, 1),
            "torch_f32_conv_on_x_hat_us": round(t_f32, 1), "torch_bf16_conv_on_bf16_x_hat_us": round(t_b16, 1),
            "relative_difference_to_float_conv": round(rel, 5),
            "float_conv_relative_difference_to_torch": float("%.2e" % rel_own)}
        del xh, xh16, codes, y
        torch.cuda.empty_cache()
    rows["note"] = ("int8 path (Eq. 3 folded) reads 1 byte per activation and writes float32; the float "
                    "convolutions (Eq. 6: this library's float_conv and torch's) read 4 and write 4 in float32, "
                    "2 and 2 in bfloat16; float_conv accumulates in binary32 on the matrix cores for both")
    return rows


def cpu_baseline(layers, bits, sample_batch, min_seconds=10.0, max_passes=8):
    """The CPU oracle, as it stands, single thread, on the tensors the GPU was timed on (their
    first `sample_batch` samples, copied to the host): whole passes (range_reduce + prescale +
    fwd + bwd) are repeated until `min_seconds` of oracle time have accumulated.  Returns GB/s
    on the same algorithmic bytes, the oracle seconds, the number of passes, and -- when the
    sample is the whole batch -- how the buffers the GPU step left behind compare with the
    oracle's results (every element of every tensor)."""
    import numpy as np
    import oracle
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from parity import to_numpy
    total_bytes = 0
    total_s = 0.0
    passes = 0
    checked = None
    whole = all(sample_batch >= L.shape[0] for L in layers) and layers[0].esize == 4
    data = [(to_numpy(L.x[:sample_batch]), to_numpy(L.dy[:sample_batch])) for L in layers]
    while passes < max_passes and (passes == 0 or total_s < min_seconds):
        if passes == 0 and whole:
            checked = {"tensors": 0, "elements": 0, "mismatching_elements": 0}
        for L, (x, dy) in zip(layers, data):
            t0 = time.perf_counter()
            mn, mx = oracle.range_reduce(x)
            s, z = oracle.prescale(mn, mx, bits)
            xh, _ = oracle.fakequant_fwd(x, s, z, bits)
            dx = oracle.fakequant_bwd(x, dy, s, z, bits)
            total_s += time.perf_counter() - t0
            total_bytes += x.size * x.itemsize * 6
            if passes == 0 and whole:
                bad = int(np.count_nonzero(to_numpy(L.x_hat) != xh)) + int(np.count_nonzero(to_numpy(L.dx) != dx))
                for got, want in ((L.q.ch_min, mn), (L.q.ch_max, mx), (L.q.scale, s), (L.q.zero_point, z)):
                    bad += int(np.count_nonzero(got.cpu().numpy() != want))
                checked["tensors"] += 1
                checked["elements"] += 2 * x.size + 4 * mn.size
                checked["mismatching_elements"] += bad
            del xh, dx
        passes += 1
    return total_bytes / total_s / 1e9, total_s, passes, checked


def cpu_baseline_threads(wl, bits, sample_batch, threads):
    """The same oracle with the batch split over `threads` host threads (ctypes releases the
    GIL): per-thread partial ranges are combined with numpy's minimum / maximum, the
    element-wise passes are independent per sample.  One whole pass."""
    import numpy as np
    import oracle
    from concurrent.futures import ThreadPoolExecutor
    total_bytes = 0
    total_s = 0.0
    with ThreadPoolExecutor(threads) as ex:
        for i, a in enumerate(wl.tensors()):
            shape = a.shape(sample_batch)
            x = workloads.make_activation(shape, a.law, wl.sigma, i, "cpu").numpy()
            dy = workloads.make_grad(shape, i, "cpu").numpy()
            step = max(1, -(-shape[0] // threads))
            cuts = [(j, min(shape[0], j + step)) for j in range(0, shape[0], step)]
            t0 = time.perf_counter()
            parts = list(ex.map(lambda ab: oracle.range_reduce(x[ab[0]:ab[1]]), cuts))
            mn = np.minimum.reduce([p[0] for p in parts])
            mx = np.maximum.reduce([p[1] for p in parts])
            s, z = oracle.prescale(mn, mx, bits)
            list(ex.map(lambda ab: oracle.fakequant_fwd(x[ab[0]:ab[1]], s, z, bits), cuts))
            list(ex.map(lambda ab: oracle.fakequant_bwd(x[ab[0]:ab[1]], dy[ab[0]:ab[1]], s, z, bits), cuts))
            total_s += time.perf_counter() - t0
            total_bytes += x.size * 4 * 6
    return total_bytes / total_s / 1e9, total_s


def launches_per_tensor(layers):
    """Kernel launches of one step per tensor, from the library's own plan: the one-call forward
    (1 to 3) plus the backward."""
    return [int(G.granq_plan_describe(L.q.desc)["one_call_launches"]) + 1 for L in layers]


def other_workloads(device, steps):
    """The other four workloads, each at its own bit-width(s), float32: the same step (one-call
    forward per tensor, then the backward in reverse order; one stream, no host synchronisation)
    and, beside it, the step issued as four separate calls."""
    out = {}
    for key, bit_list in (("config1", (3,)), ("config2", (3, 4)), ("config4", (4,)), ("config5", (3,))):
        wl = workloads.WORKLOADS[key]()
        for bits in bit_list:
            layers = build_layers(wl, torch.float32, bits, device)
            elems = sum(L.numel for L in layers)
            step_bytes = elems * 4 * 6
            k = max(5, min(steps, int(2e5 / max(1.0, step_bytes / 6.4e6))))   # about 0.2 s of GPU time
            dt, _ = time_steps(layers, k, 3, with_events=False, form="one_call")
            dt4, _ = time_steps(layers, k, 3, with_events=False, form="four_calls")
            lp = launches_per_tensor(layers)
            name = key if len(bit_list) == 1 else "%s_b%d" % (key, bits)
            out[name] = {
                "workload": wl.name, "bits": bits, "tensors": len(layers), "elements_per_step": elems,
                "value": round(step_bytes / (dt / k) / 1e9, 1), "unit": "GB/s",
                "frac_of_hbm_peak": round(step_bytes / (dt / k) / 1e9 / HBM_PEAK_GBS, 4),
                "ms_per_step": round(dt * 1e3 / k, 4), "steps": k,
                "launches_per_step": sum(lp), "launches_per_tensor": round(sum(lp) / len(lp), 2),
                "four_separate_calls": {"value": round(step_bytes / (dt4 / k) / 1e9, 1),
                                        "ms_per_step": round(dt4 * 1e3 / k, 4), "launches_per_tensor": "4 or 5"},
            }
            del layers
            torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--dtype", choices=["f32", "bf16", "f16"], default="f32")
    ap.add_argument("--bits", type=int, default=None, help="default: the workload's first bit-width")
    ap.add_argument("--form", choices=list(FORMS), default="one_call",
                    help="how the step is issued: granq_calibrate_fakequant_fwd per tensor (default), "
                         "granq_calibrate + forward, or the four separate calls; same results")
    ap.add_argument("--cpu-sample-batch", type=int, default=256,
                    help="batch size of the sample the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--workload", choices=["config1", "config2", "config3", "config4", "config5"], default="config3",
                    help="config3 = ResNet-18 ImageNet set (the metric's workload, default); the others "
                         "(ResNet-20 CIFAR, MobileNetV2, ResNet-50 sets) are timed without the extras")
    ap.add_argument("--no-extras", action="store_true", help="skip breakdown and other dtypes")
    ap.add_argument("--section", choices=["gate_bits", "conv", "distortion", "weights", "channels_last", "comparison", "single_launch"],
                    help="run ONE of the extra sections alone (for a profiler) and print it as JSON")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run a plain device copy of known size (torch copy_ of the largest "
                         "tensor, 3 launches) so that a counter run has a reference kernel")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this library is a single-GPU kernel library; it has no collectives and "
              "no multi-GPU path.  Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP library has no CPU fallback.", file=sys.stderr)
        sys.exit(2)
    G.load()

    device = "cuda"
    wl = workloads.WORKLOADS[args.workload]()
    if args.section:
        bits = args.bits or 4
        dtype = workloads.torch_dtype(args.dtype)
        run = {"gate_bits": lambda: gate_bit_variant(wl, dtype, bits, device, min(args.steps, 50), 5),
               "conv": lambda: integer_accumulation(wl, bits, device),
               "distortion": lambda: distortion_table(wl, device),
               "weights": lambda: weight_quantization(bits, device),
               "channels_last": lambda: channels_last_view(bits, device),
               "comparison": lambda: comparison_points(wl, bits, device),
               "single_launch": lambda: single_launch_form(bits, device)}[args.section]
        print(json.dumps({"section": args.section, "dtype": args.dtype, "result": run()}))
        return
    if args.bits is None:
        args.bits = 4 if args.workload == "config3" else wl.bits[0]
    variants_only = args.workload != "config3" and not args.no_extras
    if args.workload != "config3":
        args.no_extras = True
        args.cpu_sample_batch = 0
    dtype = workloads.torch_dtype(args.dtype)
    layers = build_layers(wl, dtype, args.bits, device)
    bwd_rows = G.granq_plan_describe(layers[0].q.desc)["bwd_rows"]
    esize = layers[0].esize
    elems = sum(L.numel for L in layers)
    step_bytes = elems * esize * 6

    dt, ev = time_steps(layers, args.steps, args.warmup, with_events=True, form=args.form)
    ms_per_step = dt * 1e3 / args.steps
    value = step_bytes / (dt / args.steps) / 1e9

    from paper_2503_18339_amd import profiling
    # counters were taken on one workload and dtype: they describe no other launch
    rec = profiling.load_record(workload=args.workload, dtype=args.dtype)
    traffic = round(rec["traffic_bytes_per_launch"]) if rec else None
    k_bytes = sum(e[2] for e in ev)
    k_launches = sum(e[3] for e in ev)
    k_ms = sum(e[0].elapsed_time(e[1]) for e in ev)
    achieved = k_bytes / (k_ms * 1e-3) / 1e9
    roofline = {
        "kernel": "granq::fq_bwd_cols<granq::%s, 1, %d, false, 0>" % (args.dtype.upper(), bwd_rows),
        "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
        "launches": k_launches, "avg_launch_us": round(k_ms * 1e3 / max(1, k_launches), 2),
        "bytes_per_launch": k_bytes // max(1, k_launches),
        "note": "one HIP event pair on every fourth timed step around the adjacent launches of this kernel "
                "in the backward sweep; average = span / launches",
    }

    lp = launches_per_tensor(layers)
    calls = {"one_call": "granq_calibrate_fakequant_fwd per tensor", "calibrate": "granq_calibrate + granq_fakequant_fwd per tensor",
             "four_calls": "range_reduce + prescale + fwd per tensor"}[args.form]
    out = {
        "metric": "fake-quant fwd+bwd GB/s and % of HBM peak, ResNet-18 ImageNet activations"
                  if args.workload == "config3" else "fake-quant fwd+bwd GB/s and % of HBM peak, " + wl.name,
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": "%s: %s, %d-bit, %s (ranges, scale/zero-point, forward) then bwd in reverse"
                   % (wl.name, ", ".join("%d@%dx%d" % (a.c, a.hw, a.hw) for a in wl.acts[:8])
                      + (", ... (%d tensors)" % len(wl.tensors()) if len(wl.acts) > 8 else ""), args.bits, calls),
                   "batch": wl.batch, "elements_per_step": elems, "bytes_per_step": step_bytes,
                   "launches_per_step": sum(lp) if args.form == "one_call" else None},
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4),
        "elements_per_s": round(elems / (dt / args.steps), 0),
        "roofline": roofline,
    }

    if args.cpu_sample_batch > 0:
        # before anything else touches the buffers: the oracle is timed on the very tensors the GPU
        # was timed on, and what the timed steps left in x_hat, dx and the four vectors is compared
        gbs, secs, passes, checked = cpu_baseline(layers, args.bits, args.cpu_sample_batch)
        out["cpu_baseline"] = {
            "value": round(gbs, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "the same five tensors at batch %d of %d, %s, %d-bit, %d whole pass(es) "
                      "(range_reduce+prescale+fwd+bwd), %.1f s of oracle time"
                      % (min(args.cpu_sample_batch, wl.batch), wl.batch, args.dtype, args.bits, passes, secs),
        }
        if checked is not None:
            out["timed_buffers_vs_oracle"] = checked
        threads = min(16, os.cpu_count() or 1)
        if threads > 1:
            gbs_t, secs_t = cpu_baseline_threads(wl, args.bits, args.cpu_sample_batch, threads)
            out["cpu_baseline_all_cores"] = {
                "value": round(gbs_t, 4), "unit": "GB/s", "cores": threads, "kind": "oracle",
                "sample": "one whole pass at batch %d, the batch split over %d threads, %.1f s"
                          % (args.cpu_sample_batch, threads, secs_t)}

    if args.pmc_calibration:
        big = max(layers, key=lambda L: L.numel)
        for _ in range(3):
            big.dx.copy_(big.x)
        torch.cuda.synchronize()
        out["pmc_calibration"] = {"kernel": "torch copy_ (elementwise copy)", "launches": 3,
                                  "bytes_read": big.numel * esize, "bytes_written": big.numel * esize}

    def step_forms(ls, sbytes, steps):
        res = {}
        for form in FORMS:
            d, _ = time_steps(ls, steps, 2, with_events=False, form=form)
            res[form] = {"GBs": round(sbytes / (d / steps) / 1e9, 1), "ms_per_step": round(d * 1e3 / steps, 4)}
        d = time_graph_steps(ls, steps, 2, form="one_call")
        res["one_call_hip_graph_replay"] = {"GBs": round(sbytes / (d / steps) / 1e9, 1),
                                            "ms_per_step": round(d * 1e3 / steps, 4)}
        return res

    if variants_only:
        # the other workloads run alone: the step in its three forms and as a graph replay
        out["extra"] = {"step_forms_without_kernel_events": step_forms(layers, step_bytes, args.steps)}

    if not args.no_extras:
        extra = {"per_kernel": kernel_breakdown(layers)}
        extra["per_kernel_note"] = (
            "each kernel relaunched 10 times on the same buffers: warm (256 MB memory-side cache) for the "
            "tensors whose working set fits, cold for the larger ones; the timed step itself walks 4.8 GB "
            "per pass and is cold except for the reduce-to-forward reuse the library arranges")
        # practical ceiling: the runtime's own device copy of the same tensors (read + write)
        extra["device_copy_GBs"] = {
            "x".join(map(str, L.shape)): round(2 * L.numel * esize / _timeit(lambda: L.x_hat.copy_(L.x)) / 1e3, 1)
            for L in layers}
        fb_us = sum(r["fwd_us"] + r["bwd_us"] for r in extra["per_kernel"])
        extra["fwd_bwd_kernels_only_GBs"] = round(elems * esize * 5 / fb_us / 1e3, 1)
        # the same step without the per-launch events, in its three forms, and as a graph replay
        extra["step_forms_without_kernel_events"] = step_forms(layers, step_bytes, args.steps)
        del layers
        torch.cuda.empty_cache()
        others = {}
        for dname, bits in [("f32", 4), ("f32", 5), ("bf16", 4), ("bf16", 5), ("f16", 4)]:
            if dname == args.dtype and bits == args.bits:
                continue
            ls = build_layers(wl, workloads.torch_dtype(dname), bits, device)
            d, _ = time_steps(ls, args.steps, args.warmup, with_events=False, form=args.form)
            b = elems * ls[0].esize * 6
            others["%s_b%d" % (dname, bits)] = {"GBs": round(b / (d / args.steps) / 1e9, 1),
                                                "ms_per_step": round(d * 1e3 / args.steps, 4),
                                                "elements_per_s": round(elems / (d / args.steps), 0)}
            del ls
            torch.cuda.empty_cache()
        extra["other_dtypes_bits"] = others
        extra["workloads"] = other_workloads(device, args.steps)
        extra["comparison_points"] = comparison_points(wl, args.bits, device)
        extra["integer_accumulation_1x1_batch256"] = integer_accumulation(wl, args.bits, device)
        extra["distortion_3bit"] = distortion_table(wl, device)
        extra["resnet18_weights_channelwise"] = weight_quantization(args.bits, device)
        extra["channels_last_view_256x56x56x64"] = channels_last_view(args.bits, device)
        extra["single_launch_form"] = single_launch_form(args.bits, device)
        extra["gate_bit_variant"] = gate_bit_variant(wl, dtype, args.bits, device, args.steps, args.warmup)
        extra["gate_bit_variant"]["speedup_vs_x_based_step"] = round(
            ms_per_step / extra["gate_bit_variant"]["ms_per_step"], 3)
        out["extra"] = extra

    print(json.dumps(out))


if __name__ == "__main__":
    main()
