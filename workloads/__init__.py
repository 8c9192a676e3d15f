"""Seeded synthetic activation tensors shaped like the paper's workloads.

The paper quantizes the activations of ResNet-20 (CIFAR), ResNet-18, ResNet-50
and MobileNetV2 (ImageNet) on generator-made images (Sec. 5.1); neither the
trained networks nor the images are available, so tensors with the public
architectures' activation shapes and with the statistics that matter to the
quantizer stand in: non-negative post-ReLU values, per-channel spread over
more than two decades (the "large variance along the channel axis" of Sec. 4.1)
and outlier channels (the skewed synthetic inputs of Sec. 6.1).

This module serves both the CPU oracle's tests and the HIP path's tests and
benchmark.  It holds NONE of the quantizer's arithmetic: it only draws random
numbers and lists shapes.  A tensor is generated once and the same bits are
handed to both sides.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Optional, Tuple

import torch


@dataclass(frozen=True)
class Act:
    """One activation tensor of a workload: shape, value law, repeat count."""
    c: int
    hw: int              # spatial side (H == W)
    law: str             # "relu" | "relu6" | "linear" | "laplace"
    count: int = 1       # how many layers of the network share this shape
    name: str = ""

    def shape(self, batch: int) -> Tuple[int, int, int, int]:
        return (batch, self.c, self.hw, self.hw)

    def numel(self, batch: int) -> int:
        return batch * self.c * self.hw * self.hw


# ---------------------------------------------------------------------------
# value laws
# ---------------------------------------------------------------------------

def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def channel_sigma(c: int, lo: float, hi: float, seed: int, device="cpu") -> torch.Tensor:
    """sigma_c = exp(U(ln lo, ln hi)), one per channel."""
    g = _gen(seed * 2654435761 % (2**31) + 17, "cpu")
    u = torch.rand(c, generator=g, dtype=torch.float64)
    s = torch.exp(math.log(lo) + u * (math.log(hi) - math.log(lo)))
    return s.to(torch.float32).to(device)


def _outlier_channels(c: int, frac: float, seed: int) -> torch.Tensor:
    k = max(1, int(round(frac * c)))
    g = _gen(seed * 40503 % (2**31) + 5, "cpu")
    return torch.randperm(c, generator=g)[:k]


def make_activation(shape, law: str = "relu", sigma=(0.05, 20.0), seed: int = 0,
                    device="cpu", dtype=torch.float32,
                    outlier_frac: Optional[float] = None,
                    outlier_gain: float = 50.0) -> torch.Tensor:
    """Draw one NCHW activation tensor.

    law:
      "relu"    |Normal(0, sigma_c)|                         (post-ReLU)
      "relu6"   min(|Normal(0, sigma_c)|, 6)                 (post-ReLU6)
      "linear"  Normal(0, sigma_c), signed; ``outlier_frac`` of the channels
                (default 1 %, at least one) have ``outlier_gain`` x sigma_c
      "laplace" Laplace(0, sigma_c) by inverse CDF; ``outlier_frac`` of the
                channels (default 2 %) have ``outlier_gain`` x sigma_c
    The values are drawn in float32 on ``device`` in chunks over the batch and
    then cast to ``dtype``.
    """
    n, c = int(shape[0]), int(shape[1])
    sig = channel_sigma(c, sigma[0], sigma[1], seed, device)
    if law in ("linear", "laplace"):
        frac = outlier_frac if outlier_frac is not None else (0.01 if law == "linear" else 0.02)
        idx = _outlier_channels(c, frac, seed).to(device)
        sig = sig.clone()
        sig[idx] *= outlier_gain
    g = _gen(seed, device)
    out = torch.empty(tuple(shape), dtype=dtype, device=device)
    view = [1, c] + [1] * (len(shape) - 2)
    sig_b = sig.view(view)
    rows = max(1, (1 << 24) // max(1, out[0].numel()))      # ~64 MB of float32 per chunk
    for i in range(0, n, rows):
        sub = tuple([min(rows, n - i)] + list(shape[1:]))
        if law == "laplace":
            u = torch.rand(sub, generator=g, device=device, dtype=torch.float32)
            u = u.clamp_(1e-7, 1.0 - 1e-7) - 0.5
            v = -torch.sign(u) * torch.log1p(-2.0 * u.abs())
        else:
            v = torch.randn(sub, generator=g, device=device, dtype=torch.float32)
        v = v * sig_b
        if law in ("relu", "relu6"):
            v = v.abs_()
        if law == "relu6":
            v = v.clamp_(max=6.0)
        out[i:i + sub[0]] = v.to(dtype)
    return out


def make_grad(shape, seed: int = 0, device="cpu", dtype=torch.float32) -> torch.Tensor:
    """Upstream gradient: Normal(0, 1)."""
    g = _gen(seed + 7919, device)
    n = int(shape[0])
    out = torch.empty(tuple(shape), dtype=dtype, device=device)
    rows = max(1, (1 << 24) // max(1, out[0].numel()))
    for i in range(0, n, rows):
        sub = tuple([min(rows, n - i)] + list(shape[1:]))
        out[i:i + sub[0]] = torch.randn(sub, generator=g, device=device,
                                        dtype=torch.float32).to(dtype)
    return out


# ---------------------------------------------------------------------------
# the five workloads
# ---------------------------------------------------------------------------

@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    acts: Tuple[Act, ...]
    sigma: Tuple[float, float]
    bits: Tuple[int, ...]
    dtypes: Tuple[str, ...]

    def tensors(self) -> List[Act]:
        """Every activation of one pass, repeats expanded, in network order."""
        out: List[Act] = []
        for a in self.acts:
            out.extend([a] * a.count)
        return out

    def total_numel(self) -> int:
        return sum(a.numel(self.batch) * a.count for a in self.acts)


def resnet20_first_layer() -> Workload:
    return Workload("resnet20_cifar_first_layer", 8, (Act(16, 32, "relu", 1, "conv1"),),
                    (0.1, 10.0), (3,), ("f32",))


def resnet20_cifar() -> Workload:
    return Workload("resnet20_cifar_b256", 256,
                    (Act(16, 32, "relu", 7, "stage1"), Act(32, 16, "relu", 6, "stage2"),
                     Act(64, 8, "relu", 6, "stage3")),
                    (0.05, 20.0), (3, 4), ("f32",))


def resnet18_imagenet() -> Workload:
    return Workload("resnet18_imagenet_b256", 256,
                    (Act(64, 112, "relu", 1, "stem"), Act(64, 56, "relu", 1, "layer1"),
                     Act(128, 28, "relu", 1, "layer2"), Act(256, 14, "relu", 1, "layer3"),
                     Act(512, 7, "relu", 1, "layer4")),
                    (0.05, 20.0), (4, 5), ("f32", "bf16"))


def mobilenetv2_imagenet() -> Workload:
    relu6 = [(32, 112), (96, 112), (96, 56), (144, 56), (144, 28), (192, 28), (192, 14),
             (384, 14), (576, 14), (576, 7), (960, 7)]
    linear = [(16, 112), (24, 56), (32, 28), (64, 14), (96, 14), (160, 7), (320, 7)]
    acts = tuple(Act(c, hw, "relu6", 1, "relu6_%d@%d" % (c, hw)) for c, hw in relu6) + \
        tuple(Act(c, hw, "linear", 1, "linear_%d@%d" % (c, hw)) for c, hw in linear)
    return Workload("mobilenetv2_imagenet_b256", 256, acts, (0.05, 20.0), (4,), ("f32",))


def resnet50_imagenet() -> Workload:
    """The 49 convolution inputs after the stem of a batch-256 ResNet-50."""
    acts: List[Act] = [Act(64, 112, "laplace", 1, "stem_out")]

    def stage(idx, c_in, mid, c_out, hw_in, hw_out, blocks):
        acts.append(Act(c_in, hw_in, "laplace", 1, "s%d.b0.conv1" % idx))
        acts.append(Act(mid, hw_in, "laplace", 1, "s%d.b0.conv2" % idx))
        acts.append(Act(mid, hw_out, "laplace", 1, "s%d.b0.conv3" % idx))
        for b in range(1, blocks):
            acts.append(Act(c_out, hw_out, "laplace", 1, "s%d.b%d.conv1" % (idx, b)))
            acts.append(Act(mid, hw_out, "laplace", 2, "s%d.b%d.conv2-3" % (idx, b)))

    stage(1, 64, 64, 256, 56, 56, 3)
    stage(2, 256, 128, 512, 56, 28, 4)
    stage(3, 512, 256, 1024, 28, 14, 6)
    stage(4, 1024, 512, 2048, 14, 7, 3)
    return Workload("resnet50_imagenet_b256", 256, tuple(acts), (0.05, 20.0), (3,), ("f32",))


WORKLOADS = {
    "config1": resnet20_first_layer,
    "config2": resnet20_cifar,
    "config3": resnet18_imagenet,
    "config4": mobilenetv2_imagenet,
    "config5": resnet50_imagenet,
}


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[name]


# ---------------------------------------------------------------------------
# weight tensors (channel-wise weight quantization, Sec. 5.1 of the paper)
# ---------------------------------------------------------------------------

def resnet18_weight_shapes():
    """(O, I, kh, kw) of every convolution and the classifier of ResNet-18 (ImageNet)."""
    shapes = [(64, 3, 7, 7)]
    cfg = [(64, 64, 2), (64, 128, 2), (128, 256, 2), (256, 512, 2)]
    for c_in, c_out, blocks in cfg:
        for b in range(blocks):
            first_in = c_in if b == 0 else c_out
            shapes.append((c_out, first_in, 3, 3))
            shapes.append((c_out, c_out, 3, 3))
            if b == 0 and c_in != c_out:
                shapes.append((c_out, c_in, 1, 1))      # downsample
    shapes.append((1000, 512, 1, 1))                    # classifier as a 1x1 weight
    return shapes


def make_weight(shape, seed: int = 0, device="cpu", dtype=torch.float32) -> torch.Tensor:
    """Normal(0, sqrt(2 / fan_in)) weights with a per-output-channel spread factor
    log-uniform in [0.3, 3] (trained filters differ in norm)."""
    o = int(shape[0])
    fan_in = 1
    for d in shape[1:]:
        fan_in *= int(d)
    g = _gen(seed + 104729, device)
    w = torch.randn(tuple(shape), generator=g, device=device, dtype=torch.float32) * math.sqrt(2.0 / fan_in)
    spread = channel_sigma(o, 0.3, 3.0, seed + 31, device).view([o] + [1] * (len(shape) - 1))
    return (w * spread).to(dtype)
