"""Buffer management for one activation tensor: the four calls in sequence.

Holds the caller-side buffers (ranges, scale, zero-point, workspace, and the state
of the single-launch forward where the tensor takes it) that the C ABI expects the
caller to own, and issues the calls on the current stream.  No arithmetic happens here.
"""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as B


class ActivationQuantizer:
    """Per-channel fake-quantizer for tensors of one fixed shape and dtype."""

    def __init__(self, shape, dtype: torch.dtype, bits: int, device="cuda", view: str = "channel",
                 single_launch: bool = False):
        n, c = int(shape[0]), int(shape[1])
        hw = 1
        for d in shape[2:]:
            hw *= int(d)
        h = int(shape[2]) if len(shape) > 2 else 1
        w = hw // h
        code = B.dtype_code(dtype)
        if view == "channel":            # one range per channel over (n,h,w)
            self.desc = B.make_desc(n, c, h, w, code)
        elif view == "layer":            # one range for the whole tensor
            self.desc = B.make_desc(1, 1, 1, n * c * hw, code)
        elif view == "sample_channel":   # one range per (n,c)
            self.desc = B.make_desc(1, n * c, h, w, code)
        else:
            raise ValueError("unknown view %r" % view)
        self.bits = int(bits)
        self.shape = tuple(shape)
        self.dtype = dtype
        cc = self.desc.c
        f32 = dict(dtype=torch.float32, device=device)
        self.ch_min = torch.empty(cc, **f32)
        self.ch_max = torch.empty(cc, **f32)
        self.scale = torch.empty(cc, **f32)
        self.zero_point = torch.empty(cc, **f32)
        self.workspace = torch.empty(max(16, B.granq_workspace_bytes(self.desc)), dtype=torch.uint8,
                                     device=device)
        # on request, tensors the single-launch forward takes get its state (zero before the first
        # use); measured on MI355X that form is slower than the two-launch one, so it is not the default
        nbytes = B.granq_resident_state_bytes(self.desc) if single_launch else 0
        self.state = torch.zeros(nbytes, dtype=torch.uint8, device=device) if nbytes > 0 else None

    def calibrate(self, x: torch.Tensor, stream=None) -> None:
        """range_reduce + prescale (the two in one call): refresh scale / zero-point from x."""
        B.granq_calibrate(x, self.bits, self.ch_min, self.ch_max, self.scale, self.zero_point,
                          self.workspace, stream, self.desc)

    def forward(self, x: torch.Tensor, x_hat: torch.Tensor, codes: Optional[torch.Tensor] = None,
                stream=None, recalibrate: bool = True) -> torch.Tensor:
        if recalibrate:                  # ranges, parameters and the forward in one call
            if self.state is not None and (x_hat is None or x_hat.data_ptr() != x.data_ptr()):
                if B.granq_calibrate_fakequant_fwd_resident(x, self.bits, self.ch_min, self.ch_max, self.scale,
                                                            self.zero_point, x_hat, codes, self.state, stream,
                                                            self.desc):
                    return x_hat
            B.granq_calibrate_fakequant_fwd(x, self.bits, self.ch_min, self.ch_max, self.scale, self.zero_point,
                                            x_hat, codes, self.workspace, stream, self.desc)
        else:
            B.granq_fakequant_fwd(x, self.scale, self.zero_point, self.bits, x_hat, codes, stream, self.desc)
        return x_hat

    def backward(self, x: torch.Tensor, dy: torch.Tensor, dx: torch.Tensor, stream=None) -> torch.Tensor:
        B.granq_fakequant_bwd(x, dy, self.scale, self.zero_point, self.bits, dx, stream, self.desc)
        return dx
