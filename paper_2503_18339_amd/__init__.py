"""GranQ activation fake-quantizer for AMD MI355X: Python binding of the C ABI.

The product is ``libgranq.so`` (hand-written HIP for gfx950, built from
``csrc/``); this package only loads it and marshals torch tensors.
"""
from .binding import (GRANQ_BF16, GRANQ_F16, GRANQ_ERR_HIP, GRANQ_ERR_INVALID_ARG, GRANQ_ERR_UNSUPPORTED,
                      GRANQ_ERR_WORKSPACE, GRANQ_F32, GRANQ_OK, GranqError, desc_of, granq_desc_t,
                      granq_fakequant_bwd, granq_fakequant_fwd, granq_plan_describe, granq_prescale,
                      granq_range_reduce, granq_range_reduce_noalloc, granq_workspace_bytes, library_path, load, make_desc,
                      status_string, version)
from .binding import granq_fakequant_bwd_mask, granq_fakequant_fwd_mask, granq_mask_bytes
from .binding import (granq_rowwise_fakequant_bwd_multi, granq_rowwise_fakequant_multi, rowwise_bwd_items,
                      rowwise_items)
from .binding import granq_calibrate, granq_calibrate_fakequant_fwd, granq_conv1x1_int8, granq_conv1x1_int8_as, granq_fold_weights
from .binding import granq_distortion, granq_distortion_workspace_bytes
from .binding import granq_conv1x1_int8_packed4, granq_fakequant_fwd_packed4, granq_packed4_bytes
from .binding import granq_conv1x1_float
from .binding import (granq_calibrate_fakequant_fwd_resident, granq_resident_state_bytes,
                      granq_resident_state_init)
from .binding import (granq_cmp_accumulate_inloop, granq_cmp_accumulate_prescaled,
                      granq_cmp_channel_loop_fwd)
from .quantizer import ActivationQuantizer

__all__ = [
    "GRANQ_OK", "GRANQ_ERR_INVALID_ARG", "GRANQ_ERR_UNSUPPORTED", "GRANQ_ERR_WORKSPACE",
    "GRANQ_ERR_HIP", "GRANQ_F32", "GRANQ_BF16", "GRANQ_F16", "GranqError", "granq_desc_t", "make_desc", "desc_of",
    "granq_workspace_bytes", "granq_plan_describe", "granq_range_reduce", "granq_range_reduce_noalloc", "granq_prescale", "granq_calibrate", "granq_calibrate_fakequant_fwd", "granq_conv1x1_int8_as", "granq_fakequant_fwd",
    "granq_fakequant_bwd", "load", "library_path", "status_string", "version",
    "granq_fold_weights", "granq_conv1x1_int8", "granq_conv1x1_int8_packed4", "granq_conv1x1_float", "granq_fakequant_fwd_packed4",
    "granq_packed4_bytes",
    "granq_distortion", "granq_distortion_workspace_bytes",
    "granq_calibrate_fakequant_fwd_resident", "granq_resident_state_bytes", "granq_resident_state_init",
    "granq_rowwise_fakequant_multi", "granq_rowwise_fakequant_bwd_multi", "rowwise_items",
    "rowwise_bwd_items", "granq_mask_bytes", "granq_fakequant_fwd_mask", "granq_fakequant_bwd_mask",
    "ActivationQuantizer", "granq_cmp_channel_loop_fwd", "granq_cmp_accumulate_inloop",
    "granq_cmp_accumulate_prescaled",
]
