// Functions shared between the library's translation units (not part of the C ABI).
#pragma once

#include <stddef.h>
#include <stdint.h>

#include "granq.h"

namespace granq {

// True if granq_calibrate_fakequant_fwd can take its two-launch form for this tensor and these
// pointers (first pass of the reduction; forward whose leading blocks finish the reduction).
bool two_launches_apply(const void *x, const granq_desc_t *desc, const void *x_hat,
                        const uint8_t *codes_or_null);

// That form.  Precondition: two_launches_apply().  The status is that of the whole call: all
// argument checks of granq_calibrate and granq_fakequant_fwd come before the first launch.
granq_status_t calibrate_fwd_two_launches(const void *x, const granq_desc_t *desc, int bits, float *ch_min,
                                          float *ch_max, float *scale, float *zero_point, void *x_hat,
                                          uint8_t *codes_or_null, void *workspace, size_t workspace_bytes,
                                          void *stream);

// Launches granq_calibrate_fakequant_fwd makes for this descriptor with 16-byte-aligned
// pointers: 1 (a block per channel), 2 or 3.
int one_call_forward_launches(const granq_desc_t *desc);

}  // namespace granq
