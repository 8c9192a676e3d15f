"""Are the oracle's pins tight?  Plant one plausible mistake at a time into a
COPY of the oracle's source (on the CPU, in a temp directory), build it, and
require that at least one pin in tests/oracle_pins.py fails for it.  The
committed oracle is never modified."""
import os

import pytest

import oracle
import oracle_pins

# (name, text in granq_oracle.c, replacement, how many occurrences are replaced; -1 = all)
MUTANTS = [
    ("zero_point_wrong_sign_in_code", "float v = t + z;", "float v = t - z;", 1),
    ("round_half_up", "return rintf(v);", "return floorf(v + 0.5f);", 1),
    ("round_truncates", "return rintf(v);", "return truncf(v);", 1),
    ("dequant_drops_zero_point", "float d = q - z;", "float d = q;", 1),
    ("dequant_adds_zero_point", "float d = q - z;", "float d = q + z;", 1),
    ("batch_and_channel_transposed", "(in * c + ic) * hw + k", "(ic * n + in) * hw + k", -1),
    ("range_over_first_sample_only",
     "float mx = -INFINITY;\n        for (int64_t in = 0; in < n; ++in) {",
     "float mx = -INFINITY;\n        for (int64_t in = 0; in < 1; ++in) {", 1),
    ("scale_drops_min", "float range = ch_max[ic] - ch_min[ic];", "float range = ch_max[ic];", 1),
    ("zero_point_sign", "rintf((-ch_min[ic]) / s)", "rintf((ch_min[ic]) / s)", 1),
    ("zero_point_not_rounded", "rintf((-ch_min[ic]) / s) + 0.0f", "(-ch_min[ic]) / s + 0.0f", 1),
    ("zero_point_keeps_minus_zero", "rintf((-ch_min[ic]) / s) + 0.0f", "rintf((-ch_min[ic]) / s)", 1),
    ("levels_off_by_one", "(float)((1 << bits) - 1)", "(float)(1 << bits)", 1),
    ("no_clamp", "return fminf(fmaxf(u, 0.0f), qmax);", "return u;", 1),
    ("clamp_low_side_missing", "return fminf(fmaxf(u, 0.0f), qmax);", "return fminf(u, qmax);", 1),
    ("mask_strict", "if (!(u >= 0.0f && u <= qmax))", "if (!(u > 0.0f && u < qmax))", 1),
    ("mask_on_clamped_code_always_true", "if (!(u >= 0.0f && u <= qmax))", "if (0)", 1),
    ("mask_inverted", "if (!(u >= 0.0f && u <= qmax))", "if ((u >= 0.0f && u <= qmax))", 1),
    ("degenerate_scale_not_replaced", "s = 1.0f;", "s = FLT_MIN;", 1),
    ("min_max_swapped", "ch_min[ic] = mn;\n        ch_max[ic] = mx;",
     "ch_min[ic] = mx;\n        ch_max[ic] = mn;", 1),
    ("multiply_instead_of_divide", "float t = x / s;", "float t = x * s;", 1),
    ("reciprocal_instead_of_divide", "float t = x / s;", "float t = x * (1.0f / s);", 1),
    ("double_precision_intermediate", "float t = x / s;\n    float v = t + z;\n    return rintf(v);",
     "double t = (double)x / s;\n    double v = t + z;\n    return (float)rint(v);", 1),
    ("fused_multiply_add", "float t = x / s;\n    float v = t + z;",
     "float v = fmaf(x, 1.0f / s, z);", 1),
    ("gate_bits_msb_first", "mask[i >> 3] |= (uint8_t)(1u << (i & 7));", "mask[i >> 3] |= (uint8_t)(0x80u >> (i & 7));", 1),
    ("gate_bits_strict", "if (u >= 0.0f && u <= qmax)\n                    mask[i >> 3]", "if (u > 0.0f && u < qmax)\n                    mask[i >> 3]", 1),
    ("bwd_from_mask_inverted", "if (!((mask[i >> 3] >> (i & 7)) & 1u))", "if (((mask[i >> 3] >> (i & 7)) & 1u))", 1),
    ("cosine_without_square_roots", "layer[4] = layer[0] / (sqrt(layer[1]) * sqrt(layer[2]));", "layer[4] = layer[0] / (layer[1] * layer[2]);", 1),
    ("relative_error_squared", "layer[5] = sqrt(layer[3]) / sqrt(layer[1]);", "layer[5] = layer[3] / layer[1];", 1),
    ("relative_error_over_q_norm", "layer[5] = sqrt(layer[3]) / sqrt(layer[1]);", "layer[5] = sqrt(layer[3]) / sqrt(layer[2]);", 1),
    ("distortion_difference_sign_lost", "double d = xd - qd;", "double d = xd + qd;", 1),
    ("distortion_single_precision_sums", "double xq = 0.0, xx = 0.0, qq = 0.0, dd = 0.0;", "float xq = 0.0, xx = 0.0, qq = 0.0, dd = 0.0;", 1),
    ("fold_forgets_activation_scale", "float ws = w[io * c + ic] * scale[ic];\n            if (fabsf(ws) > amax)", "float ws = w[io * c + ic];\n            if (fabsf(ws) > amax)", 1),
    ("fold_step_over_128", "float a = amax / 127.0f;", "float a = amax / 128.0f;", 1),
    ("fold_correction_sign", "cz += (int64_t)q * (int64_t)zero_point[ic];", "cz -= (int64_t)q * (int64_t)zero_point[ic];", 1),
    ("fold_correction_in_32_bits", "cz += (int64_t)q * (int64_t)zero_point[ic];", "cz = (int64_t)(int32_t)(uint32_t)(cz + (int64_t)q * (int64_t)zero_point[ic]);", 1),
    ("pack4_high_nibble_first", "packed[i] = (uint8_t)(lo | (hi << 4));", "packed[i] = (uint8_t)(hi | (lo << 4));", 1),
    ("pack4_odd_tail_repeats_last", "uint8_t hi = 2 * i + 1 < total ? codes[2 * i + 1] : 0;", "uint8_t hi = 2 * i + 1 < total ? codes[2 * i + 1] : codes[2 * i];", 1),
    ("unpack4_nibbles_swapped", "codes[i] = (i % 2 == 0) ? (uint8_t)(byte & 0x0F) : (uint8_t)(byte >> 4);", "codes[i] = (i % 2 == 1) ? (uint8_t)(byte & 0x0F) : (uint8_t)(byte >> 4);", 1),
    ("conv_correction_added", "(float)(acc - corr[io])", "(float)(acc + corr[io])", 1),
    ("conv_weights_transposed", "acc += (int64_t)wq[io * c + ic] * (int64_t)codes[(in * c + ic) * hw + k];", "acc += (int64_t)wq[ic * o + io] * (int64_t)codes[(in * c + ic) * hw + k];", 1),
    ("float_conv_weights_transposed", "double wd = (double)load_elem(w, io * c + ic, dtype);", "double wd = (double)load_elem(w, ic * o + io, dtype);", 1),
    ("float_conv_single_precision_sum", "double acc = 0.0;\n                for (int64_t ic = 0; ic < c; ++ic) {\n                    double wd", "float acc = 0.0;\n                for (int64_t ic = 0; ic < c; ++ic) {\n                    double wd", 1),
    ("float_conv_skips_first_channel", "for (int64_t ic = 0; ic < c; ++ic) {\n                    double wd", "for (int64_t ic = 1; ic < c; ++ic) {\n                    double wd", 1),
    ("float_conv_pixel_stride_is_channels", "double xd = (double)load_elem(x_hat, (in * c + ic) * hw + k, dtype);", "double xd = (double)load_elem(x_hat, (in * hw + k) * c + ic, dtype);", 1),
    ("bf16_ties_round_up", "(dropped == 0x8000u && (kept & 1u))", "(dropped == 0x8000u)", 1),
    ("bf16_truncates", "if (dropped > 0x8000u || (dropped == 0x8000u && (kept & 1u)))", "if (0)", 1),
    ("f16_ties_round_up", "double steps = rint(ldexp((double)a, 10 - e));", "double steps = floor(ldexp((double)a, 10 - e) + 0.5);", 1),
    ("f16_truncates", "double steps = rint(ldexp((double)a, 10 - e));", "double steps = floor(ldexp((double)a, 10 - e));", 1),
    ("f16_subnormals_flushed", "if (e < -14)\n        e = -14;", "if (e < -14)\n        return sign;", 1),
    ("f16_overflow_saturates", "if (e > 15)\n        return (uint16_t)(sign | 0x7C00u);", "if (e > 15)\n        return (uint16_t)(sign | 0x7BFFu);", 1),
    ("f16_widen_wrong_bias", "magnitude = ldexpf((float)(1024 + fraction), exponent - 25);", "magnitude = ldexpf((float)(1024 + fraction), exponent - 24);", 1),
    ("inloop_drops_scale", "float ws = weight[ic] * scale[ic];", "float ws = weight[ic];", 1),
    ("inloop_drops_zero_point", "- zero_point[ic];\n                float ws", ";\n                float ws", 1),
    ("prescaled_sum_skips_last_channel",
     "for (int64_t ic = 0; ic < c; ++ic) {\n                float term = weight[ic] * x_hat",
     "for (int64_t ic = 0; ic + 1 < c; ++ic) {\n                float term = weight[ic] * x_hat", 1),
]


def _first_failure(lib):
    for check in oracle_pins.ALL_CHECKS:
        try:
            check(lib)
        except AssertionError:
            return check.__name__
    return None


@pytest.mark.parametrize("name,old,new,count", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, old, new, count):
    src = open(os.path.join(os.path.dirname(oracle.__file__), "granq_oracle.c")).read()
    if count < 0:            # every occurrence, however many functions use the expression
        assert src.count(old) >= 3
    else:
        assert src.count(old) == count, "anchor text for %s not found exactly %d time(s)" % (name, count)
    mutated = tmp_path / "mutant.c"
    mutated.write_text(src.replace(old, new))
    so = str(tmp_path / "mutant.so")
    oracle.build(out=so, src=str(mutated), extra_flags=("-w",))
    lib = oracle.load(so)
    assert _first_failure(lib) is not None, "no pin notices the planted mistake %r" % name


def test_unmodified_copy_passes(tmp_path):
    """The harness itself: an unmutated copy built the same way passes every pin."""
    src = os.path.join(os.path.dirname(oracle.__file__), "granq_oracle.c")
    so = str(tmp_path / "copy.so")
    oracle.build(out=so, src=src)
    assert _first_failure(oracle.load(so)) is None
