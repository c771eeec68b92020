"""Do the pins bite?  Each case plants ONE plausible mistake in a copy of the oracle's
source (CPU only, in a temporary directory), builds it, and requires that at least one
of the pin tests fails on the broken build.  The committed oracle is never modified."""
import inspect
import os
import subprocess

import pytest

import test_oracle_quant_pins as quant_pins
import test_oracle_reduce_pins as reduce_pins
import test_oracle_recompute_pins as recompute_pins
import test_oracle_fp_pins as fp_pins
import test_oracle_nonfinite_pins as nonfinite_pins
import test_oracle_sr_pins as sr_pins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "agoq_ref.c")

# (name, text in the oracle source, replacement)
MUTANTS = [
    ("half_away_rounding", "r = rintf(t);", "r = roundf(t);"),
    ("truncation_instead_of_rounding", "r = rintf(t);", "r = truncf(t);"),
    ("inv_as_reciprocal_of_scale", "const float inv = fq / amax;", "const float inv = 1.0f / scale;"),
    ("scale_by_multiplying_reciprocal", "const float scale = amax / fq;",
     "const float scale = amax * (1.0f / fq);"),
    ("asymmetric_qmax", "return (1 << (bits - 1)) - 1;", "return (1 << (bits - 1));"),
    ("absmax_without_abs", "float a = fabsf(x[j]);", "float a = x[j];"),
    ("no_tiny_group_rule", "static const float REF_AMAX_MIN = 0x1p-100f;",
     "static const float REF_AMAX_MIN = 0.0f;"),
    ("nibbles_swapped", "put_code(codes, numel, g * group + j, bits, q[j]);",
     "put_code(codes, numel, (g * group + j) ^ 1, bits, q[j]);"),
    ("high_plane_at_wrong_offset", "uint8_t *high = codes + numel / 2;", "uint8_t *high = codes + numel / 4;"),
    ("five_bit_high_bits_reversed", "const int sh = (int)(i % 8);", "const int sh = 7 - (int)(i % 8);"),
    ("six_bit_fields_reversed", "const int sh = 2 * (int)(i % 4);", "const int sh = 6 - 2 * (int)(i % 4);"),
    ("decode_five_bit_ignores_high_plane", "field |= (uint32_t)((codes[numel / 2 + i / 8] >> (i % 8)) & 1u) << 4;",
     "field |= 0u;"),
    ("decode_six_bit_one_high_bit", "field |= (uint32_t)((codes[numel / 2 + i / 4] >> (2 * (i % 4))) & 3u) << 4;",
     "field |= (uint32_t)((codes[numel / 2 + i / 4] >> (2 * (i % 4))) & 1u) << 4;"),
    ("decode_without_sign_extension", "return (int)field - (1 << bits);", "return (int)field;"),
    ("bf16_by_truncation", "u += 0x7FFFu + lsb;", "u += 0u * lsb;"),
    ("bf16_ties_up", "u += 0x7FFFu + lsb;", "u += 0x8000u + 0u * lsb;"),
    ("reduce_two_roundings", "a = fmaf(c, s, a);", "a = a + c * s;"),
    ("reduce_reverse_order", "for (int k = 0; k < K; ++k) {\n                float c = (float)in_codes",
     "for (int k = K - 1; k >= 0; --k) {\n                float c = (float)in_codes"),
    ("reduce_wrong_scale_row", "float s = in_scales[k * stride_scales + g];",
     "float s = in_scales[g];"),
    ("reduce_codes_ignore_stride", "in_codes[k * stride_codes + g * group + j]",
     "in_codes[k * numel + g * group + j]"),
    ("accumulate_two_roundings", "acc[j] = fmaf((float)main_codes[i], s, add);",
     "acc[j] = (float)main_codes[i] * s + add;"),
    ("accumulate_drops_new_gradient", "acc[j] = fmaf((float)main_codes[i], s, add);",
     "acc[j] = fmaf((float)main_codes[i], s, 0.0f * add);"),
    ("rmsnorm_sum_instead_of_mean", "const double r = sqrt(ss / (double)cols + (double)eps);",
     "const double r = sqrt(ss + (double)eps);"),
    ("rmsnorm_eps_dropped", "const double r = sqrt(ss / (double)cols + (double)eps);",
     "const double r = sqrt(ss / (double)cols);"),
    ("rmsnorm_gamma_of_wrong_column", "y[e] = f32_to_bf16_bits((float)((double)gamma[j] * x / r));",
     "y[e] = f32_to_bf16_bits((float)((double)gamma[0] * x / r));"),
    ("rmsnorm_skips_bf16_rounding_of_input", "double x = (double)bf16_bits_to_f32(f32_to_bf16_bits(v));\n            ss += x * x;",
     "double x = (double)v;\n            ss += x * x;"),
    ("rmsnorm_fwd_gamma_squared", "(double)gamma[j] * v / rms));", "(double)gamma[j] * (double)gamma[j] * v / rms));"),
    ("rmsnorm_fwd_no_eps", "const double rms = sqrt(sumsq / (double)cols + (double)eps);",
     "const double rms = sqrt(sumsq / (double)cols);"),
    ("silu_fwd_plain_product", "z[e] = f32_to_bf16_bits((float)(up_v * gate_v / (1.0 + exp(-gate_v))));",
     "z[e] = f32_to_bf16_bits((float)(up_v * gate_v));"),
    ("silu_sigmoid_of_minus_gate", "z[e] = f32_to_bf16_bits((float)(u * g / (1.0 + exp(-g))));",
     "z[e] = f32_to_bf16_bits((float)(u * g / (1.0 + exp(g))));"),
    ("silu_applied_to_up", "z[e] = f32_to_bf16_bits((float)(u * g / (1.0 + exp(-g))));",
     "z[e] = f32_to_bf16_bits((float)(u * g / (1.0 + exp(-u))));"),
    ("fp_absmax_without_abs", "const float mag = fabsf(x[j]);", "const float mag = x[j];"),
    ("fp_ties_to_odd", "if (d < best_d || (d == best_d && (i % 2 == 0))) {",
     "if (d < best_d || (d == best_d && (i % 2 == 1))) {"),
    ("fp_ties_keep_lower", "if (d < best_d || (d == best_d && (i % 2 == 0))) {", "if (d < best_d) {"),
    ("e2m1_subnormal_step", "return 0.5f * (float)m;", "return 0.25f * (float)m;"),
    ("e2m1_exponent_bias", "return ldexpf(1.0f + 0.5f * (float)m, e - 1);", "return ldexpf(1.0f + 0.5f * (float)m, e);"),
    ("e4m3_exponent_bias", "return ldexpf(1.0f + (float)m / 8.0f, e - 7);", "return ldexpf(1.0f + (float)m / 8.0f, e - 8);"),
    ("e4m3_subnormal_scale", "return ldexpf((float)m, -9);", "return ldexpf((float)m, -10);"),
    ("fp_sign_dropped", "return (uint8_t)((signbit(t) ? 8 : 0) | idx);", "return (uint8_t)idx;"),
    ("fp8_sign_from_comparison", "return (uint8_t)((signbit(t) ? 0x80 : 0) | idx);",
     "return (uint8_t)((t < 0.0f ? 0x80 : 0) | idx);"),
    ("fp4_vmax_is_8", "const int live = fp_group_scale(xf, group, 6.0f, &scale, &inv);",
     "const int live = fp_group_scale(xf, group, 8.0f, &scale, &inv);"),
    ("fp4_dead_group_keeps_signs", "const uint8_t lo = live ? e2m1_encode(xf[j] * inv) : 0;",
     "const uint8_t lo = e2m1_encode(xf[j] * inv);"),
    ("fp4_nibbles_swapped", "codes[(g * group + j) / 2] = (uint8_t)(lo | (hi << 4));",
     "codes[(g * group + j) / 2] = (uint8_t)(hi | (lo << 4));"),
    ("fp8_reduce_two_roundings", "a = fmaf(v, in_scales[k * stride_scales + g], a);",
     "a = a + v * in_scales[k * stride_scales + g];"),
    ("fp8_reduce_ignores_stride", "const float v = e4m3_decode(in_codes[k * stride_codes + e]);",
     "const float v = e4m3_decode(in_codes[k * numel + e]);"),
    ("fp8_accumulate_two_roundings", "acc[j] = fmaf(e4m3_decode(main_codes[i]), main_scales[g], addend);",
     "acc[j] = e4m3_decode(main_codes[i]) * main_scales[g] + addend;"),
    ("fp8_accumulate_drops_addend", "acc[j] = fmaf(e4m3_decode(main_codes[i]), main_scales[g], addend);",
     "acc[j] = fmaf(e4m3_decode(main_codes[i]), main_scales[g], 0.0f * addend);"),
    ("dbca_printed_index", "return 3 * n_stages - 2 * stage + 1;", "return n_stages + 2 * stage - 1;"),
    ("dbca_floor_instead_of_round", "int r = (int)floor(b + 0.5);", "int r = (int)floor(b);"),
    ("dbca_no_cap", "if (r > 8)\n        r = 8;", ""),
    ("nonfinite_group_quantized_like_any_other", "if (!group_is_finite(x, G)) { /* Inf or NaN anywhere",
     "if (0) { /* Inf or NaN anywhere"),
    ("only_nan_counts_as_nonfinite", "if (!isfinite(x[j]))", "if (isnan(x[j]))"),
    ("only_inf_counts_as_nonfinite", "if (!isfinite(x[j]))", "if (isinf(x[j]))"),
    ("nonfinite_group_gets_scale_zero", "            q[j] = 0;\n        return quiet_nan();", "            q[j] = 0;\n        return 0.0f;"),
    ("fp_nonfinite_group_keeps_codes", "        *scale = quiet_nan();\n        *inv = 0.0f;\n        return 0;",
     "        *scale = quiet_nan();\n        *inv = 0.0f;\n        return 1;"),
    ("fp_nonfinite_group_not_detected", "    if (!group_is_finite(x, G)) {\n        *scale = quiet_nan();", "    if (0) {\n        *scale = quiet_nan();"),
    ("bf16_nan_rounded_like_a_number", "    if (isnan(f))\n        return 0x7FC0u;\n", ""),
    ("sr_rounds_to_nearest_after_the_shift", "r = floorf(shifted);", "r = rintf(shifted);"),
    ("sr_variate_subtracted", "float shifted = t + sr_u(mode.seed, first_index + j);",
     "float shifted = t - sr_u(mode.seed, first_index + j);"),
    ("sr_variate_ignores_the_group_offset", "float shifted = t + sr_u(mode.seed, first_index + j);",
     "float shifted = t + sr_u(mode.seed, j);"),
    ("sr_one_word_per_element", "const uint32_t word = sr_word(seed, (uint64_t)i >> 2);",
     "const uint32_t word = sr_word(seed, (uint64_t)i);"),
    ("sr_bytes_taken_from_the_top", "const uint32_t byte = (word >> (8 * (int)(i & 3))) & 0xFFu;",
     "const uint32_t byte = (word >> (24 - 8 * (int)(i & 3))) & 0xFFu;"),
    ("sr_variate_can_reach_one", "return (float)byte / 256.0f;", "return (float)byte / 255.0f;"),
    ("sr_first_multiplier_off", "h *= 0x85EBCA6Bu;", "h *= 0x85EBCA6Du;"),
    ("sr_middle_shift_off", "h ^= h >> 13;", "h ^= h >> 15;"),
    ("sr_seed_not_mixed", "const uint32_t key = sr_mix(seed ^ (hi * 0x9E3779B9u));",
     "const uint32_t key = seed ^ (hi * 0x9E3779B9u);"),
    ("sr_high_half_of_the_counter_ignored", "const uint32_t key = sr_mix(seed ^ (hi * 0x9E3779B9u));",
     "const uint32_t key = sr_mix(seed);"),
    ("sr_reduce_rounds_to_nearest", "return grad_reduce_any(in_codes, stride_codes, in_scales, stride_scales, K, numel, group, mode,",
     "return grad_reduce_any(in_codes, stride_codes, in_scales, stride_scales, K, numel, group, ROUND_NEAREST,"),
    ("sr_accumulate_drops_the_seed", "    const struct rounding mode = {1, seed};\n    return grad_accumulate_any(",
     "    const struct rounding mode = {1, 0};\n    return grad_accumulate_any("),
    ("sr_store_ignores_the_mode", "scales[g] = quantize_group(grad + g * group, group, 127, q, mode, g * group);",
     "scales[g] = quantize_group(grad + g * group, group, 127, q, ROUND_NEAREST, g * group);"),
    ("dequant_uses_previous_group_scale", "const float s = scales[g];\n        for (int j = 0; j < group; ++j) {\n            float v",
     "const float s = scales[g > 0 ? g - 1 : 0];\n        for (int j = 0; j < group; ++j) {\n            float v"),
]


def pin_tests():
    """Every pin test of the two pin modules, expanded over its parametrisation."""
    cases = []
    for mod in (quant_pins, reduce_pins, recompute_pins, fp_pins, nonfinite_pins, sr_pins):
        for name, fn in inspect.getmembers(mod, inspect.isfunction):
            if not name.startswith("test_") or "ref" not in inspect.signature(fn).parameters:
                continue
            grids = [{}]
            for mark in getattr(fn, "pytestmark", []):
                if mark.name != "parametrize":
                    continue
                names = [n.strip() for n in mark.args[0].split(",")]
                new = []
                for g in grids:
                    for val in mark.args[1]:
                        vals = val if len(names) > 1 else (val,)
                        new.append({**g, **dict(zip(names, vals))})
                grids = new
            cases += [(fn, g) for g in grids]
    return cases


def killed_by(oracle_obj, first=None):
    """The first pin test that fails on this oracle build (None: all pass).  `first`: the pin
    module to try before the others (the one written for the mutated function: saves running
    every other module's pins, which pass, before the one that bites)."""
    cases = pin_tests()
    if first is not None:
        cases.sort(key=lambda case: case[0].__module__ != first.__name__)
    for fn, kwargs in cases:
        try:
            fn(ref=oracle_obj, **kwargs)
        except Exception as exc:  # an assertion, or the oracle rejecting / mangling a call
            return "%s%s: %s" % (fn.__name__, kwargs or "", type(exc).__name__)
    return None


def test_pins_pass_on_the_unmodified_source(tmp_path, ref):
    assert killed_by(ref.Oracle()) is None


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, ref, name, old, new):
    import warnings
    text = open(SRC).read()
    assert text.count(old) == 1, "mutation site must be unique: %r" % old
    src = tmp_path / "mutant.c"
    src.write_text(text.replace(old, new))
    lib = tmp_path / ("libmutant_%s.so" % name)
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
                           "-w", "-shared", "-fPIC", "-o", str(lib), str(src), "-lm"])
    with warnings.catch_warnings():
        warnings.simplefilter("ignore")
        verdict = killed_by(ref.Oracle(str(lib)), first=sr_pins if name.startswith("sr_") else None)
    assert verdict is not None, "no pin noticed the planted mistake %r" % name
