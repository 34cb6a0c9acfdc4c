"""Sensitivity of the pins: plant one plausible mistake at a time in a copy of the oracle's C source
(on the CPU, in a temporary directory), rebuild it, and require that at least one pin fails.

This guards the pins, not the oracle: a pin suite that lets a dropped term, a wrong sign, a swapped
index or a transposed operand through would not be worth trusting.
"""
import os
import subprocess

import pytest

import oracle
from oracle_pins import ALL_PINS

SRC = os.path.join(os.path.dirname(oracle.__file__), "glow_oracle.c")

# (name, old text, new text, which occurrence: index or None for all)
MUTANTS = [
    ("flip_rows_f32", "- cs->pad_t + r;", "- cs->pad_t - r + cs->r - 1;", 0),
    ("flip_rows_int", "- cs->pad_t + r;", "- cs->pad_t - r + cs->r - 1;", 1),
    ("pad_sign_w_f32", "- cs->pad_l + s;", "+ cs->pad_l + s;", 0),
    ("pad_sign_w_int", "- cs->pad_l + s;", "+ cs->pad_l + s;", 1),
    ("ceil_out_dim", "return span / stride + 1;", "return (span + stride - 1) / stride + 1;", None),
    ("drop_bias_f32", "if (bias) acc += (double)bias[k];", "", None),
    ("drop_bias_int", "if (bias) acc += (int64_t)bias[k];", "", None),
    ("relu_inverted", "if (act == ORACLE_ACT_RELU && acc < 0.0) acc = 0.0;\n  return (float)acc;",
     "if (act == ORACLE_ACT_RELU && acc > 0.0) acc = 0.0;\n  return (float)acc;", None),
    ("relu_missing_fc", "if (act == ORACLE_ACT_RELU && acc < 0.0) acc = 0.0;\n      y[m * N + n]",
     "y[m * N + n]", None),
    ("filter_rs_swapped_f32", "((k * cs->r + r) * cs->s + s) * cg + cc", "((k * cs->s + s) * cs->r + r) * cg + cc", 0),
    ("filter_rs_swapped_int", "((k * cs->r + r) * cs->s + s) * cg + cc", "((k * cs->s + s) * cs->r + r) * cg + cc", 1),
    ("input_hw_swapped_f32", "((n * cs->h + ih) * cs->w + iw) * cs->c + c", "((n * cs->w + iw) * cs->h + ih) * cs->c + c", 0),
    ("input_hw_swapped_int", "((n * cs->h + ih) * cs->w + iw) * cs->c + c", "((n * cs->w + iw) * cs->h + ih) * cs->c + c", 1),
    ("stride_axes_swapped", "oh * cs->stride_h - cs->pad_t", "oh * cs->stride_w - cs->pad_t", 0),
    ("group_channel_base_f32", "const int64_t c = g * cg + cc;", "const int64_t c = cc;", 0),
    ("group_channel_base_int", "const int64_t c = g * cg + cc;", "const int64_t c = cc;", 1),
    ("fc_weight_transposed", "(double)w[k * N + n]", "(double)w[n * K + k]", None),
    ("fc_bias_index", "acc += (double)bias[n];", "acc += (double)bias[m];", None),
    ("qfc_weight_transposed", "(int64_t)w[k * N + n] - w_off", "(int64_t)w[n * K + k] - w_off", None),
    ("qfc_offset_sign", "(int64_t)a[m * K + k] - a_off", "(int64_t)a[m * K + k] + a_off", None),
    ("dequant_offset_sign", "((double)q[i] - (double)offset)", "((double)q[i] + (double)offset)", None),
    ("dequant_scale_divides", "(double)offset) * (double)scale;", "(double)offset) / (double)scale;", None),
    ("quantize_floor", "nearbyint(value[i] / (double)scale)", "floor(value[i] / (double)scale)", None),
    ("x_offset_ignored", "* cs->c + c] - x_off;", "* cs->c + c];", None),
    ("w_offset_ignored", "* cg + cc] - w_off;", "* cg + cc];", None),
    ("requant_truncates", "const int64_t half = (int64_t)1 << (shift - 1);", "const int64_t half = 0;", None),
    ("requant_rounds_to_zero", "if ((t % d) < 0) q -= 1;", "", None),
    ("requant_half_away", "const int64_t t = prod + half;", "const int64_t t = prod + (prod < 0 ? half - 1 : half);", None),
    ("requant_no_carry", "if (m == 2147483648LL) { m = 1073741824LL; e += 1; }", "", None),
    ("requant_shift_off_by_one", "const int sh = 31 - e;", "const int sh = 30 - e;", None),
    ("requant_mantissa_30_bits", "llround(f * 2147483648.0)", "2 * llround(f * 1073741824.0 / 32768.0) * 16384", None),
    ("requant_offset_before_scale", "q += y_offset;", "q -= y_offset;", None),
    ("no_upper_saturation", "if (q > 127) q = 127;", "", None),
    ("no_lower_saturation", "if (q < lo) q = lo;", "", None),
    ("relu_floor_is_zero", "if (act == ORACLE_ACT_RELU && y_offset > -128) return y_offset;",
     "if (act == ORACLE_ACT_RELU) return 0;", None),
    ("points_decode_swapped", "const int64_t ow = f % cs.ow; f /= cs.ow;\n    const int64_t oh = f % cs.oh; f /= cs.oh;\n    out[i] = conv_f32_one",
     "const int64_t oh = f % cs.oh; f /= cs.oh;\n    const int64_t ow = f % cs.ow; f /= cs.ow;\n    out[i] = conv_f32_one", None),
    ("addend_after_relu", "  if (addend) acc += (double)addend[((n * cs->oh + oh) * cs->ow + ow) * cs->k + k];\n"
     "  if (act == ORACLE_ACT_RELU && acc < 0.0) acc = 0.0;",
     "  if (act == ORACLE_ACT_RELU && acc < 0.0) acc = 0.0;\n"
     "  if (addend) acc += (double)addend[((n * cs->oh + oh) * cs->ow + ow) * cs->k + k];", None),
    ("addend_sign", "if (addend) acc += (double)addend[", "if (addend) acc -= (double)addend[", None),
    ("addend_index_transposed", "acc += (double)addend[((n * cs->oh + oh) * cs->ow + ow) * cs->k + k];",
     "acc += (double)addend[((n * cs->ow + ow) * cs->oh + oh) * cs->k + k];", None),
    ("rescale_inverted", "(double)sr / ((double)sx * (double)sw)", "((double)sx * (double)sw) / (double)sr", None),
    ("rescale_ignores_sw", "(double)sr / ((double)sx * (double)sw)", "(double)sr / (double)sx", None),
    ("rescale_offset_sign", "(int32_t)addend[o] - r_off", "(int32_t)addend[o] + r_off", None),
    ("rescale_truncates", "(int64_t)d * (int64_t)mant + ((int64_t)1 << (shift - 1));",
     "(int64_t)d * (int64_t)mant;", None),
    ("rescale_rounds_to_zero", "if ((t % den) < 0) q -= 1;", "", None),
    ("rescale_after_requantize", "acc += extra;", "", None),
    ("points_addend_index", "(int32_t)addend[flat_idx[i]] - r_off", "(int32_t)addend[i] - r_off", None),
    ("rescale_node_inverted", "oracle_requant_params(s_in, 1.0f, s_out, &mant, &shift);",
     "oracle_requant_params(s_out, 1.0f, s_in, &mant, &shift);", None),
    ("rescale_node_offset_sign", "(int32_t)in[i] - in_offset", "(int32_t)in[i] + in_offset", None),
    ("rescale_node_wrong_out_offset", "mant, shift, out_offset, -128);", "mant, shift, in_offset, -128);", None),
    ("overflow_unchecked", "if (s > INT32_MAX || s < INT32_MIN) { overflow |= 1; continue; }", "", None),
    # general chains
    ("chain_f32_add_dropped", "if (op->kind == ORACLE_OP_ADD_TENSOR) v += (double)((const float *)op->tensor)[o];",
     "if (op->kind == ORACLE_OP_ADD_TENSOR) v += 0.0;", None),
    ("chain_f32_order_reversed", "const oracle_chain_op *op = &ops[i];\n            if (op->kind == ORACLE_OP_ADD_TENSOR) v +=",
     "const oracle_chain_op *op = &ops[n_ops - 1 - i];\n            if (op->kind == ORACLE_OP_ADD_TENSOR) v +=", None),
    ("chain_f32_mul_adds", "v *= (double)op->a;", "v += (double)op->a;", None),
    ("chain_f32_max_is_min", "{ if (v < (double)op->a) v = (double)op->a; }", "{ if (v > (double)op->a) v = (double)op->a; }", None),
    ("chain_f32_clip_upper_ignored", "if (v > (double)op->b) v = (double)op->b; }", "}", None),
    ("chain_f32_bias_dropped", "if (bias) v += (double)bias[k];", "", None),
    ("chain_q_order_reversed", "const oracle_chain_op *op = &ops[i];\n            if (op->kind == ORACLE_OP_ADD_TENSOR) {\n              a +=",
     "const oracle_chain_op *op = &ops[n_ops - 1 - i];\n            if (op->kind == ORACLE_OP_ADD_TENSOR) {\n              a +=", None),
    ("chain_q_mul_keeps_scale", "s = s * (double)op->a;", "s = s;", None),
    ("chain_q_mul_divides", "s = s * (double)op->a;", "s = s / (double)op->a;", None),
    ("chain_q_threshold_truncates", "const double t = floor((double)v / s + 0.5);", "const double t = trunc((double)v / s);", None),
    ("chain_q_threshold_multiplies", "const double t = floor((double)v / s + 0.5);", "const double t = floor((double)v * s + 0.5);", None),
    ("chain_q_add_uses_initial_scale", "rc = multiplier_to_fixed((double)op->t_scale / s, &a_mant[i], &a_shift[i]);",
     "rc = multiplier_to_fixed((double)op->t_scale / ((double)sx * (double)sw), &a_mant[i], &a_shift[i]);", None),
    ("chain_q_add_offset_sign", "((const int8_t *)op->tensor)[o] - op->t_offset", "((const int8_t *)op->tensor)[o] + op->t_offset", None),
    ("chain_q_clip_upper_is_lower", "t_hi[i] = oracle_chain_threshold(op->b, s);", "t_hi[i] = oracle_chain_threshold(op->a, s);", None),
    ("chain_q_max_is_min", "} else if (op->kind == ORACLE_OP_MAX_SCALAR) {\n              if (a < t_lo[i]) a = t_lo[i];",
     "} else if (op->kind == ORACLE_OP_MAX_SCALAR) {\n              if (a > t_lo[i]) a = t_lo[i];", None),
    ("chain_q_final_scale_ignores_mul", "rc = multiplier_to_fixed(s / (double)sy, &mant, &shift);",
     "rc = multiplier_to_fixed((double)sx * (double)sw / (double)sy, &mant, &shift);", None),
    # batch-norm fold
    ("bnfold_mean_sign", "b_out[i] = (float)((b - (double)mean[i]) * scale + (double)beta[i]);",
     "b_out[i] = (float)((b + (double)mean[i]) * scale + (double)beta[i]);", None),
    ("bnfold_no_sqrt", "const double scale = (double)gamma[i] / sqrt((double)var[i] + (double)eps);",
     "const double scale = (double)gamma[i] / ((double)var[i] + (double)eps);", None),
    ("bnfold_beta_scaled", "b_out[i] = (float)((b - (double)mean[i]) * scale + (double)beta[i]);",
     "b_out[i] = (float)((b - (double)mean[i] + (double)beta[i]) * scale);", None),
    ("bnfold_filter_unscaled", "w_out[i * per + e] = (float)((double)w[i * per + e] * scale);",
     "w_out[i * per + e] = w[i * per + e];", None),
]


def _mutate(text, old, new, which):
    assert old in text, f"mutation anchor not found: {old!r}"
    if which is None:
        return text.replace(old, new)
    parts = text.split(old)
    assert len(parts) > which + 1, f"occurrence {which} of {old!r} missing"
    return old.join(parts[: which + 1]) + new + old.join(parts[which + 1:])


@pytest.mark.parametrize("name,old,new,which", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_mutant(tmp_path, name, old, new, which):
    src = open(SRC).read()
    mutated = _mutate(src, old, new, which)
    assert mutated != src
    c_path = tmp_path / f"{name}.c"
    so_path = tmp_path / f"lib{name}.so"
    c_path.write_text(mutated)
    subprocess.run(["gcc", "-std=c11", "-O1", "-fopenmp", "-fPIC", "-shared", "-w", "-o", str(so_path),
                    str(c_path), "-lm"], check=True)
    caught = []
    with oracle.use_library(str(so_path)):
        for pin in ALL_PINS:
            try:
                pin()
            except (AssertionError, oracle.OracleError):
                caught.append(pin.__name__)
                break
    assert caught, f"mutant {name} passes every pin"
