"""Are the oracle's pins sharp?  Each case plants one plausible mistake in a COPY of the oracle's C
source (on the CPU, in a temporary directory), builds it, and requires that at least one of the
pin tests in test_oracle_pins.py fails against the mutated build.  A mutation that survives
means a part of the oracle is pinned to nothing."""
import os
import subprocess

import pytest

import oracle
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(os.path.abspath(oracle.__file__)), "adamw_oracle.c")

MUTATIONS = {
    "eps_inside_root": ("(sqrt(vn / bc2) + eps)", "(sqrt(vn / bc2 + eps))"),
    "no_bias_correction_m": ("(mn / bc1)", "(mn)"),
    "no_bias_correction_v": ("sqrt(vn / bc2)", "sqrt(vn)"),
    "bias_exponent_off_by_one": ("double bc2 = 1.0 - pow(b2, (double)step);", "double bc2 = 1.0 - pow(b2, (double)step + 1.0);"),
    "update_sign": ("double pn = p - lr *", "double pn = p + lr *"),
    "betas_swapped_in_m": ("b1 * (double)exp_avg[i] + (1.0 - b1) * g;", "(1.0 - b1) * (double)exp_avg[i] + b1 * g;"),
    "betas_swapped_in_v": ("b2 * (double)exp_avg_sq[i] + (1.0 - b2) * (g * g);", "(1.0 - b2) * (double)exp_avg_sq[i] + b2 * (g * g);"),
    "v_uses_g_not_g2": ("(1.0 - b2) * (g * g);", "(1.0 - b2) * g;"),
    "m_and_v_outputs_swapped": ("exp_avg[i] = (float)mn;\n        exp_avg_sq[i] = (float)vn;", "exp_avg[i] = (float)vn;\n        exp_avg_sq[i] = (float)mn;"),
    "decay_scaled_twice": ("+ wd * p);", "+ wd * lr * p);"),
    "decay_dropped": ("+ wd * p);", ");"),
    "clip_not_clamped": ("return c < 1.0 ? c : 1.0;", "return c;"),
    "clip_guard_missing": ("double c = (double)max_grad_norm / (norm + 1e-6);", "double c = (double)max_grad_norm / norm;"),
    "clip_uses_squared_norm": ("double c = (double)max_grad_norm / (norm + 1e-6);", "double c = (double)max_grad_norm / (norm * norm + 1e-6);"),
    "unscale_forgotten_in_step": ("oracle_lowp_decode(grad[i], dtype) * inv * coef;", "oracle_lowp_decode(grad[i], dtype) * coef;"),
    "unscale_multiplies": ("void oracle_grad_accumulate(const uint16_t *grad, uint64_t numel, int dtype, float loss_scale,\n                            double *sumsq, uint32_t *found_inf)\n{\n    double inv = 1.0 / (double)loss_scale;",
                           "void oracle_grad_accumulate(const uint16_t *grad, uint64_t numel, int dtype, float loss_scale,\n                            double *sumsq, uint32_t *found_inf)\n{\n    double inv = (double)loss_scale;"),
    "norm_sums_abs": ("else s += x * x;", "else s += fabs(x);"),
    "norm_without_root": ("*norm = flag ? NAN : sqrt(sumsq);", "*norm = flag ? NAN : sumsq;"),
    # (dropping only the per-element test is an equivalent program: the non-finite value then poisons
    # the sum, which the finish step flags; the real mistake is to drop the value silently)
    "nonfinite_silently_dropped": ("if (!isfinite(x)) flag = 1;\n        else s += x * x;", "if (isfinite(x)) s += x * x;"),
    "skip_not_honoured": ("    if (found_inf) return;\n    double inv", "    if (0) return;\n    double inv"),
    "nonfinite_extra_ignored": ("uint32_t flag = found_inf_in || !isfinite(sumsq);", "uint32_t flag = found_inf_in;"),
    "encode_truncates": ("double n = rint(a / q);", "double n = floor(a / q);"),
    "encode_rounds_half_up": ("double n = rint(a / q);", "double n = floor(a / q + 0.5);"),
    "lowp_from_old_master": ("param_lp[i] = oracle_lowp_encode((float)pn, dtype);", "param_lp[i] = oracle_lowp_encode((float)p, dtype);"),
    "fp16_bias_wrong": ("else mag = ldexp(1024.0 + f, e - 15 - 10);", "else mag = ldexp(1024.0 + f, e - 16 - 10);"),
    "fp16_subnormals_flushed": ("if (e < emin) e = emin;", "if (e < emin) return (uint16_t)(sign << 15);"),
    "bf16_mantissa_width": ("return encode_grid((double)x, 7, -126, 127, 127);", "return encode_grid((double)x, 8, -126, 127, 127);"),
    "cast_truncates": ("param_lp[i] = oracle_lowp_encode(master[i], dtype);", "param_lp[i] = (uint16_t)(oracle_lowp_encode(master[i], dtype) & 0xFFFEu);"),
    "no_writeback_variant_still_skips_master": ("        if (param_lp) param_lp[i] = oracle_lowp_encode((float)pn, dtype);", "        if (param_lp) param_lp[i] = oracle_lowp_encode((float)pn, dtype); else master[i] = (float)p;"),
    "layout_one_chunk_too_many": ("while (nc * chunk_elems < off) ++nc;", "while (nc * chunk_elems <= off) ++nc;"),
    "layout_offsets_inclusive": ("        tensor_offset[t] = off;\n        off += tensor_numel[t];", "        off += tensor_numel[t];\n        tensor_offset[t] = off;"),
}

# cheap pins first; each mutation stops at the first pin that fails
BATTERY = [pins.test_hand_worked_examples, pins.test_split_path_equals_fused_and_cast_is_library_rne, pins.test_zero_gradient_is_pure_decay, pins.test_step1_is_lr_sign_g,
           pins.test_norm_closed_forms, pins.test_nonfinite_extra_sumsq_sets_flag, pins.test_clip_invariants,
           pins.test_chunk_layout_against_cumsum_and_counts, pins.test_decode_all_patterns_match_numpy_and_torch,
           pins.test_encode_roundtrip_all_patterns, pins.test_constant_gradient_closed_form_every_t,
           pins.test_padding_stays_zero, pins.test_loss_scale_invariance_bit_exact,
           lambda: pins.test_nonfinite_sets_flag_and_skips_bit_exactly(oracle.BF16, float("inf"), 511),
           lambda: pins.test_nonfinite_sets_flag_and_skips_bit_exactly(oracle.FP16, float("-inf"), 0),
           lambda: pins.test_against_torch_adamw_fp64(oracle.BF16),
           pins.test_bf16_rne_against_torch_on_ties_and_neighbours,
           pins.test_fp16_rne_against_numpy_incl_subnormals_and_overflow]


def test_every_mutation_target_exists_in_the_source():
    text = open(SRC).read()
    for name, (old, _new) in MUTATIONS.items():
        assert text.count(old) == 1, name


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name, tmp_path, monkeypatch):
    old, new = MUTATIONS[name]
    text = open(SRC).read()
    assert text.count(old) == 1
    src = tmp_path / "mutant.c"
    so = tmp_path / "libmutant.so"
    src.write_text(text.replace(old, new))
    subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-o", str(so), str(src), "-lm"])
    monkeypatch.setattr(oracle, "_lib", oracle.bind(str(so)))
    caught = None
    for pin in BATTERY:
        try:
            pin()
        except (AssertionError, ValueError, FloatingPointError, ZeroDivisionError):
            caught = getattr(pin, "__name__", "pin")
            break
    assert caught, "mutation %r survived every pin" % name
