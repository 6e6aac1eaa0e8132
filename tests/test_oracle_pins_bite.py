"""The pins must bite: plant one plausible mistake at a time in a copy of the
oracle's C source (on the CPU, in a temporary directory), load the mutated
library in place of the real one and check that at least one pin fails."""
import ctypes
import os
import subprocess

import pytest

import oracle
from tests import test_oracle_adam as A
from tests import test_oracle_cast_unshard as C

SRC = os.path.join(os.path.dirname(oracle.__file__), "zc_oracle.c")

MUTATIONS = {
    "eps_inside_sqrt": ("/ (sqrt(v_hat) + eps));", "/ sqrt(v_hat + eps));"),
    "no_bias_correction_1": ("const double bc1 = 1.0 - pow(beta1, (double)step);", "const double bc1 = 1.0;"),
    "no_bias_correction_2": ("const double bc2 = 1.0 - pow(beta2, (double)step);", "const double bc2 = 1.0;"),
    "step_off_by_one": ("const double bc1 = 1.0 - pow(beta1, (double)step);",
                        "const double bc1 = 1.0 - pow(beta1, (double)(step + 1));"),
    "wrong_sign": ("p_dec - lr * m_hat", "p_dec + lr * m_hat"),
    "v_without_square": ("(1.0 - beta2) * gi * gi", "(1.0 - beta2) * gi"),
    "m_coefficients_swapped": ("beta1 * (double)m[i] + (1.0 - beta1) * gi",
                               "(1.0 - beta1) * (double)m[i] + beta1 * gi"),
    "decay_not_scaled_by_lr": ("p_dec = p_old * (1.0 - lr * wd);", "p_dec = p_old * (1.0 - wd);"),
    "l2_ignores_wd": ("gi += wd * p_old;", "gi += 0.0 * p_old;"),
    "decay_in_both_modes": ("        if (mode == ZCO_ADAMW)\n            p_dec", "        if (1)\n            p_dec"),
    "update_uses_old_m": ("const double m_hat = (double)m[i] / bc1;",
                          "const double m_hat = ((double)m[i] - (1.0 - beta1) * gi) / beta1 / bc1;"),
    "ties_away_from_zero": ("bits += 0x7FFFu + kept_lsb;", "bits += 0x8000u;"),
    "truncation": ("bits += 0x7FFFu + kept_lsb;", "bits += 0u;"),
    "nan_not_handled": ("(bits & 0x7FFFFFFFu) > 0x7F800000u", "(bits & 0x7FFFFFFFu) > 0xFFFFFFFFu"),
    "unshard_reversed": ("dst[s][j] = gathered[src_offset[s] + j];",
                         "dst[s][numel[s] - 1 - j] = gathered[src_offset[s] + j];"),
    "unshard_ignores_offset": ("= gathered[src_offset[s] + j];", "= gathered[j];"),
    "grad_scale_ignored": ("gi *= grad_scale;", "gi *= 1.0;"),
    "inf_not_flagged": ("if (!isfinite(gi))", "if (isnan(gi))"),
    "upcast_shift": ("zco_bits_to_f32((uint32_t)b << 16)", "zco_bits_to_f32((uint32_t)b << 15)"),
    "skip_ignored": ("    if (skip)\n        return;", "    if (0)\n        return;"),
    "bf16_from_old_p": ("bf16_out[i] = zco_rne_bf16(p[i]);", "bf16_out[i] = zco_rne_bf16((float)p_old);"),
    "bf16_grads_wrong_index": ("        double gi = g_is_bf16 ? (double)zco_bf16_to_f32(g16[i])",
                               "        double gi = g_is_bf16 ? (double)zco_bf16_to_f32(g16[i / 2])"),
    "sqnorm_not_squared": ("acc += gi * gi;", "acc += gi;"),
    "clip_without_sqrt": ("const double norm = sqrt((double)sqnorm) * (double)inv_loss_scale;",
                          "const double norm = (double)sqnorm * (double)inv_loss_scale;"),
    "clip_never_clamps": ("        if (coef > 1.0)\n            coef = 1.0;", "        if (0)\n            coef = 1.0;"),
    "clip_forgets_loss_scale": ("return (float)((double)inv_loss_scale * coef);", "return (float)coef;"),
    "accumulate_overwrites": ("acc[i] = (float)((double)acc[i] + gi * scale);",
                              "acc[i] = (float)(gi * scale);"),
    # the all-fp32 second-opinion build
    "f32_no_bias_correction_2": ("const float denom_a = root * inv_sqrt_bc2;", "const float denom_a = root;"),
    "f32_wrong_sign": ("const float p_new = p_dec - delta;", "const float p_new = p_dec + delta;"),
    "f32_v_without_square": ("const float v_c = v_b * gi;", "const float v_c = v_b;"),
    "f32_eps_dropped": ("const float denom = denom_a + eps_f;", "const float denom = denom_a;"),
    "f32_decay_dropped": ("p_dec = p_old - shrink;", "p_dec = p_old;"),
    "f32_m_uses_beta2": ("const float m_a = beta1_f * m[i];", "const float m_a = beta2_f * m[i];"),
    "f32_skip_ignored": ("    if (skip != 0)\n        return;", "    if (0)\n        return;"),
    "accumulate_ignores_scale": ("acc[i] = (float)((double)acc[i] + gi * scale);",
                                 "acc[i] = (float)((double)acc[i] + gi);"),
}

PINS = [
    A.test_step1_is_lr_sign_g, A.test_step1_sign_and_direction, A.test_zero_grad_pure_decay_adamw,
    A.test_zero_grad_l2_mode_is_not_pure_decay, A.test_wd_zero_modes_agree,
    lambda: A.test_constant_gradient_closed_form(10), A.test_bias_correction_uses_step_argument,
    lambda: A.test_decimal_brute_force(1, False), lambda: A.test_decimal_brute_force(7, True),
    A.test_hand_computed_single_element, lambda: A.test_against_torch_adamw_fp64(0.01),
    A.test_against_torch_adam_l2_fp64, A.test_elementwise_independence_and_split_calls,
    A.test_bf16_grads_equal_upcast_fp32_grads, A.test_grad_scale_is_premultiplication,
    A.test_skip_touches_nothing_and_bf16_out_is_cast_of_p, A.test_nan_gradient_poisons_only_its_element,
    A.test_padding_stays_zero, A.test_grad_accumulate_closed_forms, A.test_clip_scale_closed_forms,
    A.test_groups_no_decay_range_and_lr_scale, A.test_offload_definition_is_concatenation, A.test_grad_sqnorm,
    A.test_all_fp32_build_step1_closed_form,
    lambda: A.test_all_fp32_build_stays_within_a_few_ulp_of_the_double_build(oracle.ADAMW, False),
    lambda: A.test_all_fp32_build_stays_within_a_few_ulp_of_the_double_build(oracle.ADAM_L2, True),
    A.test_all_fp32_build_skip_and_fused_cast,
    C.test_all_bf16_values_round_trip, C.test_every_tie_goes_to_even, C.test_special_values,
    C.test_nearest_value_property_on_random_bits, C.test_library_conversion_agrees,
    C.test_unshard_brute_force_ragged, C.test_unshard_hash_property_and_ranks_spanned,
]


def failing_pins():
    failed = []
    for pin in PINS:
        try:
            pin()
        except Exception as e:          # AssertionError, or a crash of the comparison itself
            failed.append((getattr(pin, "__name__", "lambda"), type(e).__name__))
    return failed


def test_unmutated_oracle_passes_every_pin():
    assert failing_pins() == []


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name, tmp_path):
    old, new = MUTATIONS[name]
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation anchor for {name} must occur exactly once (code, not comment)"
    mutated = tmp_path / "zc_oracle_mut.c"
    mutated.write_text(text.replace(old, new, 1))
    lib_path = tmp_path / "libmut.so"
    subprocess.check_call(["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fPIC", "-shared",
                           "-o", str(lib_path), str(mutated), "-lm"])
    real = oracle._load()
    oracle._lib = oracle._prepare(ctypes.CDLL(str(lib_path)))
    try:
        failed = failing_pins()
    finally:
        oracle._lib = real
    assert failed, f"no pin noticed the planted mistake '{name}'"
