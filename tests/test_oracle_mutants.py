"""Every plausible mistake planted in a copy of the oracle source must fail a pin.

The mistakes are planted in the oracle, on the CPU: the C file is copied with
one textual change, compiled with the oracle's own flags, and the pin suite is
run against the altered library.  A pin suite that lets one through does not
determine the oracle, so this test guards the pins themselves.
"""
import os

import pytest

from oracle import adama_oracle
from oracle_pins import ALL_PINS

SRC = os.path.join(os.path.dirname(adama_oracle.__file__), "adama_oracle.c")

# (name, text to find, replacement, which occurrence (0-based) or None for all)
MUTANTS = [
    ("fold_f64_no_square", "(1.0 - beta2) * (g * g)", "(1.0 - beta2) * g", 0),
    ("fold_f32_no_square", "(1.0 - beta2) * (g * g)", "(1.0 - beta2) * g", 1),
    ("fold_bf16_no_square", "(1.0 - beta2) * (g * g)", "(1.0 - beta2) * g", 2),
    ("fold_f16_no_square", "(1.0 - beta2) * (g * g)", "(1.0 - beta2) * g", 3),
    ("fold_f64_no_div_N", "double g = grad[k] / (double)N;", "double g = grad[k];", 0),
    ("fold_f32_no_div_N", "(double)grad[k] / (double)N", "(double)grad[k]", 0),
    ("fold_bf16_no_div_N", "adama_oracle_bf16_to_f64(grad[k]) / (double)N", "adama_oracle_bf16_to_f64(grad[k])", 0),
    ("fold_f16_no_div_N", "adama_oracle_f16_to_f64(grad[k]) / (double)N", "adama_oracle_f16_to_f64(grad[k])", 0),
    ("fold_v_div_N_once", "v[k] = v[k] + (1.0 - beta2) * (g * g);", "v[k] = v[k] + (1.0 - beta2) * (g * g) * (double)N;", None),
    ("fold_m_sign", "m[k] = m[k] + (1.0 - beta1) * g;", "m[k] = m[k] - (1.0 - beta1) * g;", None),
    ("fold_betas_swapped_m", "m[k] = m[k] + (1.0 - beta1) * g;", "m[k] = m[k] + (1.0 - beta2) * g;", None),
    ("fold_betas_swapped_v", "v[k] = v[k] + (1.0 - beta2) * (g * g);", "v[k] = v[k] + (1.0 - beta1) * (g * g);", None),
    ("fold_beta_not_complement", "m[k] = m[k] + (1.0 - beta1) * g;", "m[k] = m[k] + beta1 * g;", None),
    ("fold_overwrites_m", "m[k] = m[k] + (1.0 - beta1) * g;", "m[k] = (1.0 - beta1) * g;", None),
    ("decay_m_with_beta2", "m[k] = beta1 * m[k];", "m[k] = beta2 * m[k];", 0),
    ("decay_v_missing", "v[k] = beta2 * v[k];", "v[k] = v[k];", 0),
    ("decay_m_missing", "m[k] = beta1 * m[k];", "m[k] = m[k];", 0),
    ("apply_eps_inside_sqrt", "/ (sqrt(v_hat) + eps);", "/ sqrt(v_hat + eps);", 0),
    ("apply_no_sqrt", "/ (sqrt(v_hat) + eps);", "/ (v_hat + eps);", 0),
    ("apply_sign", "theta[k] = theta[k] - lr", "theta[k] = theta[k] + lr", 0),
    ("apply_no_bias1", "double m_hat = m[k] / bias1;", "double m_hat = m[k];", 0),
    ("apply_no_bias2", "double v_hat = v[k] / bias2;", "double v_hat = v[k];", 0),
    ("apply_bias_swapped", "double bias1 = 1.0 - pow(beta1, (double)t);", "double bias1 = 1.0 - pow(beta2, (double)t);", 0),
    ("apply_t_off_by_one", "double bias2 = 1.0 - pow(beta2, (double)t);", "double bias2 = 1.0 - pow(beta2, (double)(t + 1));", 0),
    ("apply_bias_multiplied", "double v_hat = v[k] / bias2;", "double v_hat = v[k] * bias2;", 0),
    ("apply_uses_raw_v", "/ (sqrt(v_hat) + eps);", "/ (sqrt(v[k]) + eps);", 0),
    ("alg1_variants_swapped", "variant ? sum_g2 : sum_g * sum_g", "variant ? sum_g * sum_g : sum_g2", 0),
    ("alg1_no_div_N", "grads[(size_t)i * n + k] / (double)N", "grads[(size_t)i * n + k]", 0),
    ("alg1_transposed", "grads[(size_t)i * n + k]", "grads[(size_t)k * N + i]", 0),
    ("ddp_v_div_M_once", "sum_v / ((double)M * (double)M)", "sum_v / (double)M", 0),
    ("ddp_m_not_averaged", "m_out[k] = sum_m / (double)M;", "m_out[k] = sum_m;", 0),
    ("f16_subnormal_scale", "ldexp((double)frac, -24)", "ldexp((double)frac, -25)", 0),
    ("f16_exponent_bias", "expo - 25", "expo - 24", 0),
    ("f16_hidden_bit", "(double)(1024 + frac)", "(double)(frac)", 0),
    ("f16_sign_dropped", "return sign ? -mag : mag;", "return mag;", 0),
    ("bf16_shift", "(uint32_t)bits << 16", "(uint32_t)bits << 15", 0),
    # variants: loss-scale factor, AdamW, momentum SGD
    ("widen_formats_swapped", "else if (gdt == 1)", "else if (gdt == 2 || gdt == 1)", 0),
    ("widen_f32_truncated", "out[k] = (double)((const float *)grad)[k];", "out[k] = (double)(int)((const float *)grad)[k];", 0),
    ("scaled_fold_scale_dropped", "double g = (grad_scale * grad[k]) / (double)N;", "double g = grad[k] / (double)N;", 0),
    ("scaled_fold_scale_inverted", "double g = (grad_scale * grad[k]) / (double)N;", "double g = (grad[k] / grad_scale) / (double)N;", 0),
    ("scaled_fold_no_div_N", "double g = (grad_scale * grad[k]) / (double)N;", "double g = (grad_scale * grad[k]);", 0),
    ("adamw_decay_sign", "theta[k] - decay - lr * m_hat", "theta[k] + decay - lr * m_hat", 0),
    ("adamw_decay_without_lr", "double decay = lr * weight_decay * theta[k];", "double decay = weight_decay * theta[k];", 0),
    ("adamw_decay_dropped", "theta[k] - decay - lr * m_hat", "theta[k] - lr * m_hat", 0),
    ("adamw_eps_inside_sqrt", "/ (sqrt(v_hat) + eps);", "/ sqrt(v_hat + eps);", 1),
    ("adamw_no_bias1", "double m_hat = m[k] / bias1;", "double m_hat = m[k];", 1),
    ("adamw_no_bias2", "double v_hat = v[k] / bias2;", "double v_hat = v[k];", 1),
    ("adamw_step_sign", "- decay - lr * m_hat", "- decay + lr * m_hat", 0),
    ("sgdm_decay_missing", "b[k] = mu * b[k];", "b[k] = b[k];", 0),
    ("sgdm_fold_overwrites", "b[k] = b[k] + g;", "b[k] = g;", 0),
    ("sgdm_fold_sign", "b[k] = b[k] + g;", "b[k] = b[k] - g;", 0),
    ("sgdm_fold_no_div_N", "double g = (grad_scale * grad[k]) / (double)N;", "double g = (grad_scale * grad[k]);", 1),
    ("sgdm_fold_scale_dropped", "double g = (grad_scale * grad[k]) / (double)N;", "double g = grad[k] / (double)N;", 1),
    ("sgdm_fold_dampened", "b[k] = b[k] + g;", "b[k] = b[k] + (1.0 - 0.9) * g;", 0),
    ("sgdm_apply_sign", "theta[k] - decay - lr * b[k];", "theta[k] - decay + lr * b[k];", 0),
    ("sgdm_apply_no_lr", "theta[k] - decay - lr * b[k];", "theta[k] - decay - b[k];", 0),
    ("sgdm_apply_decay_without_lr", "double decay = lr * weight_decay * theta[k];", "double decay = weight_decay * theta[k];", 1),
    ("adamw_zero_decay_forms_zero_times_theta", "if (weight_decay == 0.0) decay = 0.0;", "", 0),
    ("sgdm_zero_decay_forms_zero_times_theta", "if (weight_decay == 0.0) decay = 0.0;", "", 1),
    ("sgdm_apply_decay_sign", "theta[k] - decay - lr * b[k];", "theta[k] + decay - lr * b[k];", 0),
]


def _replace_nth(text, find, repl, nth):
    if nth is None:
        assert find in text, find
        return text.replace(find, repl)
    pos = -1
    for _ in range(nth + 1):
        pos = text.find(find, pos + 1)
        assert pos >= 0, f"{find!r} occurrence {nth} not in oracle source"
    return text[:pos] + repl + text[pos + len(find):]


@pytest.mark.parametrize("name,find,repl,nth", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(name, find, repl, nth, tmp_path):
    with open(SRC) as fh:
        text = fh.read()
    mutated = _replace_nth(text, find, repl, nth)
    assert mutated != text
    src = tmp_path / f"{name}.c"
    src.write_text(mutated)
    lib = adama_oracle.load(adama_oracle.build(force=True, src=str(src), out=str(tmp_path / f"{name}.so")))
    caught_by = None
    for pin in ALL_PINS:
        try:
            pin(lib)
        except AssertionError:
            caught_by = pin.__name__
            break
    assert caught_by is not None, f"planted mistake {name!r} passes every pin"
