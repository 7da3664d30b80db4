"""Do the pins have teeth?  Plant one plausible mistake at a time in a COPY of the
oracle's source (on the CPU, in a temporary directory), build it, and require that
at least one pin of tests/pins.py fails.  The real oracle is never modified.
"""
import os
import shutil

import pytest

import oracle
import pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "loco_ref.c")
MT = os.path.join(os.path.dirname(oracle.__file__), "loco_ref_mt.c")

# (name, text in loco_ref.c, replacement[, which occurrence: 0 = block-scaled form, 1 = fixed-scale form])
MUTANTS = [
    ("compensation_sign", "grad_at(grad, grad_dtype, i) + e; /* Eq. 2 */", "grad_at(grad, grad_dtype, i) - e;"),
    ("error_sign", "float delta = h - d;", "float delta = d - h;"),
    ("ema_weights_swapped", "fmaf(one_minus_beta, e, bd)", "fmaf(beta, e, one_minus_beta * delta)"),
    ("ema_history_dropped", "fmaf(one_minus_beta, e, bd)", "bd"),
    ("ema_not_weighted", "float bd = beta * delta;", "float bd = delta;"),
    ("scale_uses_2_pow_p_minus_1", "amax / (float)qmax;", "amax / (float)(qmax + 1);"),
    ("truncate_instead_of_round", "(int)rintf(h * r);", "(int)truncf(h * r);"),
    ("round_half_away", "(int)rintf(h * r);", "(int)roundf(h * r);"),
    ("max_without_abs", "float ah = fabsf(h);", "float ah = h;"),
    ("nibble_order", "codes_out[i >> 1] = (uint8_t)(codes_out[i >> 1] | ((q & 15) << 4));",
     "codes_out[i >> 1] = (uint8_t)((codes_out[i >> 1] << 4) | (q & 15));"),
    ("unsigned_nibble_decode", "return (nib ^ 8) - 8;", "return nib;"),
    ("no_average", "grad_out[i] = acc * inv;", "grad_out[i] = acc;"),
    ("reset_ignored", "reset ? 0.0f : fmaf", "0 ? 0.0f : fmaf"),
    ("reset_schedule_off_by_one", "return remainder == 0;", "return remainder == reset_period - 1;"),
    ("reset_schedule_skips_step_zero", "return remainder == 0;", "return remainder == 0 && step_index != 0;"),
    ("reset_schedule_every_step", "long long remainder = step_index % reset_period;", "long long remainder = 0;"),
    ("bf16_shift", "[i] << 16;", "[i] << 15;"),
    ("worker_scale_stride", "scales[(size_t)w * scale_stride_elems + b]", "scales[b]"),
    ("worker_code_stride", "codes + (size_t)w * code_stride_bytes", "codes"),
    ("subnormal_step_kept", "int dead = D < FLT_MIN;", "int dead = D <= 0.0f;"),
    ("state_not_compensated_in_max", "float h = grad_at(grad, grad_dtype, i) + err_state[i];",
     "float h = grad_at(grad, grad_dtype, i);"),
    ("decode_with_reciprocal", "float d = (float)q * D;   /* decompressor, Eq. 1 */",
     "float d = (float)q * r;"),
    # the paper's literal form (global scale, 8-bit state)
    ("fixed_ema_not_weighted", "float bd = beta * delta;", "float bd = delta;", 1),
    ("fixed_error_sign", "float delta = h - d;", "float delta = d - h;", 1),
    ("fixed_state_not_decoded", "float e_hat = (float)err_state8[i] / s_e;", "float e_hat = (float)err_state8[i];"),
    ("fixed_state_scale_is_s", "const float s_e = (float)se_mult * s;", "const float s_e = s;"),
    ("fixed_ema_weights_swapped", "fmaf(one_minus_beta, e_hat, bd)", "fmaf(beta, e_hat, one_minus_beta * delta)"),
    ("fixed_ema_history_dropped", "fmaf(one_minus_beta, e_hat, bd)", "bd"),
    ("fixed_state_not_rescaled", "clamp_round(e_new * s_e, -128, 127)", "clamp_round(e_new, -128, 127)"),
    ("fixed_state_wraps", "(int)clamp_round(e_new * s_e, -128, 127)", "(int)(int8_t)(int)rintf(e_new * s_e)"),
    ("fixed_no_clamp_low", "if (t < (float)lo)", "if (0)"),
    ("fixed_truncates", "float t = rintf(x);", "float t = truncf(x);"),
    ("fixed_compensation_dropped", "grad_at(grad, grad_dtype, i) + e_hat;", "grad_at(grad, grad_dtype, i);"),
    ("fixed_decode_scale", "float d = (float)q / s;                              /* decompressor(q; s) */",
     "float d = (float)q / s_e;"),
    ("fixed_reset_ignored", "int e8 = reset ? 0 :", "int e8 = 0 ? 0 :"),
    ("fixed_reduce_no_average", "grad_out[i] = acc * inv;", "grad_out[i] = acc;", 1),
    # global scale with the state kept in high precision
    ("f32state_compensation_dropped", "grad_at(grad, grad_dtype, i) + e_old;", "grad_at(grad, grad_dtype, i);"),
    ("f32state_error_sign", "float raw_err = h - d_own;", "float raw_err = d_own - h;"),
    ("f32state_ema_not_weighted", "float weighted = beta * raw_err;", "float weighted = raw_err;"),
    ("f32state_ema_history_dropped", "fmaf(one_minus_beta, e_old, weighted)", "weighted"),
    ("f32state_ema_weights_swapped", "fmaf(one_minus_beta, e_old, weighted)", "fmaf(beta, e_old, one_minus_beta * raw_err)"),
    ("f32state_reset_ignored", "err_state[i] = reset ? 0.0f : fmaf(one_minus_beta, e_old", "err_state[i] = 0 ? 0.0f : fmaf(one_minus_beta, e_old"),
    ("f32state_decode_not_scaled", "float d_own = (float)q / s;", "float d_own = (float)q;"),
    ("f32state_scale_inverted", "int q = (int)clamp_round(h * s, qmin, qmax);         /* Eq. 1, 3 */\n        float d_own",
     "int q = (int)clamp_round(h / s, qmin, qmax);\n        float d_own"),
    ("clip_one_sided", "if (g < -clip_abs)\n            g = -clip_abs;", ""),
    ("clip_sign_lost", "            g = -clip_abs;", "            g = clip_abs;"),
    ("sgd_ascent", "theta[i] = theta[i] - step;\n    }\n    return LOCO_REF_OK;\n}\n\nint loco_ref_adam_update",
     "theta[i] = theta[i] + step;\n    }\n    return LOCO_REF_OK;\n}\n\nint loco_ref_adam_update"),
    ("adam_bias_corrected_root", "float root = sqrtf(v_new + delta);", "float root = sqrtf(v_new) + delta;"),
    ("adam_second_moment_not_squared", "float g2 = g * g;", "float g2 = g;"),
    ("adam_moment_weights_swapped", "float m_new = fmaf(omb1, m[i], b1g);", "float m_new = fmaf(beta1, m[i], omb1 * g);"),
    ("adam_uses_old_v", "float root = sqrtf(v_new + delta);", "float root = sqrtf(v[i] + delta);"),
    ("adam_uses_gradient_not_momentum", "float step = eta_k * m_new;", "float step = eta_k * g;"),
    ("adam_v_not_stored", "        v[i] = v_new;\n", ""),
    ("bf16_truncates", "u += 0x7FFFu + ((u >> 16) & 1u);", ""),
    ("bf16_ties_away", "u += 0x7FFFu + ((u >> 16) & 1u);", "u += 0x8000u;"),
    ("bf16_step_stored_but_not_used", "            memcpy(&D, &wide, sizeof D);\n        }\n        float r = 0.0f;",
     "        }\n        float r = 0.0f;"),
    ("bf16_step_dead_test_before_rounding", "int dead = D < FLT_MIN;", "int dead = (amax / (float)qmax) < FLT_MIN;"),
    ("bf16_step_decode_shift", "scales16[(size_t)w * scale_stride_elems + b] << 16;",
     "scales16[(size_t)w * scale_stride_elems + b] << 15;"),
    ("bf16_step_worker_stride", "scales16[(size_t)w * scale_stride_elems + b]", "scales16[b]"),
    ("fixed_reduce_stride", "int q = code_at(codes + (size_t)w * code_stride_bytes, bits, i);\n            float d = (float)q / s;",
     "int q = code_at(codes, bits, i);\n            float d = (float)q / s;"),
]


def plant(text, old, new, which):
    parts = text.split(old)
    assert len(parts) - 1 > which, "mutation site not found"
    return old.join(parts[:which + 1]) + new + old.join(parts[which + 1:])


@pytest.mark.parametrize("mutant", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, mutant):
    name, old, new = mutant[:3]
    which = mutant[3] if len(mutant) > 3 else 0
    text = open(SRC).read()
    assert text.count(old) > which, f"mutation site for {name} not found"
    src = tmp_path / "loco_ref.c"
    src.write_text(plant(text, old, new, which))
    shutil.copy(MT, tmp_path / "loco_ref_mt.c")
    so = oracle.build(force=True, out=str(tmp_path / "libmutant.so"),
                      srcs=[str(src), str(tmp_path / "loco_ref_mt.c")], extra_flags=["-w"])
    lib = oracle.load(so)
    caught = []
    for check in pins.ALL_CHECKS:
        try:
            check(lib)
        except (AssertionError, ValueError, FloatingPointError):
            caught.append(check.__name__)
            break
    assert caught, f"no pin noticed the planted mistake {name!r}"

