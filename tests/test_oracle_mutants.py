"""Do the oracle's pins notice a mistake?  Plant plausible single-token mistakes in copies of
``oracle/po_oracle.c`` (dropped terms, wrong signs, stale state, swapped operands, misplaced epsilon,
missing bias corrections, wrong rounding), build each copy on the CPU and run the pin suite against
it: every mutant must fail at least one pin, and the untouched source must pass them all."""
import os
import tempfile

import pytest

import oracle as real_oracle
import test_oracle_pins as pins

MUTANTS = [
    ("sgdm dampening dropped", "double mt = u * m + (1.0 - tau) * gt;", "double mt = u * m + gt;"),
    ("sgdm momentum factor dropped", "double mt = u * m + (1.0 - tau) * gt;", "double mt = m + (1.0 - tau) * gt;"),
    ("sgdm direction from the stale buffer", "dW_step = dW_pred = mt;", "dW_step = dW_pred = m;"),
    ("step with the wrong sign", "*W_new = W - lr * dW_step;", "*W_new = W + lr * dW_step;"),
    ("prediction with the wrong sign", "else        *What = W - lr * (double)s * dW_pred;", "else        *What = W + lr * (double)s * dW_pred;"),
    ("prediction one version too far", "else        *What = W - lr * (double)s * dW_pred;", "else        *What = W - lr * (double)(s + 1) * dW_pred;"),
    ("prediction ignores s", "else        *What = W - lr * (double)s * dW_pred;", "else        *What = W - lr * dW_pred;"),
    ("coupled decay dropped", "double gt = g + wd * W;                   /* coupled L2", "double gt = g;  /* coupled L2"),
    ("coupled decay also in AdamW", "double gt = (opt == PO_ORACLE_ADAM) ? g + wd * W : g;", "double gt = g + wd * W;"),
    ("first moment with beta2", "double mt = beta1 * m + (1.0 - beta1) * gt;", "double mt = beta2 * m + (1.0 - beta2) * gt;"),
    ("first moment gradient weight dropped", "double mt = beta1 * m + (1.0 - beta1) * gt;", "double mt = beta1 * m + gt;"),
    ("second moment not squared", "double vt = beta2 * v + (1.0 - beta2) * gt * gt;", "double vt = beta2 * v + (1.0 - beta2) * gt;"),
    ("second moment with beta1", "double vt = beta2 * v + (1.0 - beta2) * gt * gt;", "double vt = beta1 * v + (1.0 - beta1) * gt * gt;"),
    ("no bias correction of m", "double mhat = mt / (1.0 - pow(beta1, (double)t));", "double mhat = mt;"),
    ("no bias correction of v", "double vhat = vt / (1.0 - pow(beta2, (double)t));", "double vhat = vt;"),
    ("bias correction with the wrong step index", "double mhat = mt / (1.0 - pow(beta1, (double)t));", "double mhat = mt / (1.0 - pow(beta1, (double)(t + 1)));"),
    ("epsilon inside the root", "double r = mhat / (sqrt(vhat) + eps);", "double r = mhat / sqrt(vhat + eps);"),
    ("no square root", "double r = mhat / (sqrt(vhat) + eps);", "double r = mhat / (vhat + eps);"),
    ("stale moments in the direction", "double r = mhat / (sqrt(vhat) + eps);", "double r = (m / (1.0 - pow(beta1, (double)t))) / (sqrt(vhat) + eps);"),
    ("decoupled decay dropped from the step", "dW_step = r + wd * W;                 /* decoupled decay", "dW_step = r;  /* decoupled decay"),
    ("decay flag inverted", "dW_pred = decay_in_prediction ? dW_step : r;", "dW_pred = decay_in_prediction ? r : dW_step;"),
    ("new state not stored", "*m_new = mt;\n        *v_new = vt;", "*m_new = m;\n        *v_new = vt;"),
    ("nesterov: buffer with dampening-like factor", "double mt = u * m + gt;\n        *m_new = mt;\n        *v_new = v;\n        dW_step = dW_pred = gt + u * mt;", "double mt = u * m + (1.0 - u) * gt;\n        *m_new = mt;\n        *v_new = v;\n        dW_step = dW_pred = gt + u * mt;"),
    ("nesterov: no look-ahead (plain momentum)", "dW_step = dW_pred = gt + u * mt;", "dW_step = dW_pred = mt;"),
    ("nesterov: look-ahead with the stale buffer", "dW_step = dW_pred = gt + u * mt;", "dW_step = dW_pred = gt + u * m;"),
    ("rmsprop: average without the (1-alpha) weight", "? alpha * v + (1.0 - alpha) * gt * gt : v + gt * gt;", "? alpha * v + gt * gt : v + gt * gt;"),
    ("adagrad: sum decays", "? alpha * v + (1.0 - alpha) * gt * gt : v + gt * gt;", "? alpha * v + (1.0 - alpha) * gt * gt : alpha * v + gt * gt;"),
    ("rmsprop/adagrad: epsilon inside the root", "dW_step = dW_pred = gt / (sqrt(vt) + eps);", "dW_step = dW_pred = gt / sqrt(vt + eps);"),
    ("rmsprop/adagrad: stale second moment", "dW_step = dW_pred = gt / (sqrt(vt) + eps);", "dW_step = dW_pred = gt / (sqrt(v) + eps);"),
    ("rmsprop/adagrad: raw gradient without decay in the numerator", "dW_step = dW_pred = gt / (sqrt(vt) + eps);", "dW_step = dW_pred = g / (sqrt(vt) + eps);"),
    ("version difference off by one", "return D - rank - 1;", "return D - rank;"),
    ("bf16 ties away from zero", "else                   pick = ((lo_bits >> 16) & 1u) ? hi_bits : lo_bits;", "else                   pick = hi_bits;"),
    ("bf16 truncation", "if (d_lo < d_hi)       pick = lo_bits;", "if (1)       pick = lo_bits;"),
    ("bf16 of the prediction truncated", "if (What_bf16) What_bf16[i] = po_oracle_bf16_from_f32(Wh32);\n        if (W_out)", "if (What_bf16) What_bf16[i] = (uint16_t)(bits_from_f32(Wh32) >> 16);\n        if (W_out)"),
    ("predict: no bias correction of m", "double mhat = (double)m[i] / (1.0 - pow(beta1, (double)t));", "double mhat = (double)m[i];"),
    ("predict: no bias correction of v", "double vhat = (double)v[i] / (1.0 - pow(beta2, (double)t));", "double vhat = (double)v[i];"),
    ("predict: decay for Adam too", "if (opt == PO_ORACLE_ADAMW && decay_in_prediction) dW += weight_decay * Wi;", "if (decay_in_prediction) dW += weight_decay * Wi;"),
    ("predict: decay with the wrong sign", "if (opt == PO_ORACLE_ADAMW && decay_in_prediction) dW += weight_decay * Wi;", "if (opt == PO_ORACLE_ADAMW && decay_in_prediction) dW -= weight_decay * Wi;"),
    ("predict: wrong sign", "double Wh = (s == 0) ? Wi : Wi - lr * (double)s * dW;", "double Wh = (s == 0) ? Wi : Wi + lr * (double)s * dW;"),
    ("predict: epsilon inside the root", "dW = mhat / (sqrt(vhat) + eps);", "dW = mhat / sqrt(vhat + eps);"),
]


def _pin_suite(orc):
    """The pins of test_oracle_pins.py, cheapest first, against one build of the oracle."""
    for key, rows in pins._cases(False):
        pins.test_hand_cases_table1_eq1_eq5(orc, key, rows)
    for key, rows in pins._cases(True):
        pins.test_hand_cases_predict_from_cached_state(orc, key, rows)
    pins.test_version_difference_eq4_and_fig2_indices(orc)
    pins.test_bf16_known_values(orc)
    pins.test_bf16_rounding_every_lower_half_for_sampled_upper_halves(orc)
    pins.test_direction_uses_updated_state_not_stale(orc)
    pins.test_sgdm_zero_buffer_is_plain_sgd(orc)
    pins.test_adam_first_step_from_zero_state(orc)
    pins.test_adamw_readings(orc)
    pins.test_new_optimizers_closed_forms(orc)
    pins.test_predict_sgdm_is_W_minus_s_lr_m(orc)
    pins.test_predict_adam_bias_corrections_closed_form(orc)
    pins.test_predict_s0_affine_and_adamw_readings(orc)
    for case in pins.STEP_CASES:
        pins.test_step_equals_library_optimizer(orc, *case)
    for case in pins.ALL_OPTS:
        pins.test_s0_returns_W_unchanged(orc, *case)
        pins.test_prediction_is_affine_in_s(orc, *case)
    pins.test_eq2_equals_eq3_when_direction_is_constant_sgd(orc)
    pins.test_eq2_equals_eq3_at_adam_fixed_point(orc)
    for case in pins.STEP_CASES:
        if case[0] in ("sgdm", "adam"):
            pins.test_predict_after_fused_step_equals_fused_prediction_one_further(orc, *case)


def _build_mutant(tmpdir, idx, old, new):
    src = open(real_oracle.SOURCE).read()
    assert src.count(old) == 1, "mutation site not unique or missing: %r" % old
    path = os.path.join(tmpdir, "mutant_%d.c" % idx)
    with open(path, "w") as f:
        f.write(src.replace(old, new))
    return real_oracle.OracleLib(real_oracle.compile_source(path, os.path.join(tmpdir, "mutant_%d.so" % idx)))


def test_unmutated_oracle_passes_the_suite():
    real_oracle.build()
    _pin_suite(real_oracle)


@pytest.mark.parametrize("idx", range(len(MUTANTS)), ids=[m[0] for m in MUTANTS])
def test_pins_catch_mutant(idx):
    name, old, new = MUTANTS[idx]
    with tempfile.TemporaryDirectory() as tmp:
        mutant = _build_mutant(tmp, idx, old, new)
        with pytest.raises(AssertionError):
            _pin_suite(mutant)
