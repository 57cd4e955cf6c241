"""The pins must be sharp: plant one plausible mistake at a time in a copy of
the oracle's C source (on the CPU, in a temp dir), load the mutant in place of
the real oracle and require that at least one pin test fails.  This guards the
pins themselves against going soft."""
import os
import subprocess

import pytest

import oracle
from oracle import build as obuild

import test_oracle_pins as pins

MUTANTS = [
    ("zero_point_sign", "((int32_t)x[m] - x_zp)", "((int32_t)x[m] + x_zp)",
     [pins.test_acc_special_cases]),
    ("dropped_first_k", "for (int64_t k = 0; k < K; ++k) {", "for (int64_t k = 1; k < K; ++k) {",
     [pins.test_acc_special_cases]),
    ("weight_read_unsigned", "(int32_t)W[n * ldw + k]", "(int32_t)(uint8_t)W[n * ldw + k]",
     [pins.test_acc_invariants, pins.test_acc_special_cases]),
    ("activation_read_signed", "((int32_t)x[m] - x_zp)", "((int32_t)(int8_t)x[m] - x_zp)",
     [pins.test_acc_special_cases]),
    ("unfused_multiply_add", "fmaf((float)a, s, b)", "((float)a * s + b)",
     [pins.test_dequant_bias_is_single_rounding_fma]),
    ("bias_dropped", "const float b = bias ? bias[n] : 0.0f;", "const float b = 0.0f;",
     [pins.test_rounding_pins_fixture]),
    ("round_half_away", "rintf(z * inv_out)", "roundf(z * inv_out)",
     [pins.test_rounding_pins_fixture]),
    ("zero_point_dropped", "+ (float)out_zp, lo, hi)", ", lo, hi)",
     [pins.test_rounding_pins_fixture]),
    ("s8_saturation_symmetric", "? 0.0f : -128.0f;", "? 0.0f : -127.0f;",
     [pins.test_rounding_pins_fixture]),
    ("gelu_sign", "erfc(-x / sqrt(2.0))", "erfc(x / sqrt(2.0))",
     [pins.test_gelu_textbook_normal_cdf_values]),
    ("gelu_tanh_like_constant", "sqrt(2.0)", "sqrt(2.01)",
     [pins.test_gelu_textbook_normal_cdf_values]),
    ("lut_truncates", "rint(v / (double)out_scale)", "trunc(v / (double)out_scale)",
     [lambda: pins.test_gelu_lut_all_256_entries_recomputed(1.0, 1.0, 0, "s8"),
      lambda: pins.test_gelu_lut_all_256_entries_recomputed(0.05, 0.02, -100, "s8"),
      lambda: pins.test_gelu_lut_all_256_entries_recomputed(0.3, 0.15, 4, "u8")]),
    ("lut_key_scale_swapped", "(double)i * (double)mid_scale", "(double)i * (double)out_scale",
     [lambda: pins.test_gelu_lut_all_256_entries_recomputed(0.05, 0.02, -100, "s8")]),
    ("gelu_int8_uses_out_scale", "rintf(y * inv_mid)", "rintf(y * inv_out)",
     [pins.test_gelu_int8_path_is_quantise_then_table]),
    ("scale_not_per_channel", "? w_scale[n] * x_scale :", "? w_scale[0] * x_scale :",
     [pins.test_dequant_bias_is_single_rounding_fma]),
    ("sum_before_gelu", """                float z = y;
                if (postop == ORACLE_POST_GELU)
                    z = (float)oracle_gelu((double)y);
                if (sum)
                    z = z + sum[n * ld_sum + m];""", """                float z = y;
                if (sum)
                    z = z + sum[n * ld_sum + m];
                if (postop == ORACLE_POST_GELU)
                    z = (float)oracle_gelu((double)z);""",
     [pins.test_sum_comes_after_gelu]),
    ("sum_transposed", """                    z = z + sum[n * ld_sum + m];
                ((float *)out)""", """                    z = z + sum[(m % N) * ld_sum + (n % M)];
                ((float *)out)""",
     [pins.test_sum_is_one_rounded_add_after_bias]),
    ("sum_added_in_double", """                    z = z + sum[n * ld_sum + m];
                ((float *)out)""", """                    z = (float)((double)a * (double)s + (double)b + (double)sum[n * ld_sum + m]);
                ((float *)out)""",
     [pins.test_sum_is_one_rounded_add_after_bias]),
    ("sum_after_quantize_scale", """                    z = z + sum[n * ld_sum + m];
                q = (int)sat_round(rintf(z * inv_out)""", """                    z = z + sum[n * ld_sum + m] * out_scale;
                q = (int)sat_round(rintf(z * inv_out)""",
     [lambda: pins.test_sum_comes_before_quantize("s8", -128, 127)]),
    ("sum_dropped_when_quantizing", """                if (sum)
                    z = z + sum[n * ld_sum + m];
                q = (int)sat_round""", """                q = (int)sat_round""",
     [lambda: pins.test_sum_comes_before_quantize("u8", 0, 255)]),
]


@pytest.mark.parametrize("name,old,new,checks", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(name, old, new, checks, tmp_path, monkeypatch):
    src = open(obuild.SRC).read()
    assert src.count(old) >= 1, "mutation site vanished: update the mutant list"
    mutated = src.replace(old, new, 1)
    c = tmp_path / "mutant.c"
    so = tmp_path / ("mutant_%s.so" % name)
    c.write_text(mutated)
    subprocess.check_call(["gcc", *obuild.FLAGS, str(c), "-o", str(so), "-lm"])
    oracle.lib()                                   # make sure the real one is loaded first
    monkeypatch.setattr(oracle, "_lib", oracle.load(str(so)))
    caught = False
    for chk in checks:
        try:
            chk()
        except AssertionError:
            caught = True
            break
    assert caught, "pins did not notice mutant %r" % name


def test_unmutated_oracle_passes_the_same_checks():
    for _, _, _, checks in MUTANTS:
        for chk in checks:
            chk()
