"""The pins are only worth something if a plausible mistake in the oracle makes one of them fail.
Each case below plants one mistake (a wrong sign, index, constant, operand or a dropped step) in a
COPY of the oracle's C source, builds it with the host compiler and runs the pin that should catch
it against the mutant.  CPU only; the real oracle and the HIP library are not touched."""
import importlib.util
import os
import sys

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
from tests import test_oracle_pins as pins      # noqa: E402

# (what is planted, text to find (exactly once), replacement, pins expected to fail: name or (name, args))
MUTANTS = [
    ("top-k ties prefer the higher index", "    if (sa < sb) return 0;\n    return ia < ib;", "    if (sa < sb) return 0;\n    return ia > ib;",
     ["test_topk_all_equal_keeps_prefix"]),
    ("NaN ranks above numbers", "return nb;                     /* a number ranks before a NaN */", "return na;", ["test_topk_adversarial"]),
    ("projection drops the translation", " + Rt[4 * i + 2] * xyz[2]) + Rt[4 * i + 3];", " + Rt[4 * i + 2] * xyz[2]);",
     ["test_projection_closed_forms", "test_projection_matches_homogeneous_matrix_product"]),
    ("patch index rounds toward zero", "double fu = floor((h[0] / h[2]) / patch_w)", "double fu = trunc((h[0] / h[2]) / patch_w)", ["test_projection_closed_forms"]),
    ("ring is a diamond, not a square", "(uint8_t)((du > dv ? du : dv) <= radius)", "(uint8_t)((du + dv) <= radius)",
     ["test_ring_counts_match_the_hand_counted_fixture", "test_ring_membership_is_the_chebyshev_ball"]),
    ("FPS takes the last of equal distances", "if (dmin > best_d) {", "if (dmin >= best_d) {", ["test_fps_hand_worked_sequence"]),
    ("FPS uses the distance to the nearest UNKEPT token", "                if (!kept[s]) continue;\n                long du", "                if (kept[s] || s == c) continue;\n                long du",
     ["test_fps_each_pick_maximises_the_distance_to_the_kept_set", "test_fps_hand_worked_sequence"]),
    ("the union is cut to the budget", "    if (rc == 0 && keep_total > count) {", "    if (rc == 0 && keep_total != count) {", ["test_final_set_special_cases"]),
    ("butterfly sign", "                v[j + h] = a - b;", "                v[j + h] = b - a;", ["test_fwht_matches_fixture_matrix"]),
    ("rotation not normalised", "    for (int j = 0; j < K; ++j) v[j] = v[j] * c;\n    return 0;", "    return 0;", ["test_fwht_unit_vectors", "test_rotation_leaves_the_linear_unchanged"]),
    ("quantizer divides by 8", "oracle_f32_to_f16(amax / 7.0f);\n        if (sh == 0) sh = 1;                     /* 2^-24: keeps the scale positive */", "oracle_f32_to_f16(amax / 8.0f);\n        if (sh == 0) sh = 1;",
     ["test_quantizer_error_bound_and_range", "test_quantizer_every_finite_half_as_a_row"]),
    ("quantizer truncates", "        int32_t sum = 0;\n        for (int k = 0; k < K; k += 2) {\n            int q[2];\n            for (int t = 0; t < 2; ++t) {\n                float r = rintf(v[k + t] / sf);",
     "        int32_t sum = 0;\n        for (int k = 0; k < K; k += 2) {\n            int q[2];\n            for (int t = 0; t < 2; ++t) {\n                float r = truncf(v[k + t] / sf);", ["test_quantizer_error_bound_and_range", "test_quantizer_half_way_cases_round_to_even"]),
    ("codes clamp at -7", "                if (r < -8.0f) r = -8.0f;\n                q[t] = (int)r;\n                sum += q[t];", "                if (r < -7.0f) r = -7.0f;\n                q[t] = (int)r;\n                sum += q[t];",
     ["test_quantizer_clamp_reaches_minus_eight_only_below_the_normal_scales"]),
    ("integer product transposed", "const int8_t *xr = x + (size_t)m * K, *wr = w + (size_t)n * K;", "const int8_t *xr = x + (size_t)(m % N) * K, *wr = w + (size_t)(n % M) * K;",
     ["test_int_gemm_vs_numpy_int64", "test_int_gemm_hand_cases"]),
    ("dequantisation uses one scale", "            float y = t * oracle_f16_to_f32(sw[n]);\n            Y[(size_t)m * ldy + n]", "            float y = t;\n            Y[(size_t)m * ldy + n]",
     ["test_dequant_against_numpy_half_conversion"]),
    ("retention score not averaged over heads", "scores_out[j] = (float)(acc[j] / (double)H);", "scores_out[j] = (float)(acc[j]);", ["test_attn_scores_vs_library_softmax"]),
    ("sum of squares off by a factor two", "<< (2 * e + 48);", "<< (2 * e + 47);", ["test_rmsnorm_constant_row_and_unit_rms"]),
    ("subnormal halves misread", "int e = ex ? (int)ex - 25 : -24;", "int e = ex ? (int)ex - 25 : -25;", ["test_rmsnorm_sum_of_squares_is_exact"]),
    ("eps dropped", "sqrt(Sd / (double)K + (double)eps)", "sqrt(Sd / (double)K)", ["test_rmsnorm_constant_row_and_unit_rms"]),
    ("residual subtracted", "float s = oracle_f16_to_f32(h) + oracle_f16_to_f32(delta[(size_t)i * K + k]);", "float s = oracle_f16_to_f32(h) - oracle_f16_to_f32(delta[(size_t)i * K + k]);",
     ["test_rmsnorm_gather_and_residual_update"]),
    ("silu with the wrong sign in the exponent", "float s = (float)(g / (1.0 + exp(-g)));", "float s = (float)(g / (1.0 + exp(g)));", ["test_swiglu_against_high_precision_and_identities"]),
    ("rotary embedding turns the other way", "(float)(lo * cos(a) - hi * sin(a))", "(float)(lo * cos(a) + hi * sin(a))", ["test_rope_is_a_rotation_by_position_times_frequency"]),
    ("rotary frequency uses d/2", "pow(base, -2.0 * (double)i / (double)d)", "pow(base, -(double)i / (double)d)", ["test_rope_is_a_rotation_by_position_times_frequency"]),
    ("attention sees later keys", "            int last = Sk - Sq + s;", "            int last = Sk - 1;", ["test_attention_closed_forms_and_matrix_form"]),
    ("attention not scaled by sqrt(d)", "                p[t] = dot / sqrt((double)d);\n                if (p[t] > lmax) lmax = p[t];", "                p[t] = dot;\n                if (p[t] > lmax) lmax = p[t];",
     ["test_attention_closed_forms_and_matrix_form"]),
]


def _load_mutant(tmp_path, find, replace):
    src = open(os.path.join(ROOT, "oracle", "sqap_oracle.c")).read()
    assert src.count(find) == 1, "the text to mutate must occur exactly once: %r" % find
    mutated = tmp_path / "sqap_oracle_mutant.c"
    mutated.write_text(src.replace(find, replace))
    spec = importlib.util.spec_from_file_location("oracle_mutant_%d" % abs(hash((find, replace))),
                                                  os.path.join(ROOT, "oracle", "__init__.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod._SRC = str(mutated)
    mod._LIB = str(tmp_path / "libsqap_oracle_mutant.so")
    mod.build(force=True)
    return mod


@pytest.mark.parametrize("what,find,replace,catchers", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_is_caught(tmp_path, what, find, replace, catchers):
    mutant = _load_mutant(tmp_path, find, replace)
    caught = []
    for name in catchers:
        try:
            getattr(pins, name)(mutant)
        except (AssertionError, ValueError):
            caught.append(name)
    assert caught, "no pin noticed: " + what
