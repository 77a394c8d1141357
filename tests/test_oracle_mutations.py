"""The pins must be able to fail: plant plausible mistakes in a COPY of the oracle's C source
(on the CPU), load the mutant in place of the real library, and check that at least one pin
catches each of them.  No GPU involved."""
import os
import subprocess

import pytest

from oracle import moe_oracle as orc
import test_oracle_pins as pins
import test_oracle_fp8_pins as fp8pins
import test_oracle_chain_pins as chainpins

MUTANTS = {
    "swap_w1_w3_roles": ("h[r] = (g / ((REAL)1 + real_exp(-g))) * u;", "h[r] = (u / ((REAL)1 + real_exp(-u))) * g;"),
    "silu_sign": ("real_exp(-g))) * u;", "real_exp(g))) * u;"),
    "drop_up_projection": ("real_exp(-g))) * u;", "real_exp(-g)));"),
    "transposed_w2": ("const uint16_t* a = w2 + (size_t)c * ffn;\n    for (int r = 0; r < ffn; ++r) s += (REAL)bf16_widen(a[r]) * h[r];",
                      "for (int r = 0; r < ffn; ++r) s += (REAL)bf16_widen(w2[(size_t)r * d + c]) * h[r];"),
    "drop_gate": ("acc[c] += g * y[c];", "acc[c] += y[c];"),
    "drop_shared": ("for (int s = 0; s < n_shared; ++s) {\n      oracle_expert_ffn(x, sw1 + s * per, sw3 + s * per, sw2 + s * per, d, ffn, h, y);\n      for (int c = 0; c < d; ++c) acc[c] += y[c];\n    }\n    for (int c = 0; c < d; ++c) out[(size_t)t * d + c] = (float)acc[c];\n  }\n  free(h);\n  free(y);\n  free(acc);\n  return rc;",
                    "for (int c = 0; c < d; ++c) out[(size_t)t * d + c] = (float)acc[c];\n  }\n  free(h);\n  free(y);\n  free(acc);\n  return rc;"),
    "tie_to_higher_index": ("logit[e] > logit[best]", "logit[e] >= logit[best]"),
    "argmin_instead_of_argmax": ("logit[e] > logit[best]", "logit[e] < logit[best]"),
    "gates_not_normalised": ("(float)(p[i] / sum);", "(float)(p[i]);"),
    "gates_wrong_sign": ("- l0);\n      sum += p[i];", "- l0);\n      p[i] = (REAL)1 / p[i];\n      sum += p[i];"),
    "router_wrong_row": ("router_w[(size_t)e * d + j]", "router_w[(size_t)((e + 1) % E) * d + j]"),
    "expert_offset_wrong": ("oracle_expert_ffn(x, w1 + e * per, w3 + e * per, w2 + e * per, d, ffn, h, y);\n      REAL g",
                            "oracle_expert_ffn(x, w1 + e * per, w3 + e * per, w2, d, ffn, h, y);\n      REAL g"),
    "union_skips_last_expert": ("for (int e = 0; e < E; ++e) {\n    int c = 0;", "for (int e = 0; e < E - 1; ++e) {\n    int c = 0;"),
    "token_uses_row0": ("const float* x = hidden + (size_t)t * d;\n    for (int c = 0; c < d; ++c) acc[c] = 0;\n    for (int i = 0; i < top_k; ++i) {",
                        "const float* x = hidden;\n    for (int c = 0; c < d; ++c) acc[c] = 0;\n    for (int i = 0; i < top_k; ++i) {"),
}

MUTANTS_FP8 = {
    "fp8_exponent_bias_8": ("ldexp(1.0 + (double)man / 8.0, ex - 7)", "ldexp(1.0 + (double)man / 8.0, ex - 8)"),
    "fp8_subnormal_read_as_normal": ("  if (ex == 0)\n    v = ldexp((double)man / 8.0, -6);\n  else\n", ""),
    "fp8_subnormal_flushed": ("v = ldexp((double)man / 8.0, -6);", "v = 0.0;"),
    "fp8_four_mantissa_bits": ("ldexp(1.0 + (double)man / 8.0, ex - 7)", "ldexp(1.0 + (double)man / 16.0, ex - 7)"),
    "fp8_sign_ignored": ("return sign ? -v : v;", "return v;"),
    "fp8_top_exponent_is_inf_nan": ("if (ex == 15 && man == 7) return NAN;", "if (ex == 15) return NAN;"),
    "fp8_scale_per_column": ("((REAL)s1[r] * val[q1[(size_t)r * d + j]])", "((REAL)s1[j % ffn] * val[q1[(size_t)r * d + j]])"),
    "fp8_w3_uses_w1_scale": ("((REAL)s3[r] * val[q3[(size_t)r * d + j]])", "((REAL)s1[r] * val[q3[(size_t)r * d + j]])"),
    "fp8_down_scale_dropped": ("((REAL)s2[c] * val[q2[(size_t)c * ffn + r]])", "(val[q2[(size_t)c * ffn + r]])"),
    "fp8_down_transposed": ("val[q2[(size_t)c * ffn + r]]", "val[q2[(size_t)r * d + c]]"),
    "fp8_expert_scale_offset_missing": ("q1 + e * per, s1 + (size_t)e * ffn,", "q1 + e * per, s1,"),
    "fp8_shared_scale_offset_missing": ("sq2 + s * per, ss2 + (size_t)s * d,", "sq2 + s * per, ss2,"),
    "fp8_gate_dropped": ("      REAL g = (REAL)gates[(size_t)t * top_k + i];\n      for (int c = 0; c < d; ++c) acc[c] += g * y[c];\n    }\n    for (int s = 0; s < n_shared; ++s) {\n      oracle_expert_ffn_fp8",
                         "      for (int c = 0; c < d; ++c) acc[c] += y[c];\n    }\n    for (int s = 0; s < n_shared; ++s) {\n      oracle_expert_ffn_fp8"),
}

MUTANTS_GATE = {
    "softmax_all_sums_only_the_picks": ("for (int e = 0; e < E; ++e) sum += real_exp((REAL)l[e] - m);",
                                        "for (int i = 0; i < top_k; ++i) sum += real_exp((REAL)l[ids[(size_t)t * top_k + i]] - m);"),
    "softmax_all_skips_last_expert": ("for (int e = 0; e < E; ++e) sum += real_exp((REAL)l[e] - m);",
                                      "for (int e = 0; e < E - 1; ++e) sum += real_exp((REAL)l[e] - m);"),
    "softmax_all_wrong_token_row": ("const double* l = logit + (size_t)t * E;", "const double* l = logit;"),
    "softmax_all_numerator_is_one": ("(float)(real_exp((REAL)l[ids[(size_t)t * top_k + i]] - m) / sum);", "(float)((REAL)1 / sum);"),
}

PIN_CALLS_GATE = [
    lambda: pins.test_softmax_all_gates_against_library_softmax_and_identities("f64"),
    lambda: pins.test_softmax_all_layer_scales_each_token_by_its_pick_mass("f64"),
]

MUTANTS_CHAIN = {
    "rmsnorm_sum_not_mean": ("const REAL mean = ss / (REAL)d;", "const REAL mean = ss;"),
    "rmsnorm_eps_outside_root": ("(REAL)sqrtf((float)(mean + (REAL)eps)) : (REAL)sqrt((double)mean + eps);",
                                 "(REAL)(sqrtf((float)mean) + (float)eps) : (REAL)(sqrt((double)mean) + eps);"),
    "rmsnorm_gamma_index_off_by_one": ("(REAL)bf16_widen(gamma[j]));", "(REAL)bf16_widen(gamma[(j + 1) % d]));"),
    "rmsnorm_uses_first_token_stats": ("ss += (REAL)xt[j] * (REAL)xt[j];", "ss += (REAL)x[j] * (REAL)x[j];"),
    "rmsnorm_no_root": ("y[(size_t)t * d + j] = (float)(((REAL)xt[j] / root)", "y[(size_t)t * d + j] = (float)(((REAL)xt[j] / (mean + (REAL)eps))"),
    "residual_drops_skip_path": ("x_out[i] = (float)((REAL)x_in[i] + (REAL)delta[i]);", "x_out[i] = (float)((REAL)delta[i]);"),
}

MUTANTS_ATTN = {
    "attn_no_scale": ("p[u] = s * scale;", "p[u] = s;"),
    "attn_values_of_later_tokens_leak": ("for (int u = 0; u <= t; ++u) acc += (p[u] / sum) *", "for (int u = 0; u < T; ++u) acc += (p[u < t ? u : t] / sum) *"),
    "attn_denominator_over_all_tokens": ("for (int u = 0; u <= t; ++u) {\n        p[u] = real_exp(p[u] - m);", "for (int u = 0; u < T; ++u) {\n        p[u] = real_exp(p[u < t ? u : t] - m);"),
    "attn_kv_head_of_query_head": ("const int g = h / (H / Hkv);", "const int g = h % Hkv;"),
    "attn_value_rows_are_key_rows": ("qkv[(size_t)u * nout + nq + nkv + (size_t)g * dh + j];", "qkv[(size_t)u * nout + nq + (size_t)g * dh + j];"),
    "attn_softmax_not_normalised": ("acc += (p[u] / sum) *", "acc += p[u] *"),
    "attn_out_projection_transposed": ("wo[(size_t)c * nq + j]", "wo[(size_t)j * d + c]"),
    "attn_query_is_token_zero": ("const REAL* q = qkv + (size_t)t * nout + (size_t)h * dh;", "const REAL* q = qkv + (size_t)h * dh;"),
}

PIN_CALLS_ATTN = [
    lambda: chainpins.test_attention_stub_matches_the_tensor_library_attention("f64"),
    lambda: chainpins.test_attention_stub_special_cases("f64"),
]

PIN_CALLS_CHAIN = [
    lambda: chainpins.test_rmsnorm_hand_values_and_invariants("f64"),
    lambda: chainpins.test_rmsnorm_eps_sits_inside_the_root_next_to_the_mean("f64"),
    lambda: chainpins.test_chained_block_wiring("f64"),
]

PIN_CALLS_FP8 = [
    lambda: fp8pins.test_e4m3_golden_corner_values(),
    lambda: fp8pins.test_e4m3_all_codes_match_library_type_and_structure(),
    lambda: fp8pins.test_fp8_ffn_equals_bf16_oracle_when_effective_weights_fit_bf16("f64"),
    lambda: fp8pins.test_fp8_ffn_general_scales_is_three_library_gemvs(),
    lambda: fp8pins.test_fp8_row_scales_closed_form("f64"),
    lambda: fp8pins.test_fp8_combine_gate_weighting_experts_and_shared("f64"),
]

PIN_CALLS = [
    lambda: pins.test_route_brute_force("f64", 8, 2),
    lambda: pins.test_route_ties_go_to_lower_index_and_uniform_gates("f64"),
    lambda: pins.test_route_topk_equals_E_is_permutation_and_row_permutation_equivariance("f64"),
    lambda: pins.test_gates_closed_forms("f64"),
    lambda: pins.test_union_structure_and_paper_example(),
    lambda: pins.test_expert_ffn_closed_form_selection_matrices("f64"),
    lambda: pins.test_top1_layer_is_three_library_gemvs("f64"),
    lambda: pins.test_combine_closed_form_gate_weighting_and_shared("f64"),
    lambda: pins.test_zero_w1_gives_zero_and_dense_masked_agrees("f64"),
    lambda: pins.test_batch_invariance_and_token_permutation("f64"),
]


_GROUPS = ((MUTANTS, lambda: PIN_CALLS), (MUTANTS_FP8, lambda: PIN_CALLS_FP8), (MUTANTS_GATE, lambda: PIN_CALLS_GATE),
           (MUTANTS_CHAIN, lambda: PIN_CALLS_CHAIN), (MUTANTS_ATTN, lambda: PIN_CALLS_ATTN))


@pytest.mark.parametrize("name", sorted(MUTANTS) + sorted(MUTANTS_FP8) + sorted(MUTANTS_GATE) + sorted(MUTANTS_CHAIN)
                         + sorted(MUTANTS_ATTN))
def test_pins_catch_planted_mistake(name, tmp_path, monkeypatch):
    table, get_calls = next((m, c) for m, c in _GROUPS if name in m)
    old, new = table[name]
    calls = get_calls()
    src = open(os.path.join(os.path.dirname(orc.__file__), "moe_oracle.c")).read()
    assert src.count(old) >= 1, f"mutation site for {name} not found"
    mutated = src.replace(old, new, 1)
    c = tmp_path / "mutant.c"
    so = tmp_path / "mutant.so"
    c.write_text(mutated)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-DREAL=double",
                    str(c), "-o", str(so), "-lm"], check=True)
    mutant = orc._load(str(so), "f64")
    orc._lib("f64")
    monkeypatch.setitem(orc._LIBS, "f64", mutant)
    caught = False
    for call in calls:
        try:
            call()
        except (AssertionError, ValueError):
            caught = True
            break
    assert caught, f"no pin noticed the planted mistake '{name}'"
