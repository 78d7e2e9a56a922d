"""Do the pins bite?  Each case plants ONE plausible mistake in a copy of the oracle's C source
(a dropped term, a wrong sign or index, a rounding moved to another quantity), compiles that copy
on the CPU, points the oracle wrapper at it, and asserts that at least one pin of
tests/test_oracle_pins.py fails.  CPU only; the HIP path is not involved."""
import os
import subprocess

import pytest

import oracle
from tests import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "sea_oracle.c")

# (name, text in sea_oracle.c, replacement)
MUTATIONS = [
    ("own_column_drops_key_t", "j = block_start(ct, T, KK); j <= t; ++j", "j = block_start(ct, T, KK); j < t; ++j"),
    ("bucket_map_by_fixed_width", "return (j * K) / T; }", "return j / ((T + K - 1) / K); }"),
    ("key_norm_term_dropped", "(j < len) ? exp(dot - 0.5 * ny)", "(j < len) ? exp(dot)"),
    ("key_projection_sign", "(j < len) ? exp(dot - 0.5 * ny)", "(j < len) ? exp(-dot - 0.5 * ny)"),
    ("query_norm_term_sign", "arg[i] = dot - 0.5 * nx;", "arg[i] = dot + 0.5 * nx;"),
    ("tie_goes_to_higher_column", "Arow[c] > Arow[best]", "Arow[c] >= Arow[best]"),
    ("no_even_spacing", "const int64_t j = s0 + (i * w) / rep;", "const int64_t j = s0 + i;"),
    ("logit_scale_dropped", "s[x] = p->scale * dot;", "s[x] = dot;"),
    ("expansion_drops_last_key", "if (j <= jmax) irow[ni++]", "if (j < jmax) irow[ni++]"),
    ("candidates_one_short", "bucket_of(jmax, Tw, KK) + 1 : 0;", "bucket_of(jmax, Tw, KK) : 0;"),
    ("block_start_floor", "return (c * T + K - 1) / K;", "return (c * T) / K;"),
    ("rounding_half_away", "double r = nearbyint(s);", "double r = floor(s + 0.5);"),
    ("own_column_from_full_state", "if (!p->causal || c < ct) {", "if (!p->causal || c <= ct) {"),
    ("projection_transposed_operand", "for (int64_t e = 0; e < d; ++e) dot += W[i * d + e] * y[e];\n          phiK",
     "for (int64_t e = 0; e < d; ++e) dot += W[i * d + e] * y[d - 1 - e];\n          phiK"),
    ("softmax_not_normalised", "const double pj = s[x] / z;", "const double pj = s[x];"),
    ("k_hat_truncates", "int64_t r = (2 * num + T) / (2 * (int64_t)T);", "int64_t r = num / T;"),
    # the reduced-precision mode: each rounding point moved or removed
    ("r8_state_not_rounded", "state[x] = ref_round8(state[x]);", "state[x] = state[x];"),
    ("r8_query_features_not_rounded", "if (p->round8) phiQ[i] = ref_round8(phiQ[i]);", ";"),
    ("r8_own_column_keys_not_rounded", "acc += phiQ[i] * (p->round8 ? ref_round8(f) : f);", "acc += phiQ[i] * f;"),
    ("r8_row_width_keys_not_rounded", "dotp += phiQ[i] * (p->round8 ? ref_round8(f) : f);", "dotp += phiQ[i] * f;"),
    ("r8_state_rounded_per_key", "state[c * m + i] += phiK[j * m + i];",
     "state[c * m + i] += p->round8 ? ref_round8(phiK[j * m + i]) : phiK[j * m + i];"),
    ("r8_query_rounded_before_shift_to_7_bits", "double s = ldexp(f, 8);           /* |s| in [128, 256) */\n  double r = nearbyint(s);          /* default mode: ties to even */\n  return ldexp(r, e - 8);",
     "double s = ldexp(f, 7);\n  double r = nearbyint(s);\n  return ldexp(r, e - 7);"),
    ("mix_importance_not_stretched", "const double wj = ihat[bucket_of(j, T, KK)];", "const double wj = ihat[j % KK];"),
    ("mix_running_mean_off_by_one", "avg[e] / (double)(t + 1)", "avg[e] / (double)(t > 0 ? t : 1)"),
]

# pins in the order they are tried (cheap ones first); parametrised ones with their arguments
PINS = [
    (pins.test_k_hat_formula_golden, {}),
    (pins.test_round8_matches_library_bf16_cast, {}),
    (pins.test_expansion_hand_enumerated_T8_K4, {}),
    (pins.test_expansion_equals_library_nearest_resize, {"T": 37, "K": 5}),
    (pins.test_replication_cap_k_star, {}),
    (pins.test_topk_equals_full_sort_and_tie_rule, {}),
    (pins.test_full_selection_is_dense_attention, {"causal": True, "T": 24, "K": 6}),
    (pins.test_sparse_softmax_rows_sum_to_one, {}),
    (pins.test_estimate_closed_form_zero_inputs, {"T": 23, "K": 5}),
    (pins.test_estimate_literal_favor_with_stretched_identity, {}),
    (pins.test_reduced_precision_points_hand_built_case, {}),
    (pins.test_reduced_precision_points_with_library_casts, {}),
    (pins.test_row_width_reduced_precision_points_with_library_casts, {}),
    (pins.test_output_mix_limits_and_closed_forms, {}),
    (pins.test_estimate_converges_to_exact_softmax_buckets, {"causal": True}),
]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_a_pin(tmp_path, name, old, new):
    src = open(SRC).read()
    assert src.count(old) >= 1, f"mutation {name}: text not found in the oracle source"
    mutated = tmp_path / "sea_oracle_mut.c"
    mutated.write_text(src.replace(old, new, 1))
    lib = tmp_path / f"libsea_oracle_{name}.so"
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-D_GNU_SOURCE", "-o", str(lib),
                    str(mutated), "-lm"], check=True)
    good = oracle._load()
    caught = None
    try:
        oracle._lib = oracle._open(str(lib))
        for fn, kw in PINS:
            try:
                fn(**kw)
            except Exception:          # an assertion, or a crash of the check on nonsense values
                caught = fn.__name__
                break
    finally:
        oracle._lib = good
    assert caught is not None, f"no pin noticed the planted mistake '{name}'"
