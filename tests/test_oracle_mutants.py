"""Planted mistakes in the CPU oracle are caught by its pins (CPU only).

Each case edits one expression of ``oracle/chai_oracle.c`` (a dropped factor, a wrong index, a flipped
comparison ...), builds the broken copy in a temporary directory and runs the pins that are supposed to notice.
A pin set that lets a mutant through is too weak to vouch for the oracle.  The mistakes are planted in the
oracle, on the CPU; the HIP library is not involved.

The repair rule's donor condition ("the donor cluster holds at least two heads") has its own mutant: hand-worked
cases in tests/golden/kmeans_worked.json have a lone head that is the farthest on the board while another centre is
empty, so taking it changes the partition (or the number of passes).
"""
import os
import subprocess

import pytest

import oracle_pins as P
from oracle import chai_oracle as O

SRC = os.path.join(os.path.dirname(O.__file__), "chai_oracle.c")

# (name, text to replace, replacement, which occurrence (0-based), pins expected to fail)
MUTANTS = [
    ("clustered_scale_dropped", "s[t] = scale * acc;", "s[t] = acc;", 0,
     ["pin_clustered_matches_library"]),
    ("prefill_scale_dropped", "s[t] = scale * acc;", "s[t] = acc;", 1,
     ["pin_prefill_matches_library_and_decode"]),
    ("dense_scale_dropped", "s[t] = scale * acc;", "s[t] = acc;", 2,
     ["pin_dense_matches_library"]),
    ("clustered_keys_of_cluster_id_instead_of_representative",
     "int64_t koff = ((int64_t)b * H + r) * (int64_t)T_cap * d;", "int64_t koff = ((int64_t)b * H + j) * (int64_t)T_cap * d;", 0,
     ["pin_clustered_matches_library", "pin_attention_worked_example"]),
    ("clustered_query_of_cluster_id", "int64_t qoff = ((int64_t)b * H + r) * d;", "int64_t qoff = ((int64_t)b * H + j) * d;", 0,
     ["pin_clustered_matches_library"]),
    ("member_reuses_representatives_values",
     "int64_t voff = ((int64_t)b * H + h) * (int64_t)T_cap * d;",
     "int64_t voff = ((int64_t)b * H + rep_heads[(int64_t)b * k + c]) * (int64_t)T_cap * d;", 0,
     ["pin_attention_worked_example", "pin_clustered_identical_qk_is_exact"]),
    ("probabilities_reversed_against_values", "acc += p[t] * load_elem(v, voff", "acc += p[T - 1 - t] * load_elem(v, voff", 0,
     ["pin_attention_worked_example", "pin_clustered_matches_library"]),
    ("token_stride_T_instead_of_T_cap", "int64_t coff = ((int64_t)b * H + h) * (int64_t)T_cap * d;",
     "int64_t coff = ((int64_t)b * H + h) * (int64_t)T * d;", 0, ["pin_dense_matches_library"]),
    ("softmax_without_max", "p[t] = exp(s[t] - m);", "p[t] = exp(s[t]);", 0, ["pin_softmax_properties"]),
    ("softmax_not_normalised", "p[t] = p[t] / z;", "p[t] = p[t];", 0, ["pin_attention_worked_example"]),
    ("softmax_of_negated_scores", "p[t] = exp(s[t] - m);", "p[t] = exp(m - s[t]);", 0, ["pin_attention_worked_example"]),
    ("bf16_shift", "]) << 16;", "]) << 15;", 0, ["pin_bf16_bits"]),
    ("features_transposed", "f[i * n_tok + j] = (j <= i) ? (float)p[j] : 0.0f;", "f[j * n_tok + i] = (j <= i) ? (float)p[j] : 0.0f;", 0,
     ["pin_features_worked_example", "pin_features_match_library"]),
    ("features_unscaled", "s[j] = scale * acc;", "s[j] = acc;", 0, ["pin_features_match_library"]),
    ("kmeans_ties_to_highest_centre", "if (dj < bd) { bd = dj; best = j; }", "if (dj <= bd) { bd = dj; best = j; }", 0,
     ["pin_kmeans_worked_examples"]),
    ("kmeans_distance_not_squared", "double sq = diff * diff;", "double sq = fabs(diff);", 0,
     ["pin_kmeans_matches_sklearn_lloyd", "pin_kmeans_brute_force"]),
    ("kmeans_mean_not_divided", "centre[j * F + f] = acc / (double)count[j];", "centre[j * F + f] = acc;", 0,
     ["pin_kmeans_worked_examples"]),
    ("kmeans_repair_takes_zero_distance", "dmin[h] > far) { far = dmin[h]; pick = h; }", "dmin[h] >= far) { far = dmin[h]; pick = h; }", 0,
     ["pin_kmeans_worked_examples"]),
    ("kmeans_repair_takes_a_lone_head", "if (count[assign[h]] >= 2 && dmin[h] > far)", "if (count[assign[h]] >= 1 && dmin[h] > far)", 0,
     ["pin_kmeans_worked_examples"]),
    ("kmeans_never_stops_early", "if (!changed || it >= max_iter) break;", "if (it >= max_iter) break;", 0,
     ["pin_kmeans_worked_examples"]),
    ("kmeans_labels_not_canonical", "head_to_cluster[(int64_t)b * H + h] = label[a];", "head_to_cluster[(int64_t)b * H + h] = a;", 0,
     ["pin_kmeans_worked_examples"]),
    ("kmeans_single_pass", "if (!changed || it >= max_iter) break;", "if (!changed || it >= 1) break;", 0,
     ["pin_kmeans_worked_examples"]),
    ("cluster_error_mean_over_all_heads", "mean[f] = acc / (double)cnt;", "mean[f] = acc / (double)H;", 0,
     ["pin_cluster_error_and_count"]),
    ("cluster_error_distance_not_squared_sum", "if (label_of[h] == j) total += sqdist(X + (int64_t)h * F, mean, F);",
     "if (label_of[h] == j) total += sqrt(sqdist(X + (int64_t)h * F, mean, F));", 0, ["pin_cluster_error_and_count"]),
    ("cluster_count_measured_from_first_point", "if (err[i] - err[n - 1] <= tol * drop)", "if (err[0] - err[i] >= tol * drop)", 0,
     ["pin_cluster_error_and_count"]),
    ("cluster_count_returns_index", "{ *k_out = ks[i]; return 0; }", "{ *k_out = i; return 0; }", 0,
     ["pin_cluster_error_and_count"]),
    ("shared_v_keeps_own_values", "acc += p[t] * load_elem(v, roff + (int64_t)t * d + i, dtype);",
     "acc += p[t] * load_elem(v, ((int64_t)b * H + h) * (int64_t)T_cap * d + (int64_t)t * d + i, dtype);", 0,
     ["pin_shared_v_takes_the_whole_representative"]),
    ("shared_v_scale_dropped", "s[t] = scale * acc;", "s[t] = acc;", 3, ["pin_shared_v_takes_the_whole_representative"]),
    ("closest_representative_is_farthest", "if (best < 0 || dist < best_d) {", "if (best < 0 || dist > best_d) {", 0,
     ["pin_closest_representatives"]),
    ("closest_representative_ties_to_highest", "if (best < 0 || dist < best_d) {", "if (best < 0 || dist <= best_d) {", 0,
     ["pin_closest_representatives"]),
    ("closest_representative_mean_over_all_heads", "mean[f] = acc / (double)cnt;", "mean[f] = acc / (double)H;", 1,
     ["pin_closest_representatives"]),
    ("prefill_sees_one_key_too_few", "const int n = q_start + i + 1;               /* keys this row sees */",
     "const int n = q_start + i > 0 ? q_start + i : 1;", 0, ["pin_prefill_matches_library_and_decode"]),
    ("prefill_not_causal", "const int n = q_start + i + 1;               /* keys this row sees */",
     "const int n = q_start + Tq;", 0, ["pin_prefill_matches_library_and_decode"]),
    ("prefill_query_row_stride", "int64_t qoff = (((int64_t)b * H + r) * Tq + i) * d;",
     "int64_t qoff = (((int64_t)b * H + r) * Tq + (Tq - 1 - i)) * d;", 0, ["pin_prefill_matches_library_and_decode"]),
    ("projection_uses_slot_index_as_head", "int64_t woff = ((int64_t)r * d + c) * D;", "int64_t woff = ((int64_t)j * d + c) * D;", 0,
     ["pin_projection_of_representatives"]),
    ("projection_keys_from_query_weights", "ak += xe * load_elem(w_k, woff + e, dtype);", "ak += xe * load_elem(w_q, woff + e, dtype);", 0,
     ["pin_projection_of_representatives"]),
    ("projection_weight_read_column_major", "int64_t woff = ((int64_t)r * d + c) * D;", "int64_t woff = ((int64_t)r * d + c);", 0,
     ["pin_projection_of_representatives"]),
    ("projection_token_stride", "int64_t xoff = ((int64_t)b * Tn + i) * D;", "int64_t xoff = ((int64_t)b * Tn) * D + i;", 0,
     ["pin_projection_of_representatives"]),
    ("compaction_source_stride", "int64_t src = ((int64_t)b * H + r) * T_cap + t;", "int64_t src = ((int64_t)b * H + r) * Tc_cap + t;", 0,
     ["pin_compaction_is_a_gather"]),
    ("compaction_copies_cluster_id_head", "int64_t src = ((int64_t)b * H + r) * T_cap + t;", "int64_t src = ((int64_t)b * H + j) * T_cap + t;", 0,
     ["pin_compaction_is_a_gather"]),
    ("append_all_keys_from_head_0", "(const char *)k_new + ((size_t)b * H + r) * row, row);", "(const char *)k_new + ((size_t)b * H + 0) * row, row);", 0,
     ["pin_append_writes_one_row"]),
    ("e4m3_decode_bias_8", "else mag = ldexp(1.0 + (double)m / 8.0, e - 7);", "else mag = ldexp(1.0 + (double)m / 8.0, e - 8);", 0,
     ["pin_e4m3_codes_match_the_format"]),
    ("e4m3_decode_subnormals_as_normals", "if (e == 0) mag = ldexp((double)m / 8.0, 1 - 7);",
     "if (e == 0) mag = ldexp(1.0 + (double)m / 8.0, 0 - 7);", 0, ["pin_e4m3_codes_match_the_format"]),
    ("e4m3_encode_truncates", "double r = nearbyint(a / step);", "double r = floor(a / step);", 0,
     ["pin_e4m3_encode_is_nearest_even"]),
    ("e4m3_encode_ties_away_from_zero", "double r = nearbyint(a / step);", "double r = round(a / step);", 0,
     ["pin_e4m3_encode_is_nearest_even"]),
    ("e4m3_encode_no_subnormal_spacing", "if (e < -6) e = -6;", "if (e < -9) e = -9;", 0,
     ["pin_e4m3_encode_is_nearest_even", "pin_quantized_rows"]),
    ("e4m3_encode_does_not_saturate", "if (a >= 448.0) return sign | 0x7e;", "if (a >= 448.0) return sign | 0x7f;", 0,
     ["pin_e4m3_encode_is_nearest_even", "pin_quantized_rows"]),
    ("quantize_scale_to_240", "float scale = amax / 448.0f;", "float scale = amax / 240.0f;", 0, ["pin_quantized_rows"]),
    ("quantize_amax_signed", "float v = fabsf((float)load_elem(x, r * d + i, dtype));", "float v = (float)load_elem(x, r * d + i, dtype);", 0,
     ["pin_quantized_rows"]),
    ("q8_key_scale_of_first_row", "* (double)kscale[row0 + t];", "* (double)kscale[row0];", 0,
     ["pin_quantized_attention_matches_library"]),
    ("q8_value_scale_dropped", "* (double)vscale[row0 + t];", ";", 0, ["pin_quantized_attention_matches_library"]),
    ("q8_values_of_representative", "int64_t row0 = ((int64_t)b * H + h) * (int64_t)T_cap;",
     "int64_t row0 = ((int64_t)b * H + rep_heads[(int64_t)b * k + c]) * (int64_t)T_cap;", 0,
     ["pin_quantized_attention_matches_library"]),
    ("append_row_off_by_one", "* T_cap + pos) * row,", "* T_cap + pos - 1) * row,", 0, ["pin_append_writes_one_row"]),
]
# a mutant made of several edits: the feature block computed without the causal mask
MULTI = {
    "features_not_causal": (
        [("for (int j = 0; j <= i; ++j) {\n                    double acc = 0.0;\n                    for (int c = 0; c < d; ++c)",
          "for (int j = 0; j < n_tok; ++j) {\n                    double acc = 0.0;\n                    for (int c = 0; c < d; ++c)", 0),
         ("softmax_row(s, i + 1, p);", "softmax_row(s, n_tok, p);", 0),
         ("f[i * n_tok + j] = (j <= i) ? (float)p[j] : 0.0f;", "f[i * n_tok + j] = (float)p[j];", 0)],
        ["pin_features_worked_example", "pin_features_match_library"]),
}
MUTANTS += [(name, None, None, 0, pins) for name, (_, pins) in MULTI.items()]


def _replace_nth(text, old, new, n):
    pos = -1
    for _ in range(n + 1):
        pos = text.find(old, pos + 1)
        assert pos >= 0, f"mutation site not found: {old!r} (occurrence {n})"
    return text[:pos] + new + text[pos + len(old):]


@pytest.fixture(scope="module")
def source():
    with open(SRC) as f:
        return f.read()


@pytest.mark.parametrize("name,old,new,nth,pins", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(tmp_path, source, name, old, new, nth, pins):
    if name in MULTI:
        text = source
        for o, n, i in MULTI[name][0]:
            text = _replace_nth(text, o, n, i)
    else:
        text = _replace_nth(source, old, new, nth)
    assert text != source
    c = tmp_path / "mutant.c"
    so = tmp_path / f"libmutant_{name}.so"
    c.write_text(text)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC", str(c), "-o",
                    str(so), "-lm"], check=True)
    caught = []
    with O.use_library(str(so)):
        for pin in pins:
            try:
                getattr(P, pin)()
            except AssertionError:
                caught.append(pin)
    assert caught, f"mutant {name} passed {pins}"


def test_unmutated_copy_passes_the_same_pins(tmp_path, source):
    """The harness itself does not make pins fail: an unedited copy built the same way passes all of them."""
    c = tmp_path / "copy.c"
    so = tmp_path / "libcopy.so"
    c.write_text(source)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC", str(c), "-o",
                    str(so), "-lm"], check=True)
    with O.use_library(str(so)):
        for pin in P.ALL_PINS:
            pin()
