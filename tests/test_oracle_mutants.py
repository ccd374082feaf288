"""The pins have teeth: each planted mistake in a copy of the oracle's C source (built
and run on the CPU only) must be caught by at least one pin."""
import os
import subprocess

import pytest

import oracle
from pins import ALL_PINS

SRC = os.path.join(os.path.dirname(oracle.__file__), "evo_oracle.c")

# (name, text in evo_oracle.c, replacement)
MUTANTS = [
    ("tolerance_scaled_by_candidate", "const float scaled = rtol * ar;", "const float scaled = rtol * fabsf(c);"),
    ("tolerance_fused_multiply_add", "const float tol = atol + scaled;", "const float tol = fmaf(rtol, ar, atol);"),
    ("tolerance_product_in_binary64", "const float tol = atol + scaled;", "const float tol = (float)((double)atol + (double)rtol * (double)ar);"),
    ("f64_tolerance_fused_multiply_add", "const double tol_d = atol_d + scaled_d;", "const double tol_d = fma(rtol_d, ard, atol_d);"),
    ("tolerance_drops_atol", "const float tol = atol + scaled;", "const float tol = scaled;"),
    ("tolerance_drops_rtol", "const float tol = atol + scaled;", "const float tol = atol;"),
    ("strict_less_than", "match = (d <= tol);", "match = (d < tol);"),
    ("no_equality_shortcut", "if (c == r) {", "if (0) {"),
    ("no_finiteness_guard", "} else if (r_fin && c_fin) {", "} else if (1) {"),
    ("signed_difference", "const float d = fabsf(c - r);\n            match", "const float d = (c - r);\n            match"),
    ("difference_becomes_sum", "const float d = fabsf(c - r);\n            match", "const float d = fabsf(c + r);\n            match"),
    ("division_instead_of_reciprocal", "q = d * inv;", "q = (inv != 0.0f) ? d / ar : 0.0f;"),
    ("fmin_threshold_exclusive", "if (ar >= 1.17549435e-38f)", "if (ar > 1.17549435e-38f)"),
    ("rel_sum_adds_abs", "a->sum_rel_err += (double)q;", "a->sum_rel_err += (double)d;"),
    ("fp32_sum", "a->sum_abs_err += (double)d;", "a->sum_abs_err = (double)((float)a->sum_abs_err + d);"),
    ("max_abs_is_min", "if (d > a->max_abs_err)", "if (d < a->max_abs_err)"),
    ("max_rel_tracks_abs", "if (q > a->max_rel_err) a->max_rel_err = q;", "if (d > a->max_rel_err) a->max_rel_err = d;"),
    ("stats_include_nonfinite", "        if (r_fin && c_fin) {\n            const float d = fabsf(c - r); /* may", "        if (r_fin) {\n            const float d = fabsf(c - r); /* may"),
    ("nan_site_one_sided", "if (c_nan != r_nan)", "if (c_nan && !r_nan)"),
    ("inf_diff_ignores_equality", "&& !c_nan && !r_nan && c != r)", "&& !c_nan && !r_nan)"),
    ("cand_ref_flags_swapped", "if (c_inf) a->flags |= ORACLE_F_CAND_INF;", "if (c_inf) a->flags |= ORACLE_F_REF_INF;"),
    ("bf16_shift", "(uint32_t)h << 16", "(uint32_t)h << 15"),
    ("f16_bias", "w = sign | ((exp + 112u) << 23) | (frac << 13);", "w = sign | ((exp + 111u) << 23) | (frac << 13);"),
    ("f16_subnormal_exponent", "w = sign | ((uint32_t)(113 - shift) << 23) | (frac << 13);", "w = sign | ((uint32_t)(112 - shift) << 23) | (frac << 13);"),
    ("f16_nan_payload_dropped", "w = sign | 0x7f800000u | (frac << 13);", "w = sign | 0x7f800000u;"),
    ("median_upper_middle", "const float s = scratch[T / 2 - 1] + scratch[T / 2];", "const float s = scratch[T / 2] + scratch[T / 2];"),
    ("median_no_half", "*median = 0.5f * s;", "*median = s;"),
    ("odd_median_off_by_one", "*median = scratch[T / 2];", "*median = scratch[(T - 1) / 2 + (T > 1)];"),
    ("mean_of_sorted_is_fine_but_wrong_divisor", "acc / (double)T", "acc / (double)(T + 1)"),
    ("speedup_inverted", "speedup[p] = base_median / median_ms[p];", "speedup[p] = median_ms[p] / base_median;"),
    ("invalid_keeps_fitness", "fitness[p] = valid[p] ? speedup[p] : 0.0f;", "fitness[p] = speedup[p];"),
    ("last_of_ties_wins", "if (fitness[p] > best_fit) {", "if (fitness[p] >= best_fit) {"),
    ("no_floor", "pop->best_speedup = (best_fit > 1.0f) ? best_fit : 1.0f;", "pop->best_speedup = best_fit;"),
    ("zero_sample_accepted", "if (!(row[k] > 0.0f) || isinf(row[k]))", "if (!(row[k] >= 0.0f) || isinf(row[k]))"),
    ("inf_sample_accepted", "if (!(row[k] > 0.0f) || isinf(row[k]))", "if (!(row[k] > 0.0f))"),
    ("elite_last_of_ties", "if (best == P || fitness[i] > fitness[best])", "if (best == P || fitness[i] >= fitness[best])"),
    ("elite_takes_infeasible", "            if (!(fitness[i] > 0.0f))\n                continue;", "            if (0)\n                continue;"),
    ("elite_worst_first", "if (best == P || fitness[i] > fitness[best])", "if (best == P || fitness[i] < fitness[best])"),
    ("valid_rate_over_T", "(float)n_valid / (float)P", "(float)n_valid / (float)T"),
    ("f64_tolerance_scaled_by_candidate", "const double scaled_d = rtol_d * ard;", "const double scaled_d = rtol_d * fabs(cd);"),
    ("f64_strict_less_than", "match = (fabs(cd - rd) <= tol_d);", "match = (fabs(cd - rd) < tol_d);"),
    ("f64_difference_in_binary32", "match = (fabs(cd - rd) <= tol_d);", "match = (fabs((double)((float)cd - (float)rd)) <= tol_d);"),
    ("f64_no_equality_shortcut", "if (cd == rd)", "if (0)"),
    ("f64_no_finiteness_guard", "else if (rd_fin && cd_fin)", "else if (1)"),
    ("f64_dbl_min_exclusive", "if (ard >= 2.2250738585072014e-308)", "if (ard > 2.2250738585072014e-308)"),
    ("f64_binary32_threshold", "if (ard >= 2.2250738585072014e-308)", "if (ard >= 1.17549435e-38)"),
    ("f64_sum_of_rounded_terms", "a->sum_abs_err += dd;", "a->sum_abs_err += (double)d32;"),
    ("f64_division_instead_of_reciprocal", "qd = dd * inv_d;", "qd = (inv_d != 0.0) ? dd / ard : 0.0;"),
    ("f64_rel_max_tracks_abs", "if (q32 > a->max_rel_err) a->max_rel_err = q32;", "if (d32 > a->max_rel_err) a->max_rel_err = d32;"),
    ("f64_nan_site_one_sided", "if (cd_nan != rd_nan)", "if (cd_nan && !rd_nan)"),
    ("int_mismatch_one_sided", "        if (c != r)\n            a->n_mismatch += 1;", "        if (c > r)\n            a->n_mismatch += 1;"),
    ("int_off_by_one_tolerated", "        if (c != r)\n            a->n_mismatch += 1;", "        if (c > r + 1 || r > c + 1)\n            a->n_mismatch += 1;"),
    ("int_difference_not_a_magnitude", "diff = (c > r) ? (uint64_t)c - (uint64_t)r : (uint64_t)r - (uint64_t)c;", "diff = (uint64_t)c - (uint64_t)r;"),
    ("int_difference_in_32_bits", "diff = (c > r) ? (uint64_t)c - (uint64_t)r : (uint64_t)r - (uint64_t)c;", "diff = (uint32_t)((c > r) ? (uint64_t)c - (uint64_t)r : (uint64_t)r - (uint64_t)c);"),
    ("int_reference_read_unsigned", "r = ((const int32_t *)ref)[i];", "r = ((const uint32_t *)ref)[i];"),
    ("int_sum_in_binary32", "a->sum_abs_err += (double)diff;", "a->sum_abs_err += (double)diff32;"),
    ("int_not_counted_finite", "        diff32 = (float)diff;\n        a->n_finite += 1;", "        diff32 = (float)diff;"),
    ("mean_reducer_keeps_median_baseline", "speedup[p] = base_mean / mean_ms[p];", "speedup[p] = base_median / mean_ms[p];"),
    ("mean_reducer_ignored", "else if (reducer == ORACLE_REDUCE_MEAN)", "else if (0)"),
    ("diverse_ignores_keys", "                if (keys[elite[q]] == keys[i])\n                    key_taken = 1;", "                if (elite[q] == i)\n                    key_taken = 1;"),
    ("diverse_infeasible_blocks_key", "            int key_taken = 0;\n            if (!(fit[i] > 0.0f))\n                continue;", "            int key_taken = 0;\n            if (0)\n                continue;"),
    ("diverse_last_of_ties", "                top = i; /* strict: of equal fitness the first wins */", "                top = i; /* mutated */\n            else if (fit[i] == fit[top]) top = i;"),
    ("mean_reducer_always", "else if (reducer == ORACLE_REDUCE_MEAN)", "else if (1)"),
]


@pytest.fixture(scope="module")
def source():
    with open(SRC) as fh:
        return fh.read()


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(name, old, new, source, tmp_path):
    assert source.count(old) == 1, "mutation site must be unique: %r" % old
    c_path = tmp_path / (name + ".c")
    so_path = tmp_path / (name + ".so")
    c_path.write_text(source.replace(old, new))
    subprocess.check_call(["gcc", *oracle.CFLAGS, "-o", str(so_path), str(c_path), "-lm"])
    variant = oracle.Variant(str(so_path))
    caught = []
    for pin in ALL_PINS:
        try:
            pin(variant)
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, "no pin noticed the planted mistake '%s'" % name
