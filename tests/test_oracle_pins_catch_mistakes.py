"""The oracle's pins are only worth something if they fail when the oracle is wrong.

Each case below plants one plausible mistake (a dropped term, a wrong sign, swapped
weights, a lost tie-break, an off-by-one in an index) in a *copy* of the oracle's C
source, compiles the copy, points the oracle's Python driver at it and runs the
pin tests named for that part of the algorithm: at least one of them must fail.
Everything happens on the CPU; the oracle that the other tests use is untouched.
"""
import ctypes as C
import os
import subprocess

import numpy as np
import pytest

from oracle import ivf_oracle as orc
import test_oracle_build as pins_build
import test_oracle_query as pins_query

SRC = os.path.join(os.path.dirname(os.path.abspath(orc.__file__)), "ivf_oracle.c")

# name -> (text in the source, replacement, pin tests that cover it)
MUTATIONS = {
    "eq7_constant_dropped": (
        "(1.0 - a) * d_c + a * d_s - a * (1.0 - a) * (double)cs_dist2[r * L + l];",
        "(1.0 - a) * d_c + a * d_s;",
        ["test_scores_equal_distance_to_explicit_subcentroid", "test_hand_example_eq7_eq6"]),
    "eq7_constant_sign": (
        "(1.0 - a) * d_c + a * d_s - a * (1.0 - a) * (double)cs_dist2[r * L + l];",
        "(1.0 - a) * d_c + a * d_s + a * (1.0 - a) * (double)cs_dist2[r * L + l];",
        ["test_scores_equal_distance_to_explicit_subcentroid", "test_hand_example_eq7_eq6"]),
    "eq7_weights_swapped": (
        "(1.0 - a) * d_c + a * d_s - a",
        "a * d_c + (1.0 - a) * d_s - a",
        ["test_scores_alpha_zero_and_one", "test_scores_equal_distance_to_explicit_subcentroid"]),
    "lut_sign": (
        "T[(q * M + m) * 256 + j] = -2.0 * s;",
        "T[(q * M + m) * 256 + j] = 2.0 * s;",
        ["test_lut_is_inner_product_table", "test_scan_equals_distance_to_explicitly_decoded_points"]),
    "lut_factor": (
        "T[(q * M + m) * 256 + j] = -2.0 * s;",
        "T[(q * M + m) * 256 + j] = -1.0 * s;",
        ["test_lut_is_inner_product_table", "test_scan_equals_distance_to_explicitly_decoded_points"]),
    "scan_constant_dropped": (
        "d += const_exact ? const_exact[i] : (double)const_table[const_byte[i]];",
        "d += 0.0;",
        ["test_scan_equals_distance_to_explicitly_decoded_points", "test_hand_example_eq7_eq6"]),
    "tie_break_lost": (
        "    if (a->t < b->t) return -1;\n    if (a->t > b->t) return 1;\n    return 0;",
        "    if (a->t < b->t) return 1;\n    if (a->t > b->t) return -1;\n    return 0;",
        ["test_smallest_against_python_sort", "test_probe_is_bruteforce_knn_with_id_tiebreak",
         "test_prune_is_global_bruteforce_sort"]),
    "neighbours_contain_self": (
        "row[j] = (j == r) ? INFINITY : sq_dist(C + r * D, C + j * D, D);",
        "row[j] = sq_dist(C + r * D, C + j * D, D);",
        ["test_neighbours_bruteforce_excluding_self"]),
    "alpha_without_clamp": (
        "        double a = den[r] > 0.0 ? num[r] / den[r] : pooled;\n        if (a < 0.0) a = 0.0;\n        if (a > 1.0) a = 1.0;",
        "        double a = den[r] > 0.0 ? num[r] / den[r] : pooled;",
        ["test_alpha_clamped_and_degenerate"]),
    "alpha_residual_sign": (
        "double res = xc2 - 2.0 * a * dot + a * a * n2;",
        "double res = xc2 + 2.0 * a * dot + a * a * n2;",
        ["test_alpha_hand_example", "test_alpha_recovers_planted_factor_and_minimises_objective"]),
    "constant_term_factor": (
        "s += 2.0 * mu[i * D + m * ds + c] * r + r * r;",
        "s += mu[i * D + m * ds + c] * r + r * r;",
        ["test_scan_equals_distance_to_explicitly_decoded_points", "test_sub_assign_and_encode_against_numpy_bruteforce"]),
    "prune_subregion_id": (
        "sid[p * L + l] = (int64_t)probe_id[q * P + p] * L + l;",
        "sid[p * L + l] = (int64_t)p * L + l;",
        ["test_prune_is_global_bruteforce_sort"]),
    "select_tie_by_position": (
        "tie[i] = ids[cand_pos[i]];",
        "tie[i] = cand_pos[i];",
        ["test_select_bruteforce_and_padding"]),
    "pq_codeword_block": (
        "double u = E[i * D + m * ds + t] - (double)codebook[((int64_t)m * 256 + j) * ds + t];",
        "double u = E[i * D + m * ds + t] - (double)codebook[((int64_t)j * ds) + t];",
        ["test_sub_assign_and_encode_against_numpy_bruteforce"]),
    "quantiser_tie_rule": (
        "            double d = fabs(t[i] - (double)table[j]);\n            if (d < best) { best = d; bj = j; }",
        "            double d = fabs(t[i] - (double)table[j]);\n            if (d <= best) { best = d; bj = j; }",
        ["test_scalar_quantiser"]),
    "budget_stops_before_crossing": (
        "visit[q * S + at] = collected < R ? 1 : 0;\n            if (collected < R) collected += (int64_t)sub_offsets[b + 1] - (int64_t)sub_offsets[b];",
        "collected += (int64_t)sub_offsets[b + 1] - (int64_t)sub_offsets[b];\n            visit[q * S + at] = collected <= R ? 1 : 0;",
        ["test_budget_walk_against_python_traversal"]),
    "budget_order_by_position": (
        "orc_smallest(kept_score + q * S, kept_sub + q * S, S, S, order, val);",
        "orc_smallest(kept_score + q * S, NULL, S, S, order, val);",
        ["test_budget_walk_against_python_traversal"]),
    "budget_counts_subregions": (
        "if (collected < R) collected += (int64_t)sub_offsets[b + 1] - (int64_t)sub_offsets[b];",
        "if (collected < R) collected += 1;",
        ["test_budget_walk_against_python_traversal", "test_budget_nested_and_unbounded_budget_is_plain_search"]),
    "rotation_transposed": (
        "for (int b = 0; b < D; ++b) s += (double)R[(int64_t)a * D + b] * X[i * D + b];",
        "for (int b = 0; b < D; ++b) s += (double)R[(int64_t)b * D + a] * X[i * D + b];",
        ["test_rotate_is_the_matrix_product", "test_rotated_scan_equals_distance_to_points_decoded_in_the_original_space"]),
    "rotation_not_applied_to_query": (
        "            orc_rotate(qin, 1, D, rotation, qr);",
        "            (void)qin;",
        ["test_rotated_scan_equals_distance_to_points_decoded_in_the_original_space"]),
    "subcentroid_weights": (
        "double mu = (double)c[t] + a * ((double)s[t] - (double)c[t]);",
        "double mu = (double)c[t] + (1.0 - a) * ((double)s[t] - (double)c[t]);",
        ["test_sub_assign_and_encode_against_numpy_bruteforce"]),
}


def _pin(name):
    for mod in (pins_query, pins_build):
        if hasattr(mod, name):
            return getattr(mod, name)
    raise KeyError(name)


def _call(fn, tiny):
    """Calls a pin test with the fixtures it asks for."""
    import inspect
    args = {}
    for p in inspect.signature(fn).parameters:
        if p == "tiny":
            args[p] = tiny
        elif p == "rng":
            args[p] = np.random.default_rng(20180207)
        else:
            raise KeyError(p)
    fn(**args)


@pytest.fixture
def swapped_oracle(tmp_path):
    """Yields a function that loads a mutated build as the driver's library; restores the real one."""
    real = orc.lib()

    def load(old, new):
        text = open(SRC).read()
        assert text.count(old) >= 1, old
        out_c, out_so = tmp_path / "mutant.c", tmp_path / "mutant.so"
        out_c.write_text(text.replace(old, new))
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", str(out_so), str(out_c), "-lm"])
        m = C.CDLL(str(out_so))
        m.orc_num_kept.restype = C.c_int64
        m.orc_num_kept.argtypes = [C.c_double, C.c_int64, C.c_int]
        orc._lib = m

    yield load
    orc._lib = real


def test_the_pins_pass_on_the_real_oracle(tiny):
    for name in sorted({n for _, _, names in MUTATIONS.values() for n in names}):
        _call(_pin(name), tiny)


@pytest.mark.parametrize("mutation", sorted(MUTATIONS))
def test_a_planted_mistake_fails_a_pin(mutation, tiny, swapped_oracle):
    old, new, names = MUTATIONS[mutation]
    swapped_oracle(old, new)
    caught = []
    for name in names:
        try:
            _call(_pin(name), tiny)
        except AssertionError:
            caught.append(name)
    assert caught, f"no pin noticed the mistake '{mutation}' (ran {names})"
