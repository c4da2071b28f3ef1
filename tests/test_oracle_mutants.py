"""Are the oracle's pins sharp?  Plant one plausible mistake at a time in a COPY of the oracle
source (CPU only), build it, point the ctypes wrapper at it, and require that at least one pin
from test_oracle_sparse / test_oracle_cluster fails.  The oracle itself is never modified.
"""
import ctypes
import os
import subprocess

import pytest

import oracle
import conftest
import test_oracle_cluster as tc
import test_oracle_sparse as ts
import test_oracle_variants as tv

SRC = os.path.join(os.path.dirname(oracle.__file__), "bitsnap_oracle.c")

# (name, text to find, replacement, occurrence index)
MUTANTS = [
    ("mask_msb_first", "(1u << (i & 7))", "(0x80u >> (i & 7))", 0),
    ("payload_takes_base", "payload[nc] = cur[i];", "payload[nc] = base[i];", 0),
    ("payload_stores_difference", "payload[nc] = cur[i];", "payload[nc] = (uint16_t)(cur[i] - base[i]);", 0),
    ("delta_payload_is_sum", "payload[nc] = delta ? (uint16_t)(c ^ b) : c;", "payload[nc] = delta ? (uint16_t)(c + b) : c;", 0),
    ("delta_decode_drops_base", "out[i] = delta ? (uint16_t)(base[i] ^ payload[r]) : payload[r];", "out[i] = payload[r];", 0),
    ("new_base_only_where_changed", "        if (new_base)\n            new_base[i] = c;\n    }", "        if (new_base && c != b)\n            new_base[i] = c;\n    }", 0),
    ("wide_elements_compare_low_half", "        const uint32_t c = cur[i], b = base[i];\n        if (c != b) {", "        const uint32_t c = cur[i], b = base[i];\n        if ((uint16_t)c != (uint16_t)b) {", 0),
    ("wide_delta_decode_drops_base", "out[i] = delta ? (base[i] ^ payload[r]) : payload[r];", "out[i] = payload[r];", 0),
    ("offsets_inclusive", "off[t] = run;", "off[t] = run + 1;", 0),
    ("sample_std", "sqrt(q / (double)len)", "sqrt(q / (double)(len - 1))", 0),
    ("mean_not_subtracted", "double d = (double)x[i] - mean;", "double d = (double)x[i];", 0),
    ("edge_sign", "double e = (double)mu + prod;", "double e = (double)mu - prod;", 0),
    ("edge_strict_compare", "if (edges[k - 1] <= x)", "if (edges[k - 1] < x)", 0),
    ("quantile_k_plus_1", "long double p = (long double)k / (long double)m;", "long double p = (long double)(k + 1) / (long double)(m + 2);", 0),
    ("scale_is_max", "seen[c] ? (mx[c] - mn[c]) : 0.0f;", "seen[c] ? mx[c] : 0.0f;", 0),
    ("offset_is_max", "seen[c] ? mn[c] : 0.0f;", "seen[c] ? mx[c] : 0.0f;", 0),
    ("params_swapped", "pg[2 * l + 1], pg[2 * l + 0]);", "pg[2 * l + 0], pg[2 * l + 1]);", 0),
    ("code_without_offset", "float d = x - b;", "float d = x;", 0),
    ("code_floor", "float r = rintf(y);", "float r = floorf(y);", 0),
    ("code_ties_away_from_zero", "float r = rintf(y);", "float r = roundf(y);", 0),
    ("code_256_levels", "float inv = 255.0f / S;", "float inv = 256.0f / S;", 0),
    ("label_nibbles_swapped", "(l << ((idx & 1) * 4))", "(l << ((1 - (idx & 1)) * 4))", 0),
    ("dequant_drops_offset", "out[i] = t + b;", "out[i] = t;", 0),
    ("dequant_wrong_group", "int64_t g = i / G;", "int64_t g = 0;", 0),
    # format variants: a general map Q, cluster-major codes
    ("table_tie_takes_highest", "if (dist < bd) {", "if (dist <= bd) {", 0),
    ("table_code_without_offset", "float d = x - b;", "float d = x;", 1),
    ("table_scaled_to_255", "float inv = 1.0f / S;", "float inv = 255.0f / S;", 0),
    ("table_distance_signed", "float dist = fabsf(qmap[j] - t);", "float dist = qmap[j] - t;", 0),
    ("table_dequant_drops_scale", "t = qmap[q] * S;", "t = qmap[q];", 0),
    ("table_dequant_linear_levels", "t = qmap[q] * S;", "t = (float)q / 255.0f * S;", 0),
    ("major_clusters_descending", "for (int c = 0; c < m; ++c)\n                for (int64_t i = 0; i < len; ++i) {",
     "for (int c = m - 1; c >= 0; --c)\n                for (int64_t i = 0; i < len; ++i) {", 0),
    ("major_members_reversed", "for (int c = 0; c < m; ++c)\n                for (int64_t i = 0; i < len; ++i) {",
     "for (int c = 0; c < m; ++c)\n                for (int64_t i = len - 1; i >= 0; --i) {", 0),
    ("major_over_the_whole_tensor", "uint8_t q = cluster_major ? codes[lo + start[l] + seen[l]] : codes[idx];",
     "uint8_t q = cluster_major ? codes[start[l] + seen[l]] : codes[idx];", 0),
    ("decluster_start_off_by_one_cluster", "start[c] = start[c - 1] + count[c - 1];", "start[c] = start[c - 1] + count[c];", 0),
    ("decluster_rank_not_advanced", "            seen[l] += 1;\n", "", 0),
]


def _pins(golden):
    yield lambda: ts.test_roundtrip_lossless(4097, 0.06)
    yield lambda: ts.test_roundtrip_lossless(65, 1.0)
    yield lambda: ts.test_space_formula_and_ratios(golden)
    yield lambda: ts.test_mask_payload_offsets_against_library_routines(4097)
    yield lambda: ts.test_naive_mask_and_coo_crossovers(golden)
    yield ts.test_decode_uses_payload_in_order
    yield lambda: ts.test_delta_payload_is_the_nonzero_part_of_the_bitwise_difference(4097, 0.06)
    yield lambda: ts.test_new_base_is_a_copy_of_cur_also_in_place(True)
    yield lambda: ts.test_32_bit_elements_against_library_routines(4097, 0.06, True)
    yield lambda: tc.test_quantiles_are_correctly_rounded(16)
    yield tc.test_equal_probability_edges
    yield tc.test_fit_exact_on_integers
    yield lambda: tc.test_fit_against_exact_summation(0)
    yield lambda: tc.test_labels_equal_searchsorted(16)
    yield lambda: tc.test_params_are_cluster_min_and_range(4096)
    yield tc.test_error_bound_endpoints_and_monotone_codes
    yield lambda: tc.test_codes_against_bruteforce_argmin(4)
    yield tc.test_one_cluster_is_plain_minmax_uint8
    yield lambda: tc.test_exact_ties_round_to_the_even_code(1.0)
    yield tc.test_dequantize_formula
    yield lambda: tc.test_stored_size_formula(golden)
    yield tc.test_degenerate_groups
    yield lambda: tv.test_cluster_major_is_a_stable_sort_by_label_inside_each_group(1000, 4321)
    yield tv.test_cluster_major_on_a_hand_made_group
    yield lambda: tv.test_decluster_returns_every_value_to_its_position(512, 5000, 7)
    yield lambda: tv.test_table_codes_are_the_nearest_entries("normal")
    yield lambda: tv.test_table_codes_against_exhaustive_search("square")
    yield tv.test_exact_ties_and_repeated_entries_take_the_lowest_index
    yield lambda: tv.test_table_dequantisation_error_is_within_half_a_gap("square")
    yield tv.test_table_dequantise_on_hand_made_inputs


@pytest.mark.parametrize("name,find,repl,occ", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, find, repl, occ):
    golden = conftest.load_golden("paper_closed_forms.txt")
    text = open(SRC).read()
    parts = text.split(find)
    assert len(parts) > occ + 1, f"mutation site for {name} not found: the oracle changed, update this list"
    text = find.join(parts[: occ + 1]) + repl + find.join(parts[occ + 1:])
    src = tmp_path / "mutant.c"
    lib = tmp_path / "libmutant.so"
    src.write_text(text)
    subprocess.run(["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-ffp-contract=off", "-o", str(lib), str(src), "-lm"],
                   check=True)
    good = oracle._load()
    mut = ctypes.CDLL(str(lib))
    for sym in ("oracle_encode_sparse", "oracle_encode_sparse_ex", "oracle_decode_sparse_ex", "oracle_encode_sparse32_ex", "oracle_decode_sparse32_ex", "oracle_encode_sparse_naive", "oracle_tile_offsets", "oracle_decode_sparse",
                "oracle_norm_quantile", "oracle_cluster_fit", "oracle_cluster_edges", "oracle_quantize_cluster",
                "oracle_dequantize_cluster", "oracle_code_bruteforce", "oracle_quantize_cluster_ex",
                "oracle_dequantize_cluster_ex", "oracle_code_qmap_bruteforce"):
        getattr(mut, sym).argtypes = getattr(good, sym).argtypes
        getattr(mut, sym).restype = getattr(good, sym).restype
    oracle._lib = mut
    try:
        caught = False
        for pin in _pins(golden):
            try:
                pin()
            except AssertionError:
                caught = True
                break
        assert caught, f"no pin noticed the planted mistake '{name}'"
    finally:
        oracle._lib = good
