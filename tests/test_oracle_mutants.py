"""The pins must be able to fail: each plausible mistake planted in a copy of the
oracle's source (on the CPU, in a temporary build) has to be caught by at least
one pin of tests/test_oracle_codec.py or tests/test_oracle_qgz.py."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "zpp_oracle.c")

MUTANTS = {
    "truncate_instead_of_round_even": ("float r = nearbyintf(t);", "float r = truncf(t);"),
    "round_half_away": ("float r = nearbyintf(t);", "float r = roundf(t);"),
    "scale_divides_by_qmax_plus_one": ("const float scale = a / qmax;", "const float scale = a / (qmax + 1.0f);"),
    "inverse_from_rounded_scale": ("const float inv = qmax / a;", "const float inv = 1.0f / scale;"),
    "max_without_abs": ("float m = fabsf(v[i]);", "float m = v[i];"),
    "tiny_threshold_moved": ("if (a < 0x1p-100f) {", "if (a < 0x1p-60f) {"),
    "high_nibble_first": ("if (i & 1) *p = (uint8_t)((*p & 0x0fu) | (nib << 4));\n        else *p = (uint8_t)((*p & 0xf0u) | nib);",
                          "if (!(i & 1)) *p = (uint8_t)((*p & 0x0fu) | (nib << 4));\n        else *p = (uint8_t)((*p & 0xf0u) | nib);"),
    "nibble_order_swapped_both_ways": None,     # two edits, see below
    "reorder_roles_exchanged": ("long long j = w / Y, i = w % Y;\n    return st * T + i * X + j;",
                                "long long j = w % X, i = w / X;\n    return st * T + i * X + j;"),
    "reorder_drops_stage_offset": ("long long j = w / Y, i = w % Y;\n    return st * T + i * X + j;",
                                   "long long j = w / Y, i = w % Y;\n    return i * X + j;"),
    "fused_reorder_reads_unpermuted": ("size_t in_base = src * L + r * (size_t)block;",
                                       "size_t in_base = p * L + r * (size_t)block;"),
    "intra_sum_descending": ("for (int k = 0; k < X; ++k)\n                s = s + dequant_elem(codes_in[k]",
                             "for (int k = X - 1; k >= 0; --k)\n                s = s + dequant_elem(codes_in[k]"),
    "inter_sum_descending": ("for (int i = 0; i < Y; ++i)\n            s = s + dequant_elem(codes_in[i]",
                             "for (int i = Y - 1; i >= 0; --i)\n            s = s + dequant_elem(codes_in[i]"),
    "multiply_by_reciprocal_of_divisor": ("out[e] = s / divisor;", "out[e] = s * (1.0f / divisor);"),
    "decode_uses_first_scale": ("return q * scales[e / (size_t)B];", "return q * scales[0];"),
    "bf16_ties_away": ("if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) keep += 1;",
                       "if (rest >= 0x8000u) keep += 1;"),
    "f16_ties_away": ("if (rest > 0x1000u || (rest == 0x1000u && (keep & 1u))) h += 1;",
                      "if (rest >= 0x1000u) h += 1;"),
    "f16_subnormal_scale_wrong": ("float v = (float)m * 0x1p-24f;", "float v = (float)m * 0x1p-25f;"),
    "intra_sum_in_double": ("float s = 0.0f;\n            for (int k = 0; k < X; ++k)", "double s = 0.0;\n            for (int k = 0; k < X; ++k)"),
    "inter_sum_in_double": ("float s = 0.0f;\n        for (int i = 0; i < Y; ++i)", "double s = 0.0;\n        for (int i = 0; i < Y; ++i)"),
    "intra_decode_fused_into_the_add": (
        "s = s + dequant_elem(codes_in[k], scales_in[k], bits, block, base + (size_t)i);",
        "s = fmaf((float)get_code(codes_in[k], bits, base + (size_t)i), scales_in[k][(base + (size_t)i) / (size_t)block], s);"),
    "inter_divides_every_addend": None,         # two edits, see below
    "reorder_leaves_scales_unpermuted": ("scales[ob] = quant_block(v, block, bits, codes, out_base);",
                                         "scales[in_base / (size_t)block] = quant_block(v, block, bits, codes, out_base);"),
    "absmax_skips_last_element": ("for (int i = 0; i < B; ++i) {\n        float m = fabsf(v[i]);",
                                  "for (int i = 0; i < B - 1; ++i) {\n        float m = fabsf(v[i]);"),
    "nibble_eight_decoded_as_plus_eight": ("return nib >= 8 ? nib - 16 : nib;", "return nib > 8 ? nib - 16 : nib;"),
    "f16_overflows_just_above_max": ("if (a >= 65520.0f) return", "if (a > 65504.0f) return"),
    "f16_subnormal_narrowing_floors": ("float r = nearbyintf(a * 0x1p24f);", "float r = floorf(a * 0x1p24f);"),
    "scatter_map_is_not_the_inverse": ("long long i = w / X, j = w % X;\n    return st * T + j * Y + i;",
                                       "long long i = w / Y, j = w % Y;\n    return st * T + j * Y + i;"),
    "int8_code_sign_lost": ("if (bits == 8) return ((const int8_t*)codes)[i];", "if (bits == 8) return ((const uint8_t*)codes)[i];"),
}
TWO_EDITS = {
    "inter_divides_every_addend": [("s = s + dequant_elem(codes_in[i], scales_in[i], bits, block, (size_t)e);",
                                    "s = s + dequant_elem(codes_in[i], scales_in[i], bits, block, (size_t)e) / divisor;"),
                                   ("out[e] = s / divisor;", "out[e] = s;")],
    "nibble_order_swapped_both_ways": [MUTANTS["high_nibble_first"],
                                       ("int nib = (i & 1) ? (b >> 4) : (b & 0xf);", "int nib = (i & 1) ? (b & 0xf) : (b >> 4);")],
}


# the pin expected to catch each mistake (run first; every pin is tried if it does not)
CAUGHT_BY = {
             'intra_sum_in_double': 'tests/test_oracle_qgz.py::test_intra_reduce_matches_ordered_replay',
             'inter_sum_in_double': 'tests/test_oracle_qgz.py::test_inter_reduce_matches_ordered_replay',
             'intra_decode_fused_into_the_add': 'tests/test_oracle_qgz.py::test_intra_reduce_matches_ordered_replay',
             'inter_divides_every_addend': 'tests/test_oracle_qgz.py::test_inter_reduce_matches_ordered_replay',
             'reorder_leaves_scales_unpermuted': 'tests/test_oracle_qgz.py::test_fused_reorder_equals_quantize_then_permute',
             'absmax_skips_last_element': 'tests/test_oracle_codec.py::test_every_finite_fp16_value_matches_second_evaluator',
             'nibble_eight_decoded_as_plus_eight': 'tests/test_oracle_codec.py::test_every_code_value_decodes_as_twos_complement',
             'fused_reorder_reads_unpermuted': 'tests/test_oracle_qgz.py::test_fused_reorder_equals_quantize_then_permute',
             'reorder_roles_exchanged': 'tests/test_oracle_qgz.py::test_reorder_matches_the_papers_examples',
             'intra_sum_descending': 'tests/test_oracle_qgz.py::test_summation_order_is_ascending_peer_index',
             'max_without_abs': 'tests/test_oracle_codec.py::test_absmax_element_gets_extreme_code',
             'int8_code_sign_lost': 'tests/test_oracle_codec.py::test_power_of_two_grid_is_coded_exactly',
             'nibble_order_swapped_both_ways': 'tests/test_oracle_codec.py::test_int4_byte_layout_low_nibble_first',
             'f16_subnormal_scale_wrong': 'tests/test_oracle_codec.py::test_widen_f16_every_pattern_matches_numpy',
             'bf16_ties_away': 'tests/test_oracle_codec.py::test_narrow_bf16_matches_torch_rounding',
             'high_nibble_first': 'tests/test_oracle_codec.py::test_int4_byte_layout_low_nibble_first',
             'multiply_by_reciprocal_of_divisor': 'tests/test_oracle_qgz.py::test_two_hops_with_reorder_are_a_reduce_scatter',
             'reorder_drops_stage_offset': 'tests/test_oracle_qgz.py::test_stages_permute_inside_each_stage_only',
             'inter_sum_descending': 'tests/test_oracle_qgz.py::test_summation_order_is_ascending_peer_index',
             'round_half_away': 'tests/test_oracle_codec.py::test_ties_round_to_even',
             'decode_uses_first_scale': 'tests/test_oracle_codec.py::test_random_tensors_match_second_evaluator',
             'inverse_from_rounded_scale': 'tests/test_oracle_codec.py::test_every_finite_fp16_value_matches_second_evaluator',
             'scale_divides_by_qmax_plus_one': 'tests/test_oracle_codec.py::test_scale_is_correctly_rounded_quotient_exact_rational',
             'f16_ties_away': 'tests/test_oracle_codec.py::test_narrow_f16_matches_numpy_rounding',
             'truncate_instead_of_round_even': 'tests/test_oracle_codec.py::test_ties_round_to_even',
             'tiny_threshold_moved': 'tests/test_oracle_codec.py::test_zero_and_tiny_blocks'
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name, tmp_path):
    text = open(SRC).read()
    for old, new in TWO_EDITS.get(name) or [MUTANTS[name]]:
        assert text.count(old) == 1, f"mutation site for {name} not found exactly once"
        text = text.replace(old, new)
    src = tmp_path / "mutant.c"
    lib = tmp_path / "libmutant.so"
    src.write_text(text)
    subprocess.run(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC", "-shared",
                    str(src), "-o", str(lib), "-lm"], check=True)
    env = dict(os.environ, ZPP_ORACLE_LIB=str(lib))

    def pins(*targets):
        return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *targets],
                              env=env, cwd=ROOT, capture_output=True, text=True)

    first = CAUGHT_BY.get(name)
    r = pins(os.path.join(ROOT, *first.split("/"))) if first else None
    if r is None or r.returncode != 1:
        r = pins(os.path.join(ROOT, "tests", "test_oracle_qgz.py"), os.path.join(ROOT, "tests", "test_oracle_codec.py"))
    assert r.returncode == 1 and "failed" in r.stdout, f"mutant {name} survived every pin:\n{r.stdout[-2000:]}"
