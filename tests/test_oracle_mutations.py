"""Do the oracle's pins have teeth?  Each case plants one plausible mistake in a
copy of the oracle's C source (CPU only), builds it, swaps it in for the real
library and expects at least one pin to fail."""
import os
import subprocess

import pytest

import oracle
import test_oracle_pack_unpack as pins_pack
import test_oracle_stats_awp as pins_stats
import test_oracle_unpack16 as pins16

SRC = os.path.join(os.path.dirname(oracle.__file__), "adt_oracle.c")

PACK_PINS = [
    pins_pack.test_worked_examples_from_ieee754,
    pins_pack.test_format_field_widths_of_section_v_a,
    pins_pack.test_figure2_size_and_order,
    pins_pack.test_four_bytes_is_memcpy_and_identity,
    pins_pack.test_two_bytes_is_bfloat16_by_truncation,
    lambda: [pins_pack.test_stream_equals_numpy_byte_slicing(r) for r in (1, 2, 3, 4)],
    pins_pack.test_layers_concatenate_without_padding,
    pins_pack.test_invariants,
    pins_pack.test_special_values_documented_behaviour,
    lambda: [pins16.test_bf16_is_the_two_byte_stream_of_the_same_weights(r) for r in (1, 2, 3, 4)],
    pins16.test_fp16_hand_examples,
]
STATS_PINS = [
    pins_stats.test_closed_forms,
    pins_stats.test_matches_numpy_and_torch_float64_norms,
    pins_stats.test_squares_are_taken_in_double,
    pins_stats.test_nan_and_inf,
    pins_stats.test_group_norms,
]
RULE_PINS = [
    pins_stats.test_constant_norm_upgrades_every_interval_until_32_bits,
    pins_stats.test_paper_thresholds_never_fire_on_growing_norms,
    pins_stats.test_counter_is_cumulative_not_consecutive,
    pins_stats.test_signed_comparison_and_strictness,
    pins_stats.test_bits_to_bytes_rounds_up,
    pins_stats.test_non_byte_step_and_layers_independent,
    pins_stats.test_zero_previous_norm,
]

# (name, text to find, replacement, pins that must notice)
MUTANTS = [
    ("pack keeps the LOW bytes", "(word >> (8 * (dropped + k)))", "(word >> (8 * k))", PACK_PINS),
    ("pack stores bytes most significant first",
     "Pw[POffset + k] = (uint8_t)((word >> (8 * (dropped + k))) & 0xFFu);",
     "Pw[POffset + RoundTo - 1 - k] = (uint8_t)((word >> (8 * (dropped + k))) & 0xFFu);", PACK_PINS),
    ("pack forgets to advance the offset per weight", "            POffset += RoundTo;\n        }\n    }\n    return POffset;\n}\n\n/*\n * Bitunpack",
     "        }\n        POffset += RoundTo;\n    }\n    return POffset;\n}\n\n/*\n * Bitunpack", PACK_PINS),
    ("unpack shifts one byte too few", "q << ((4 - RoundTo) * 8)", "q << ((3 - RoundTo) * 8 + (RoundTo == 4 ? 8 : 0))", PACK_PINS),
    ("unpack assembles bytes in reverse", "q |= (uint32_t)Pw[POffset + k] << (8 * k);",
     "q |= (uint32_t)Pw[POffset + k] << (8 * (RoundTo - 1 - k));", PACK_PINS),
    ("unpack fills the low bits with ones", "uint32_t word = q << ((4 - RoundTo) * 8);",
     "uint32_t word = (q << ((4 - RoundTo) * 8)) | ((RoundTo < 4) ? ((1u << ((4 - RoundTo) * 8)) - 1u) : 0u);", PACK_PINS),
    ("pack rounds to nearest instead of truncating", "memcpy(&word, &W[i], 4);            /* the weight as a 32-bit word */",
     "memcpy(&word, &W[i], 4); if (RoundTo < 4 && (word & 0x7F800000u) != 0x7F800000u) word += 1u << ((4 - RoundTo) * 8 - 1);", PACK_PINS),
    ("squares summed in float", "double w = (double)W[i];\n            sumsq += w * w;\n            if (isnan(w))",
     "double w = (double)W[i];\n            sumsq += (double)(W[i] * W[i]);\n            if (isnan(w))", STATS_PINS),
    ("sum of absolute values instead of squares", "sumsq += w * w;\n            if (isnan(w))", "sumsq += fabs(w);\n            if (isnan(w))", STATS_PINS),
    ("norm without the square root", "stats[layer * ORACLE_NSTATS + 1] = sqrt(sumsq);", "stats[layer * ORACLE_NSTATS + 1] = sumsq;", STATS_PINS),
    ("largest value instead of largest magnitude", "else if (fabs(w) > absmax) absmax = fabs(w);", "else if (w > absmax) absmax = w;", STATS_PINS),
    ("last weight of a layer skipped", "for (int64_t i = layer_offsets[layer]; i < layer_offsets[layer + 1]; ++i) {\n            double w",
     "for (int64_t i = layer_offsets[layer]; i + 1 < layer_offsets[layer + 1]; ++i) {\n            double w", STATS_PINS),
    ("group norm sums the norms instead of the squares", "            sumsq += w * w;\n        }\n        l2_group[g] = sqrt(sumsq);",
     "            sumsq += w * w;\n        }\n        l2_group[g] = (group_offsets[g + 1] - group_offsets[g] > 1) ? sumsq : sqrt(sumsq);", STATS_PINS),
    ("rule compares with <= ", "if (delta < T)", "if (delta <= T)", RULE_PINS),
    ("rule uses |delta|", "if (delta < T)", "if (fabs(delta) < fabs(T))", RULE_PINS),
    ("counter resets on a batch that does not count", "if (delta < T)\n                counter[layer] += 1;",
     "if (delta < T)\n                counter[layer] += 1;\n            else\n                counter[layer] = 0;", RULE_PINS),
    ("relative change divided by the new norm", "/ l2_prev[layer];", "/ l2_now[layer];", RULE_PINS),
    ("bits not capped", "if (bits[layer] > 32) bits[layer] = 32;", "", RULE_PINS),
    ("counter not cleared after an upgrade", "                counter[layer] = 0;\n", "", RULE_PINS),
    ("bytes rounded down", "(uint8_t)((bits[layer] + 7) / 8)", "(uint8_t)(bits[layer] / 8 ? bits[layer] / 8 : 1)", RULE_PINS),
    ("first batch already counts", "if (!is_first_batch) {", "if (1) {", RULE_PINS),
    ("previous norm never updated", "l2_prev[layer] = l2_now[layer];", "if (is_first_batch) l2_prev[layer] = l2_now[layer];", RULE_PINS),
]


@pytest.mark.parametrize("name,find,replace,pins", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_is_caught(tmp_path, name, find, replace, pins):
    text = open(SRC).read()
    assert text.count(find) >= 1, "mutation site not found: the oracle's source changed"
    mutated = text.replace(find, replace, 1)
    c = tmp_path / "mutant.c"
    so = tmp_path / "mutant.so"
    c.write_text(mutated)
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-shared", "-fPIC", "-w", "-o", str(so), str(c), "-lm"])
    real = oracle._load()
    try:
        oracle._lib = oracle._load(str(so))
        caught = []
        for pin in pins:
            try:
                pin()
            except AssertionError:
                caught.append(pin)
            except Exception:          # a crash of the checker also counts as noticed
                caught.append(pin)
        assert caught, f"no pin noticed: {name}"
    finally:
        oracle._lib = real


def test_the_unmutated_oracle_passes_every_pin_used_above():
    for pin in PACK_PINS + STATS_PINS + RULE_PINS:
        pin()
