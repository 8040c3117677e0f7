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
    ("pack keeps the LOW bytes", "slot[b] = byte_of(word, dropped + b);", "slot[b] = byte_of(word, b);", PACK_PINS),
    ("pack stores bytes most significant first", "slot[b] = byte_of(word, dropped + b);",
     "slot[keep - 1 - b] = byte_of(word, dropped + b);", PACK_PINS),
    ("pack places every weight of a layer at the layer's start",
     "uint8_t *slot = stream + layer_start + i * keep;\n            for (int b = 0; b < keep; ++b)\n                slot[b] = byte_of",
     "uint8_t *slot = stream + layer_start;\n            for (int b = 0; b < keep; ++b)\n                slot[b] = byte_of", PACK_PINS),
    ("pack starts every layer where the previous one started", "layer_start += count * keep;\n    }\n    return layer_start;\n}\n\n/*\n * Bitunpack",
     "layer_start += (layer + 1 < n_layers) ? 0 : count * keep;\n    }\n    return layer_start;\n}\n\n/*\n * Bitunpack", PACK_PINS),
    ("unpack shifts one byte too few", "stored << ((4 - keep) * 8)", "stored << ((3 - keep) * 8 + (keep == 4 ? 8 : 0))", PACK_PINS),
    ("unpack assembles bytes in reverse", "stored |= (uint32_t)slot[b] << (8 * b);",
     "stored |= (uint32_t)slot[b] << (8 * (keep - 1 - b));", PACK_PINS),
    ("unpack fills the low bits with ones", "weight_of(stored << ((4 - keep) * 8));",
     "weight_of((stored << ((4 - keep) * 8)) | ((keep < 4) ? ((1u << ((4 - keep) * 8)) - 1u) : 0u));", PACK_PINS),
    ("pack rounds to nearest instead of truncating", "const uint32_t word = word_of(layer_weights[i]);",
     "uint32_t word = word_of(layer_weights[i]); if (keep < 4 && (word & 0x7F800000u) != 0x7F800000u) word += 1u << ((4 - keep) * 8 - 1);", PACK_PINS),
    ("squares summed in float", "const double w = (double)weights[i];\n        total += w * w;",
     "const double w = (double)weights[i];\n        total += (double)(weights[i] * weights[i]);", STATS_PINS),
    ("sum of absolute values instead of squares", "total += w * w;", "total += fabs(w);", STATS_PINS),
    ("norm without the square root", "row[1] = sqrt(squares);", "row[1] = squares;", STATS_PINS),
    ("largest value instead of largest magnitude", "const double magnitude = fabs((double)weights[i]);",
     "const double magnitude = (double)weights[i];", STATS_PINS),
    ("last weight of a range skipped", "for (int64_t i = first; i < last; ++i) {\n        const double w",
     "for (int64_t i = first; i + 1 < last; ++i) {\n        const double w", STATS_PINS),
    ("group norm without the square root for groups of several layers", "l2_group[g] = sqrt(sum_of_squares(weights, first, last));",
     "l2_group[g] = (group_offsets[g + 1] - group_offsets[g] > 1) ? sum_of_squares(weights, first, last) : sqrt(sum_of_squares(weights, first, last));", STATS_PINS),
    ("rule compares with <= ", "if (change < threshold)", "if (change <= threshold)", RULE_PINS),
    ("rule uses the magnitude of the change", "if (change < threshold)", "if (fabs(change) < fabs(threshold))", RULE_PINS),
    ("count resets on a batch that does not count", "if (change < threshold)\n        layer->counted += 1;",
     "if (change < threshold)\n        layer->counted += 1;\n    else\n        layer->counted = 0;", RULE_PINS),
    ("relative change divided by the new norm", "(norm - layer->previous_norm) / layer->previous_norm;",
     "(norm - layer->previous_norm) / norm;", RULE_PINS),
    ("bits not capped", "if (layer->bits > 32) layer->bits = 32;", "", RULE_PINS),
    ("count not cleared after a precision step", "        layer->counted = 0;\n    }\n}", "    }\n}", RULE_PINS),
    ("bytes rounded down", "(uint8_t)((state.bits + 7) / 8)", "(uint8_t)(state.bits / 8 ? state.bits / 8 : 1)", RULE_PINS),
    ("first batch already counts", "if (!is_first_batch)\n            awp_layer_step", "if (1)\n            awp_layer_step", RULE_PINS),
    ("previous norm never updated", "state.previous_norm = l2_now[layer];", "if (is_first_batch) state.previous_norm = l2_now[layer];", RULE_PINS),
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
