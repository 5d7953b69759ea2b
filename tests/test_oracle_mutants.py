"""Are the oracle's pins sharp?  Plant one mistake at a time in a COPY of the
oracle source (CPU only), rebuild it, and require that the pin suite of
test_oracle.py fails for every planted mistake."""
import os
import types

import pytest

from oracle import build as oracle_build
from oracle import zvc_ref
from tests import test_oracle as pins
from tests import test_oracle_relu as relu_pins
from tests import test_oracle_window as window_pins
from tests.golden_cases import load_handbuilt, load_relu_cases, load_window_cases

MUTANTS = [
    ("msb_first_bit_order", "m |= (uint32_t{1} << b);", "m |= (uint32_t{1} << (31 - b));"),
    ("mask_bit_for_zero", "if (element_bits(in, i, w) != 0) {\n                m |=",
     "if (element_bits(in, i, w) == 0) {\n                m |="),
    ("keeps_zeros_too", "++kept;\n            }\n        }\n        masks[g] = m;",
     "}\n            ++kept;\n        }\n        masks[g] = m;"),
    ("tail_not_clipped", "if (i >= n) break;", "if (i > n) break;"),
    ("float_style_zero_test_drops_sign", "word = v;\n    } else {\n        uint16_t v;",
     "word = v & 0x7FFFFFFFu;\n    } else {\n        uint16_t v;"),
    ("halfword_reads_low_byte_only", "std::memcpy(&v, in + i * 2, 2);", "std::memcpy(&v, in + i * 2, 1);"),
    ("values_before_masks", "out + 4 * groups);\n    for (uint64_t g = 0; g < groups; ++g) {\n        // little",
     "out);\n    for (uint64_t g = 0; g < groups; ++g) {\n        // little"),
    ("big_endian_masks", "out[4 * g + 0] = static_cast<unsigned char>(m & 0xFF);",
     "out[4 * g + 0] = static_cast<unsigned char>((m >> 24) & 0xFF);"),
    ("size_counts_bits_not_bytes", "return 4 * zvc_ref_groups(n) + static_cast<uint64_t>(w) * nnz;",
     "return zvc_ref_groups(n) + static_cast<uint64_t>(w) * nnz;"),
    ("groups_floor_instead_of_ceil", "return n / 32 + (n % 32 != 0 ? 1 : 0);", "return n / 32 + (n % 32 != 0 ? 1 : 0) - (n % 32 == 31 ? 1 : 0);"),
    ("decoder_reads_wrong_bit", "if ((m >> (i % 32)) & 1u) {\n            std::memcpy(out + i * w",
     "if ((m >> ((i + 1) % 32)) & 1u) {\n            std::memcpy(out + i * w"),
    ("decoder_does_not_advance", "std::memcpy(out + i * w, values + used * w, static_cast<size_t>(w));\n            ++used;",
     "std::memcpy(out + i * w, values + used * w, static_cast<size_t>(w));\n            used += (i % 64 == 63) ? 0 : 1;"),
    ("decoder_skips_zero_fill", "std::memset(out + i * w, 0, static_cast<size_t>(w));", "(void)0;"),
    ("count_ignores_high_half", "kept += (element_bits(in, i, w) != 0) ? 1 : 0;",
     "kept += ((element_bits(in, i, w) & 0xFFFFu) != 0) ? 1 : 0;"),
    ("relu_ignores_sign", "const bool positive = (word & sign) == 0 && word != 0;",
     "const bool positive = word != 0;"),
    ("relu_keeps_negatives_instead", "const bool positive = (word & sign) == 0 && word != 0;",
     "const bool positive = (word & sign) != 0;"),
    ("relu_halfword_sign_in_wrong_bit", "const uint32_t sign = w == 4 ? 0x80000000u : 0x8000u;",
     "const uint32_t sign = w == 4 ? 0x80000000u : 0x4000u;"),
    ("relu_leaves_dropped_elements_in_place", "std::memset(out + i * w, 0, static_cast<size_t>(w));\n    }\n    return 0;",
     "(void)0;\n    }\n    return 0;"),
    ("window_values_before_their_mask", "            pos += 4;\n            // ... then its non-zero elements, in order",
     "            // ... then its non-zero elements, in order"),
    ("window_encoder_drops_ragged_last_group", "        offsets[k] = pos;\n        const uint64_t first = k * window_elems;\n        const uint64_t last = first + window_elems < n ? first + window_elems : n;\n        for (uint64_t g0 = first; g0 < last; g0 += 32) {",
     "        offsets[k] = pos;\n        const uint64_t first = k * window_elems;\n        const uint64_t last = first + window_elems < n ? first + window_elems : n;\n        for (uint64_t g0 = first; g0 + 32 <= last; g0 += 32) {"),
    ("window_offsets_one_late", "        offsets[k] = pos;\n        const uint64_t first = k * window_elems;\n        const uint64_t last = first + window_elems < n ? first + window_elems : n;\n        for (uint64_t g0 = first; g0 < last; g0 += 32) {\n            // the group's mask first ...",
     "        offsets[k] = pos + 4;\n        const uint64_t first = k * window_elems;\n        const uint64_t last = first + window_elems < n ? first + window_elems : n;\n        for (uint64_t g0 = first; g0 < last; g0 += 32) {\n            // the group's mask first ..."),
    ("window_decoder_starts_at_stream_start", "        uint64_t pos = offsets[k];\n        const uint64_t first = k * window_elems;\n        const uint64_t last = first + window_elems < n ? first + window_elems : n;\n        for (uint64_t g0 = first; g0 < last; g0 += 32) {\n            const uint32_t m =",
     "        uint64_t pos = offsets[first_window];\n        const uint64_t first = k * window_elems;\n        const uint64_t last = first + window_elems < n ? first + window_elems : n;\n        for (uint64_t g0 = first; g0 < last; g0 += 32) {\n            const uint32_t m ="),
    ("window_big_endian_mask", "            out[pos + 0] = static_cast<unsigned char>(m & 0xFF);\n            out[pos + 1] = static_cast<unsigned char>((m >> 8) & 0xFF);",
     "            out[pos + 1] = static_cast<unsigned char>(m & 0xFF);\n            out[pos + 0] = static_cast<unsigned char>((m >> 8) & 0xFF);"),
    ("fused_skips_relu", "return zvc_ref_compress_stream(activated.data(), n, w, out);",
     "return zvc_ref_compress_stream(in, n, w, out);"),
]


def _pin_suite(oracle):
    for case in load_handbuilt():
        pins.test_handbuilt_cases(oracle, case)
    pins.test_paper_all_zero_group_is_32x(oracle)
    pins.test_paper_dense_group_overhead(oracle)
    pins.test_paper_headline_ratios_follow_the_size_formula(oracle)
    pins.test_paper_60_percent_zero_example(oracle)
    for w in (2, 4):
        for n in (0, 31, 33, 95, 4097):
            pins.test_matches_library_routines(oracle, n, w)
        pins.test_extremes(oracle, w)
        pins.test_ratio_closed_form_on_bernoulli(oracle, w)
    pins.test_single_nonzero_every_position_bruteforce(oracle)
    pins.test_decoder_places_values_by_mask_bruteforce(oracle)
    pins.test_special_float_patterns_are_kept(oracle)
    pins.test_layout_independence(oracle)
    pins.test_random_byte_soup_round_trip(oracle)
    pins.test_values_preserve_order(oracle)
    for case in load_window_cases():
        window_pins.test_window_handbuilt_cases(oracle, case)
    for w in (2, 4):
        for n in (33, 1025, 4097):
            window_pins.test_window_stream_holds_the_planar_masks_and_values(oracle, n, w)
        window_pins.test_any_window_range_decodes_on_its_own(oracle, w)
    for case in load_relu_cases():
        relu_pins.test_relu_handbuilt_cases(oracle, case)
    relu_pins.test_relu_matches_numpy_maximum_fp32(oracle)
    relu_pins.test_relu_rule_on_every_16bit_pattern(oracle)
    for w in (2, 4):
        for n in (33, 4097):
            relu_pins.test_fused_is_zvc_of_relu(oracle, n, w)


def _bound(lib):
    ns = types.SimpleNamespace()
    for name in ("groups", "compressed_bytes", "compress", "compress_stream", "decompress",
                 "decompress_stream", "count_nonzero", "relu", "relu_compress_stream", "window_count", "window_compress",
                 "window_decompress"):
        fn = getattr(zvc_ref, name)
        setattr(ns, name, (lambda f: lambda *a: f(*a, lib=lib))(fn))
    return ns


def test_unmodified_copy_passes(tmp_path):
    out = oracle_build.build(output=str(tmp_path / "libclean.so"))
    _pin_suite(_bound(zvc_ref.load(out)))


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, old, new):
    src = open(oracle_build.SOURCE).read()
    assert src.count(old) >= 1, "mutation target vanished from the oracle source: " + name
    mutated = tmp_path / (name + ".cpp")
    mutated.write_text(src.replace(old, new, 1))
    lib_path = oracle_build.build(output=str(tmp_path / (name + ".so")), source=str(mutated))
    mutant = _bound(zvc_ref.load(lib_path))
    with pytest.raises((AssertionError, ValueError)):
        _pin_suite(mutant)
