"""Do the pins of the oracle notice a mistake in it?  Each entry below plants one plausible mistake in a
copy of oracle/mxfp4_ref.c (a wrong bias, sign, index, nibble order, tie rule, clamp, a dropped rounding
...), builds the copy with gcc, puts it in the oracle's place for the duration of the check and runs the
pins named with it: at least one of them has to fail.  Everything happens on the CPU, in a temporary
directory; the oracle itself is restored afterwards and is never modified.  The pins are this suite's own
tests, so on the oracle as it is they pass in the same run.

Two mistakes that no pin can notice, because they change nothing, are left out on purpose: the scale of
the re-quantizing FP8-column form compared with >= instead of > (a group maximum is 1.0 or 1.5 times a
power of two, 448 is 1.75 times one: they never meet), and an upper clamp of the scale byte at 255 for
FP32 inputs (6 * 2^127 is not an FP32 number; the clamp is pinned on doubles instead)."""
import ctypes
import importlib
import os
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

import pytest

from oracle import build as oracle_build
from oracle import ref

# (what is planted, text in oracle/mxfp4_ref.c, replacement, which occurrence, pins "module:test" that notice it)
MISTAKES = [
    ('E4M3 exponent bias off by one',
     'return ldexp(1.0 + (double)m / 8.0, (int)e - 7);',
     'return ldexp(1.0 + (double)m / 8.0, (int)e - 6);', 0,
     ['test_oracle_formats:test_e4m3_decode_matches_torch_cast', 'test_oracle_formats:test_e4m3_round_matches_torch_cast']),
    ('E4M3 subnormals one binade too high',
     'return ldexp((double)m, -9);',
     'return ldexp((double)m, -8);', 0,
     ['test_oracle_formats:test_e4m3_decode_matches_torch_cast', 'test_oracle_formats:test_e4m3_round_matches_torch_cast']),
    ('E2M1 subnormal 0.5 read as 0.25',
     'return 0.5 * (double)m;',
     'return 0.25 * (double)m;', 0,
     ['test_oracle_formats:test_e2m1_decode_is_the_format_table', 'test_oracle_formats:test_e2m1_round_matches_paper_lgs_rule_and_brute_force']),
    ('E2M1 rounding: ties to the odd code',
     '(err == best_err && (c & 1u) == 0u)',
     '(err == best_err && (c & 1u) == 1u)', 0,
     ['test_oracle_formats:test_e2m1_round_matches_paper_lgs_rule_and_brute_force', 'test_oracle_quant:test_all_codes_times_scale_sweep_against_exact_brute_force']),
    ('E4M3 rounding: ties to the odd code',
     '(err == best_err && (c & 1u) == 0u)',
     '(err == best_err && (c & 1u) == 1u)', 1,
     ['test_oracle_formats:test_e4m3_round_matches_torch_cast', 'test_oracle_row_to_fp8_col:test_hand_worked_column']),
    ('E2M1 rounding: no saturation test',
     'if (!(y <= FP4_MAX))\n        return 7u;',
     'if (y != y)\n        return 7u;', 0,
     ['test_oracle_formats:test_e2m1_round_matches_paper_lgs_rule_and_brute_force', 'test_oracle_quant:test_all_codes_times_scale_sweep_against_exact_brute_force']),
    ('scale rule: strict comparison at 6 * 2^k',
     'int k = (f <= 0.75) ? e - 3 : e - 2;',
     'int k = (f < 0.75) ? e - 3 : e - 2;', 0,
     ['test_oracle_formats:test_scale_byte_is_smallest_power_of_two_covering_gmax_over_6', 'test_oracle_quant:test_all_codes_times_scale_sweep_against_exact_brute_force']),
    ('scale rule: floor(log2 max) - 2 of the OCP specification',
     'int k = (f <= 0.75) ? e - 3 : e - 2;',
     'int k = e - 3;', 0,
     ['test_oracle_formats:test_scale_byte_is_smallest_power_of_two_covering_gmax_over_6', 'test_oracle_quant:test_all_codes_times_scale_sweep_against_exact_brute_force']),
    ('scale rule: maximum 4 instead of 6',
     'int k = (f <= 0.75) ? e - 3 : e - 2;',
     'int k = (f <= 0.5) ? e - 3 : e - 2;', 0,
     ['test_oracle_formats:test_scale_byte_is_smallest_power_of_two_covering_gmax_over_6', 'test_oracle_quant:test_all_codes_times_scale_sweep_against_exact_brute_force']),
    ('scale byte not clamped at 0',
     'if (b < 0)\n        b = 0;',
     'if (b < -300)\n        b = 0;', 0,
     ['test_oracle_formats:test_scale_byte_is_smallest_power_of_two_covering_gmax_over_6', 'test_oracle_quant:test_all_codes_times_scale_sweep_against_exact_brute_force']),
    ('scale byte clamped at 255',
     'if (b > 254)\n        b = 254;',
     'if (b > 255)\n        b = 255;', 0,
     ['test_oracle_formats:test_scale_byte_is_smallest_power_of_two_covering_gmax_over_6']),
    ('sign of a zero dropped',
     'unsigned sign = signbit(v[i]) ? 1u : 0u;',
     'unsigned sign = v[i] < 0.0 ? 1u : 0u;', 0,
     ['test_oracle_quant:test_all_codes_times_scale_sweep_against_exact_brute_force', 'test_oracle_quant:test_hand_worked_blocks']),
    ('block maximum over the signed values',
     'if (fabs(v[i]) > gmax)\n            gmax = fabs(v[i]);',
     'if (v[i] > gmax)\n            gmax = v[i];', 0,
     ['test_oracle_quant:test_all_codes_times_scale_sweep_against_exact_brute_force', 'test_oracle_quant:test_invariants_zero_sign_nan_saturation']),
    ('quant: exact product, no FP32 rounding',
     'float p = (float)(a * s);',
     'double p = a * s;', 0,
     ['test_oracle_quant:test_all_codes_times_scale_sweep_against_exact_brute_force', 'test_oracle_quant:test_hand_worked_blocks']),
    ('quant: tile scale of the neighbouring tile',
     'x_scale[r * (K / 128) + j / 4]',
     'x_scale[r * (K / 128) + (j / 4 ^ 1) % (K / 128)]', 0,
     ['test_oracle_quant:test_invariants_zero_sign_nan_saturation', 'test_oracle_dequant:test_round_trips']),
    ('quant: high nibble holds the even element',
     '(uint8_t)(code[2 * e] | (code[2 * e + 1] << 4))',
     '(uint8_t)(code[2 * e + 1] | (code[2 * e] << 4))', 0,
     ['test_oracle_quant:test_all_codes_times_scale_sweep_against_exact_brute_force', 'test_oracle_quant:test_hand_worked_blocks']),
    ('quant from BF16: high nibble holds the even element',
     '(uint8_t)(code[2 * e] | (code[2 * e + 1] << 4))',
     '(uint8_t)(code[2 * e + 1] | (code[2 * e] << 4))', 1,
     ['test_oracle_quant_bf16:test_agrees_with_the_fp8_path_where_both_are_exact', 'test_oracle_quant_bf16:test_invariants']),
    ('quant: NaN block keeps a finite scale',
     'code[i] = 0;\n        return 0xFFu;',
     'code[i] = 0;\n        return 0x7Fu;', 0,
     ['test_oracle_quant:test_all_codes_times_scale_sweep_against_exact_brute_force', 'test_oracle_quant:test_invariants_zero_sign_nan_saturation']),
    ('BF16 subnormals one binade too low',
     'a = ldexp((double)m, -133);',
     'a = ldexp((double)m, -134);', 0,
     ['test_oracle_quant_bf16:test_random_and_edge_blocks_against_exact_brute_force']),
    ('BF16 exponent bias off by one',
     'a = ldexp(1.0 + (double)m / 128.0, (int)e - 127);',
     'a = ldexp(1.0 + (double)m / 128.0, (int)e - 126);', 0,
     ['test_oracle_quant_bf16:test_agrees_with_the_fp8_path_where_both_are_exact', 'test_oracle_quant_bf16:test_random_and_edge_blocks_against_exact_brute_force']),
    ('dequant: tile scale with delta 5',
     'int b8 = bmax - 6;',
     'int b8 = bmax - 5;', 0,
     ['test_oracle_formats:test_ue8m0_decode_against_torch', 'test_oracle_dequant:test_every_code_and_shift_against_algorithm_1_where_it_applies']),
    ('dequant: elements aligned with delta 5',
     'double r = ldexp(e2m1_magnitude(nib & 7u), 6 - d);',
     'double r = ldexp(e2m1_magnitude(nib & 7u), 5 - d);', 0,
     ['test_oracle_dequant:test_every_code_and_shift_against_algorithm_1_where_it_applies', 'test_oracle_dequant:test_hand_worked_tile_of_algorithm_1']),
    ('dequant: shift by b_i - min instead of max - b_i',
     'else if (b[j] > bmax)\n                    bmax = b[j];',
     'else if (j == 0 || b[j] < bmax)\n                    bmax = b[j];', 0,
     ['test_oracle_formats:test_ue8m0_decode_against_torch', 'test_oracle_dequant:test_every_code_and_shift_against_algorithm_1_where_it_applies']),
    ('dequant: odd element from the low nibble',
     'unsigned nib = (k & 1) ? (byte >> 4) : (byte & 0xFu);',
     'unsigned nib = (k & 1) ? (byte & 0xFu) : (byte >> 4);', 0,
     ['test_oracle_dequant:test_every_code_and_shift_against_algorithm_1_where_it_applies', 'test_oracle_dequant:test_hand_worked_tile_of_algorithm_1']),
    ('dequant: sign bit dropped',
     'out = (uint8_t)(((nib >> 3) << 7) | e4m3_round_nearest_even(r, grid));\n                    }\n                    x[i * K + k] = out;',
     'out = (uint8_t)(e4m3_round_nearest_even(r, grid));\n                    }\n                    x[i * K + k] = out;', 0,
     ['test_oracle_dequant:test_every_code_and_shift_against_algorithm_1_where_it_applies', 'test_oracle_dequant:test_hand_worked_tile_of_algorithm_1']),
    ('dequant: NaN byte takes part in the maximum',
     'if (b[j] == 0xFFu)\n                    any_nan = 1;\n                else if (b[j] > bmax)',
     'if (b[j] == 0xFFu)\n                    any_nan = 1;\n                if (b[j] > bmax)', 0,
     ['test_oracle_dequant:test_nan_scale_byte']),
    ('row->col: scale of the neighbouring k-block',
     'unsigned b = sf_row[m * (K / 32) + k / 32];\n                if (b == 0xFFu) {\n                    has_nan = 1;',
     'unsigned b = sf_row[m * (K / 32) + (k / 32 ^ 1)];\n                if (b == 0xFFu) {\n                    has_nan = 1;', 0,
     ['test_oracle_row_to_col:test_equals_integer_re_derivation', 'test_oracle_row_to_col:test_exact_rational_brute_force_on_tiles']),
    ('row->col: odd column from the low nibble',
     'unsigned nib = (k & 1) ? (byte >> 4) : (byte & 0xFu);',
     'unsigned nib = (k & 1) ? (byte & 0xFu) : (byte >> 4);', 1,
     ['test_oracle_row_to_col:test_equals_integer_re_derivation', 'test_oracle_row_to_col:test_exact_rational_brute_force_on_tiles']),
    ('row->col: row scale applied with the wrong sign',
     'double a = ldexp(e2m1_magnitude(nib & 7u), (int)b - 127);\n                v[e] = (nib & 8u) ? -a : a;',
     'double a = ldexp(e2m1_magnitude(nib & 7u), 127 - (int)b);\n                v[e] = (nib & 8u) ? -a : a;', 0,
     ['test_oracle_row_to_col:test_equals_integer_re_derivation', 'test_oracle_row_to_col:test_exact_rational_brute_force_on_tiles']),
    ('row->col: column scales stored untransposed',
     'sf_col[k * B + mb] = (uint8_t)bc;',
     'sf_col[mb * K + k] = (uint8_t)bc;', 0,
     ['test_oracle_row_to_col:test_equals_integer_re_derivation', 'test_oracle_row_to_col:test_exact_rational_brute_force_on_tiles']),
    ('row->col: odd m in the low nibble',
     'q_col[k * P + mb * 16 + e] = (uint8_t)(code[2 * e] | (hi << 4));',
     'q_col[k * P + mb * 16 + e] = (uint8_t)(hi | (code[2 * e] << 4));', 0,
     ['test_oracle_row_to_col:test_equals_integer_re_derivation', 'test_oracle_row_to_col:test_exact_rational_brute_force_on_tiles']),
    ('row->col: NaN row scale ignored',
     'if (b == 0xFFu) {\n                    has_nan = 1;\n                    continue;\n                }\n                double a',
     'if (b == 0xFFu) {\n                    continue;\n                }\n                double a', 0,
     ['test_oracle_row_to_col:test_nan_row_scale_poisons_the_column_blocks_it_touches', 'test_oracle_row_to_col:test_ragged_splits_without_padding']),
    ('FP8 column: scale without delta',
     '(float)ldexp(1.0, bmax - 6 - 127)',
     '(float)ldexp(1.0, bmax - 127)', 0,
     ['test_oracle_row_to_fp8_col:test_exact_rational_brute_force_and_library_cast', 'test_oracle_row_to_fp8_col:test_hand_worked_column']),
    ("FP8 column: maximum over the k-block's neighbour",
     'unsigned b = sf_row[(g * 128 + e) * (K / 32) + k / 32];\n                if (b == 0xFFu)\n                    any_nan = 1;',
     'unsigned b = sf_row[(g * 128 + e) * (K / 32) + (k / 32 ^ 1)];\n                if (b == 0xFFu)\n                    any_nan = 1;', 0,
     ['test_oracle_row_to_fp8_col:test_hand_worked_column', 'test_oracle_row_to_fp8_col:test_nan_scale_byte_and_edges']),
    ('FP8 column: neighbouring rows swapped',
     'x_col[k * M + m] = out;',
     'x_col[k * M + (m ^ 1) % M] = out;', 0,
     ['test_oracle_row_to_fp8_col:test_exact_rational_brute_force_and_library_cast', 'test_oracle_row_to_fp8_col:test_hand_worked_column']),
    ('FP8 column: elements aligned with delta 7',
     'double r = ldexp(e2m1_magnitude(nib & 7u), 6 - (bmax - (int)b));',
     'double r = ldexp(e2m1_magnitude(nib & 7u), 7 - (bmax - (int)b));', 0,
     ['test_oracle_row_to_fp8_col:test_exact_rational_brute_force_and_library_cast', 'test_oracle_row_to_fp8_col:test_hand_worked_column']),
    ('FP8 column requant: 256 as the E4M3 maximum',
     'while (amax > ldexp(448.0, j))',
     'while (amax > ldexp(256.0, j))', 0,
     ['test_oracle_row_to_fp8_col_requant:test_exact_rational_brute_force_library_cast_and_integer_form', 'test_oracle_row_to_fp8_col_requant:test_hand_worked_column']),
    ('FP8 column requant: scale of an all-zero group',
     'int j = 0; /* S = 2^j */',
     'int j = -127; /* S = 2^j */', 0,
     ['test_oracle_row_to_fp8_col_requant:test_nan_scale_byte_and_edges']),
    ('FP8 column requant: NaN rows take part in the maximum',
     'if (b == 0xFFu) {\n            any_nan = 1;\n            continue;\n        }\n        double a = ldexp',
     'if (b == 0xFFu) {\n            any_nan = 1;\n        }\n        double a = ldexp', 0,
     ['test_oracle_row_to_fp8_col_requant:test_nan_scale_byte_and_edges']),
    ('grouped row->col: expert outputs at K * off / 2',
     'bytes_before += (T + 1) / 2;',
     'bytes_before += T / 2;', 0,
     ['test_oracle_row_to_col:test_ragged_splits_without_padding']),
    ('grouped row->col: scale blocks rounded down',
     'blocks_before += (T + 31) / 32;',
     'blocks_before += T / 32;', 0,
     ['test_oracle_row_to_col:test_ragged_splits_without_padding']),
    ('grouped FP8 column: scale groups rounded down',
     'groups_before += (T + 127) / 128;',
     'groups_before += T / 128;', 0,
     ['test_oracle_row_to_fp8_col:test_ragged_splits_without_padding', 'test_oracle_row_to_fp8_col_requant:test_ragged_groups_equal_zero_padded_flat']),
    ('scatter: only the first destination written',
     'for (int32_t j = 0; j < fanout; ++j) {\n            int64_t d = dst_idx',
     'for (int32_t j = 0; j < 1; ++j) {\n            int64_t d = dst_idx', 0,
     ['test_oracle_quant:test_scatter_is_the_gather_turned_around']),
    ('gather: index ignored',
     'int64_t r = gather_idx ? (int64_t)gather_idx[i] : i;',
     'int64_t r = gather_idx ? i % M_src : i;', 0,
     ['test_oracle_quant:test_gather_and_strides', 'test_oracle_quant:test_scatter_is_the_gather_turned_around']),
    ('a NaN product (NaN scale, infinity times zero) counted as zero instead of poisoning its block',
     'if (isnan(p)) { /* NaN scale, or 0 * inf */\n                    has_nan = 1;',
     'if (isnan(p)) { /* NaN scale, or 0 * inf */\n                    has_nan = 0;', 0,
     ['test_oracle_quant:test_scales_outside_the_format_follow_ieee_products']),
]


def planted(source, old, new, occurrence):
    at = -1
    for _ in range(occurrence + 1):
        at = source.index(old, at + 1)
    return source[:at] + new + source[at + len(old):]


def test_every_planted_mistake_fails_a_pin():
    source = open(oracle_build.SRC).read()
    original_path, original_lib = oracle_build.LIB, ref.lib()
    with tempfile.TemporaryDirectory() as tmp:
        def compile_one(i):
            _, old, new, occurrence, _ = MISTAKES[i]
            c, so = os.path.join(tmp, f"m{i}.c"), os.path.join(tmp, f"m{i}.so")
            with open(c, "w") as f:
                f.write(planted(source, old, new, occurrence))
            subprocess.run(["gcc", "-std=c11", "-O2", "-fno-fast-math", "-ffp-contract=off", "-shared", "-fPIC",
                            c, "-o", so, "-lm"], check=True)
            return so
        with ThreadPoolExecutor(8) as pool:
            libs = list(pool.map(compile_one, range(len(MISTAKES))))
        unnoticed = []
        try:
            for (what, _, _, _, pins), so in zip(MISTAKES, libs):
                ref._LIB, oracle_build.LIB = None, so        # the oracle's front end now loads the copy
                ref.lib()
                noticed = False
                for pin in pins:
                    module, name = pin.split(":")
                    try:
                        getattr(importlib.import_module("tests." + module), name)()
                    except AssertionError:
                        noticed = True
                        break
                if not noticed:
                    unnoticed.append(what)
        finally:
            ref._LIB, oracle_build.LIB = original_lib, original_path
    assert ref.lib() is original_lib
    assert not unnoticed, unnoticed

