"""Do the pins notice a wrong oracle?  Each case plants one plausible mistake in a COPY of
the oracle's C source (text substitution), compiles the copy on the CPU and demands that at
least one pin fails on it.  The committed oracle itself is never modified.
"""
import pathlib
import subprocess

import pytest

import oracle_pins
from oracle.w4a16_oracle import Oracle

SRC = pathlib.Path(__file__).resolve().parent.parent / "oracle" / "w4a16_oracle.c"

# (name, text to find, replacement, which occurrence: index or "all")
MUTATIONS = [
    # the definition (w4a16_oracle_gemm)
    ("qweight_field_order_in_gemm", "const int qd = field_of(qweight, (size_t)(kk / 8) * n + j, kk % 8);",
     "const int qd = field_of(qweight, (size_t)(kk / 8) * n + j, 7 - kk % 8);", 0),
    ("qzeros_field_order_in_gemm", "const int zd = field_of(qzeros, (size_t)grp * (n / 8) + j / 8, j % 8);",
     "const int zd = field_of(qzeros, (size_t)grp * (n / 8) + j / 8, 7 - j % 8);", 0),
    ("qzeros_word_column_in_gemm", "const int zd = field_of(qzeros, (size_t)grp * (n / 8) + j / 8, j % 8);",
     "const int zd = field_of(qzeros, (size_t)grp * (n / 8) + j % (n / 8), j % 8);", 0),
    ("zero_point_plus_one", "const float wd = (float)(qd - zd) * sd;", "const float wd = (float)(qd - zd - 1) * sd;", 0),
    ("sign_flipped", "const float wd = (float)(qd - zd) * sd;", "const float wd = (float)(zd - qd) * sd;", 0),
    ("group_boundary_off_by_one", "const int grp = kk / group_size;",
     "const int grp = (kk == k - 1 ? kk : kk + 1) / group_size;", 0),
    ("A_transposed", "const float ad = w4a16_oracle_half_to_float(A[(size_t)i * k + kk]);",
     "const float ad = w4a16_oracle_half_to_float(A[(size_t)kk * m + i]);", 0),
    ("last_k_term_dropped", "for (int kk = 0; kk < k; ++kk) {\n                    if (partition_of",
     "for (int kk = 0; kk < k - 1; ++kk) {\n                    if (partition_of", 0),
    ("first_k_term_dropped", "for (int kk = 0; kk < k; ++kk) {\n                    if (partition_of",
     "for (int kk = 1; kk < k; ++kk) {\n                    if (partition_of", 0),
    ("last_partial_sum_dropped", "for (int p = 0; p < split_k; ++p) {\n                double part64",
     "for (int p = 0; p < split_k - (split_k > 1); ++p) {\n                double part64", 0),
    ("partial_sums_not_added_f32", "total32 += part32;", "total32 = part32;", 0),
    ("partial_sums_not_added_f64", "total64 += part64;", "total64 = part64;", 0),
    ("strided_partition_ignores_block", "return (kk / block_k) % split_k;", "return kk % split_k < 0 ? 0 : (kk / (k / split_k)) % split_k;", 0),
    ("scale_column_swapped", "const float sd = w4a16_oracle_half_to_float(scales[(size_t)grp * n + j]);",
     "const float sd = w4a16_oracle_half_to_float(scales[(size_t)grp * n + (j ^ 1)]);", 0),
    ("fp32_mode_accumulates_in_fp64", "const float prod = ad * wd;\n                        part32 += prod;",
     "part64 += (double)ad * (double)wd;\n                        part32 = (float)part64;", 0),
    # the arrangement for the timed baseline (w4a16_oracle_gemm_blocked): held to the definition
    ("blocked_zero_point_plus_one", "wrow[jj] = (float)(q - z) * s;", "wrow[jj] = (float)(q - z - 1) * s;", 0),
    ("blocked_group_boundary_off_by_one", "const int gi = kk / group_size;\n            const int p",
     "const int gi = (kk == k - 1 ? kk : kk + 1) / group_size;\n            const int p", 0),
    ("blocked_last_block_dropped", "const int n_blocks = (n + col_block - 1) / col_block;", "const int n_blocks = n / col_block > 0 ? n / col_block : 1;", 0),
    ("blocked_last_partial_sum_dropped_f64", "for (int p = 0; p < split_k; ++p) t += part64",
     "for (int p = 0; p < split_k - (split_k > 1); ++p) t += part64", 0),
    ("blocked_last_partial_sum_dropped_f32", "for (int p = 0; p < split_k; ++p) t += part32",
     "for (int p = 0; p < split_k - (split_k > 1); ++p) t += part32", 0),
    ("ties_away_from_zero", "(rem == halfway && (q & 1))", "(rem == halfway)", 0),
    ("truncating_conversion", "if (rem > halfway || (rem == halfway && (q & 1))) ++q;", "", 0),
    ("subnormal_exponent", "127 - 15 + 1 - shift", "127 - 15 - shift", 0),
    ("unpack_qweight_field_order", "q[(size_t)kk * n + j] = (uint8_t)((word >> (4 * (kk % 8))) & 0xFu);",
     "q[(size_t)kk * n + j] = (uint8_t)((word >> (4 * (7 - kk % 8))) & 0xFu);", 0),
    ("unpack_qzeros_field_order", "z[(size_t)gi * n + j] = (uint8_t)((word >> (4 * (j % 8))) & 0xFu);",
     "z[(size_t)gi * n + j] = (uint8_t)((word >> (4 * (7 - j % 8))) & 0xFu);", 0),
    ("pack_qweight_field_order", "word |= (uint32_t)(q[(size_t)(8 * r + i) * n + j] & 0xFu) << (4 * i);",
     "word |= (uint32_t)(q[(size_t)(8 * r + i) * n + j] & 0xFu) << (4 * (7 - i));", 0),
    ("bits_field_shift_fixed_at_4", "return (int)(((uint32_t)words[word_index] >> (bits * field)) & mask);",
     "return (int)(((uint32_t)words[word_index] >> (4 * field)) & mask);", 0),
    ("bits_mask_one_bit_short", "const uint32_t mask = (1u << bits) - 1u;\n    return (int)",
     "const uint32_t mask = (1u << (bits - 1)) - 1u;\n    return (int)", 0),
    ("bits_qweight_word_row", "field_of_width(qweight, (size_t)(kk / f) * n + j, kk % f, bits);\n                const int zv",
     "field_of_width(qweight, (size_t)(kk / 8) * n + j, kk % f, bits);\n                const int zv", 0),
    ("bits_qzeros_word_column", "const int zv = field_of_width(qzeros, (size_t)gi * (n / f) + j / f, j % f, bits);",
     "const int zv = field_of_width(qzeros, (size_t)gi * (n / f) + j / f, f - 1 - j % f, bits);", 0),
    ("bits_zero_point_dropped", "const float wv = (float)(qv - zv) * sv;", "const float wv = (float)(qv) * sv;", 0),
    ("bits_group_index", "const int gi = kk / group_size;\n                const int qv",
     "const int gi = 0;\n                const int qv", 0),
    ("bits_unpack_qzeros_row_stride", "z[(size_t)gi * n + j] = (uint8_t)field_of_width(qzeros, (size_t)gi * (n / f) + j / f, j % f, bits);",
     "z[(size_t)gi * n + j] = (uint8_t)field_of_width(qzeros, (size_t)gi * (n / 8) + j / f, j % f, bits);", 0),
    ("bits_pack_field_order", "word |= ((uint32_t)q[(size_t)(f * r + i) * n + j] & mask) << (bits * i);",
     "word |= ((uint32_t)q[(size_t)(f * r + i) * n + j] & mask) << (bits * (f - 1 - i));", 0),
    ("stream3_value_bit_order", "3 * u + t) << t;", "3 * u + t) << (2 - t);", 0),
    ("stream3_word_of_a_bit", "words[first_word + (size_t)(b / 32) * word_stride] >> (b % 32)) & 1u);",
     "words[first_word + (size_t)(b / 33) * word_stride] >> (b % 32)) & 1u);", 0),
    ("stream3_gemm_value_order", "(size_t)n, kk % 32);\n                const int z3", "(size_t)n, 31 - kk % 32);\n                const int z3", 0),
    ("stream3_gemm_zero_column", "(size_t)(j / 32) * 3, 1, j % 32);\n                const float s3",
     "(size_t)(j / 32) * 3, 1, (j + 1) % 32);\n                const float s3", 0),
    ("stream3_zero_point_dropped", "const float w3 = (float)(q3 - z3) * s3;", "const float w3 = (float)(q3) * s3;", 0),
    ("stream3_group_index", "const int group = kk / group_size;", "const int group = kk / 32 % (k / group_size);", 0),
    ("stream3_unpack_qzeros_stream_base", "z[(size_t)gi * n + j] = (uint8_t)stream3_value(qzeros, (size_t)gi * row_words + (size_t)(j / 32) * 3, 1, j % 32);",
     "z[(size_t)gi * n + j] = (uint8_t)stream3_value(qzeros, (size_t)gi * row_words + (size_t)(j / 32) * 3, 1, 31 - j % 32);", 0),
    ("stream3_pack_clears_wrong_bit", "w &= ~(1u << (b % 32));", "w &= ~(1u << (t % 32));", 0),
    ("gidx_ignored", "const int row_group = g_idx[kk];", "const int row_group = kk / (k / groups);", 0),
    ("gidx_scale_from_row_position", "const float sf = w4a16_oracle_half_to_float(scales[(size_t)row_group * n + j]);",
     "const float sf = w4a16_oracle_half_to_float(scales[(size_t)(kk / (k / groups)) * n + j]);", 0),
    ("gidx_zero_from_row_position", "qzeros[(size_t)row_group * (n / 8) + j / 8]", "qzeros[(size_t)(kk / (k / groups)) * (n / 8) + j / 8]", 0),
    ("gidx_zero_point_dropped", "const float wf = (float)(qf - zf) * sf;", "const float wf = (float)(qf) * sf;", 0),
    ("dequant_drops_zero_point", "W[(size_t)kk * n + j] = (float)(q - z) * s;", "W[(size_t)kk * n + j] = (float)(q) * s;", 0),
]


@pytest.mark.parametrize("name,old,new,_which", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_pins_catch_planted_mistake(tmp_path, name, old, new, _which):
    text = SRC.read_text()
    assert text.count(old) >= 1, f"mutation site for {name} no longer exists in the oracle source"
    mutated = text.replace(old, new, 1)
    c = tmp_path / f"{name}.c"
    so = tmp_path / f"lib{name}.so"
    c.write_text(mutated)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                    "-o", str(so), str(c)], check=True)
    bad = Oracle(so)
    failed = []
    for pin in oracle_pins.ALL_PINS:
        try:
            pin(bad)
        except AssertionError:
            failed.append(pin.__name__)
            break
    assert failed, f"no pin noticed the planted mistake '{name}'"
