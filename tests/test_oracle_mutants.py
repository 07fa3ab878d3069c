"""Plausible mistakes planted in a copy of the oracle (on the CPU) must each trip at least one pin."""
import os

import pytest

import oracle
import pins

# (name, text in attn_oracle.c, replacement): each a mistake someone could plausibly make.
MUTANTS = [
    ("mask_off_by_one_tight", "long lim = i + (Skv - Sq);", "long lim = i + (Skv - Sq) - 1;"),
    ("mask_off_by_one_loose", "long lim = i + (Skv - Sq);", "long lim = i + (Skv - Sq) + 1;"),
    ("mask_top_left_aligned", "long lim = i + (Skv - Sq);", "long lim = i;"),
    ("gqa_interleaved_heads", "const long g = h / (Hq / Hkv);", "const long g = h % Hkv;"),
    ("no_scale", "s[j] = scale * acc;", "s[j] = acc;"),
    ("scale_squared", "s[j] = scale * acc;", "s[j] = scale * scale * acc;"),
    ("no_max_subtraction_in_lse", "*lse_out = mx + log(l);", "*lse_out = log(l);"),
    ("lse_base_two", "*lse_out = mx + log(l);", "*lse_out = mx + log2(l);"),
    ("lse_sign", "*lse_out = mx + log(l);", "*lse_out = mx - log(l);"),
    ("no_normalisation", "for (long d = 0; d < D; ++d) o_row[d] /= l;", ""),
    ("exp_sign", "s[j] = exp(s[j] - mx);", "s[j] = exp(mx - s[j]);"),
    ("no_max_subtraction", "s[j] = exp(s[j] - mx);", "s[j] = exp(s[j]);"),
    ("q_row_layout_bhsd", "const double *qrow = q + ((b * Sq + i) * Hq + h) * D;",
     "const double *qrow = q + ((b * Hq + h) * Sq + i) * D;"),
    ("k_uses_query_head", "const double *krow = k + ((b * Skv + j) * Hkv + g) * D;",
     "const double *krow = k + ((b * Skv + j) * Hkv + (h % Hkv)) * D;"),
    ("v_row_is_k_row_index_shift", "const double *vrow = v + ((b * Skv + j) * Hkv + g) * D;",
     "const double *vrow = v + ((b * Skv + (j + 1) % Skv) * Hkv + g) * D;"),
    ("v_ignores_batch", "const double *vrow = v + ((b * Skv + j) * Hkv + g) * D;",
     "const double *vrow = v + ((0 * Skv + j) * Hkv + g) * D;"),
    ("lse_layout_bsh", "lse + (b * Hq + h) * Sq + i);", "lse + (b * Sq + i) * Hq + h);"),
    ("dot_drops_last_dim", "for (long d = 0; d < D; ++d) acc += qrow[d] * krow[d];",
     "for (long d = 0; d + 1 < D || d == 0; ++d) acc += qrow[d] * krow[d];"),
    ("max_over_all_keys_not_valid", "if (s[j] > mx) mx = s[j];", "if (fabs(s[j]) > mx) mx = fabs(s[j]);"),
    ("rows_entry_swaps_b_h", "one_row(q, k, v, rows[3 * r], rows[3 * r + 1], rows[3 * r + 2],",
     "one_row(q, k, v, rows[3 * r + 1] % B, rows[3 * r] % Hq, rows[3 * r + 2],"),
    ("probs_entry_swaps_b_h", "one_row(q, k, zeros, b, h, i,", "one_row(q, k, zeros, h % B, b % Hq, i,"),
    ("probs_entry_ignores_batch", "one_row(q, k, zeros, b, h, i,", "one_row(q, k, zeros, 0, h, i,"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(tmp_path, name, old, new):
    src = open(oracle.SRC).read()
    assert src.count(old) == 1, f"mutation site for {name} not unique in the oracle source"
    msrc = tmp_path / "mut.c"
    msrc.write_text(src.replace(old, new))
    so = oracle.compile_c(str(msrc), str(tmp_path / f"libmut_{name}.so"))
    mut = oracle.Oracle(so)
    caught = []
    for pin in pins.ALL_PINS:
        try:
            pin(mut)
        except AssertionError:
            caught.append(pin.__name__)
        except Exception:            # e.g. overflow turned into NaN/exception: also a detection
            caught.append(pin.__name__)
    assert caught, f"mutant {name} passed every pin"
