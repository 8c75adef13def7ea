"""The pins are sharp: a plausible mistake planted in the oracle makes at least one of them fail.

Each case edits a temporary copy of oracle/pc_oracle.c (one textual substitution: a dropped term, a wrong sign,
index or operand), compiles it with the host compiler and runs the pins named for that part of the oracle against the
mutated build.  Nothing here touches the GPU path; the committed oracle is never modified.
"""
import contextlib
import os
import subprocess
import tempfile

import pytest

import oracle
import test_oracle_pins as pins


@contextlib.contextmanager
def planted(old: str, new: str):
    src = open(oracle._SRC).read()
    assert src.count(old) >= 1, f"the oracle no longer contains: {old!r}"
    with tempfile.TemporaryDirectory() as td:
        c_path, so_path = os.path.join(td, "mutant.c"), os.path.join(td, "libmutant.so")
        with open(c_path, "w") as f:
            f.write(src.replace(old, new, 1))
        subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-o", so_path, c_path, "-lm"], check=True)
        oracle._load()
        saved = oracle._lib
        oracle._lib = oracle._bind(so_path)
        try:
            yield
        finally:
            oracle._lib = saved


def _fails(check) -> bool:
    try:
        check()
    except (AssertionError, pytest.fail.Exception):
        return True
    except Exception:   # a mutant may also break a shape or raise inside a pin: that counts as caught
        return True
    return False


# (what is planted, text in the oracle, replacement, pins that must notice)
MUTANTS = [
    ("union spans the sum of its children", "if (size[j] > widest) widest = size[j];", "widest += size[j];",
     [pins.test_layout_union_shares_start_and_spans_largest_child, pins.test_layout_brute_force_random_schemas]),
    ("union children laid one after the other", "start[j] = (int)cursor;\n                if (size[j] > widest)",
     "start[j] = (int)cursor + widest;\n                if (size[j] > widest)",
     [pins.test_layout_union_shares_start_and_spans_largest_child, pins.test_layout_brute_force_random_schemas]),
    ("module start ignores the module before it", "cursor += size[i];", "cursor += 0;",
     [pins.test_layout_printed_example]),
    ("text starts one position late", "pos[i] = prev_start + prev_len + i;", "pos[i] = prev_start + prev_len + i + 1;",
     [pins.test_text_positions_continue_after_preceding_module]),
    ("rotation turns the other way", "v[i] = lo * c - hi * s;\n                v[i + half] = hi * c + lo * s;",
     "v[i] = lo * c + hi * s;\n                v[i + half] = hi * c - lo * s;",
     [pins.test_rope_closed_forms_fix_direction_pairing_and_frequency, pins.test_rope_matches_complex_formulation_at_discontinuous_positions]),
    ("rotation frequency exponent halved", "pow(base, -2.0 * (double)i / (double)d)", "pow(base, -1.0 * (double)i / (double)d)",
     [pins.test_rope_closed_forms_fix_direction_pairing_and_frequency, pins.test_rope_matches_complex_formulation_at_discontinuous_positions]),
    ("rotation by the row index instead of the position ID", "double angle = (double)pos[t] * theta;", "double angle = (double)t * theta;",
     [pins.test_rope_matches_complex_formulation_at_discontinuous_positions, pins.test_rope_identity_norm_and_additivity]),
    ("rotation pairs neighbours instead of halves", "double lo = v[i], hi = v[i + half];\n                v[i] = lo * c - hi * s;\n                v[i + half] = hi * c + lo * s;",
     "double lo = v[2 * i], hi = v[2 * i + 1];\n                v[2 * i] = lo * c - hi * s;\n                v[2 * i + 1] = hi * c + lo * s;",
     [pins.test_rope_closed_forms_fix_direction_pairing_and_frequency, pins.test_rope_matches_complex_formulation_at_discontinuous_positions]),
    ("assembled position is the buffer row", "out_pos[row] = mod_start[m] + i;", "out_pos[row] = (int32_t)row;",
     [pins.test_assemble_is_packed_concat_with_schema_positions, pins.test_omitting_a_module_leaves_other_positions_unchanged]),
    ("assembled V copied from K", "out_V[(size_t)row * row_bytes + b] = mod_V[m]", "out_V[(size_t)row * row_bytes + b] = mod_K[m]",
     [pins.test_assemble_is_packed_concat_with_schema_positions, pins.test_assemble_keeps_every_bit_pattern]),
    ("a token does not see its own position", "if (k_pos[j] <= q_pos[q]) {\n                const double *k = K + ((size_t)j * Hkv + kvh) * d;\n                double dot = 0.0;\n                for (int c = 0; c < d; ++c) dot += qrot[c]",
     "if (k_pos[j] < q_pos[q]) {\n                const double *k = K + ((size_t)j * Hkv + kvh) * d;\n                double dot = 0.0;\n                for (int c = 0; c < d; ++c) dot += qrot[c]",
     [pins.test_attn_contiguous_positions_is_textbook_causal_attention, pins.test_attn_single_visible_key_returns_its_value]),
    ("mask dropped", "if (k_pos[j] <= q_pos[q]) {\n                const double *k = K + ((size_t)j * Hkv + kvh) * d;\n                double dot = 0.0;\n                for (int c = 0; c < d; ++c) dot += qrot[c]",
     "if (1) {\n                const double *k = K + ((size_t)j * Hkv + kvh) * d;\n                double dot = 0.0;\n                for (int c = 0; c < d; ++c) dot += qrot[c]",
     [pins.test_attn_masked_slots_cannot_leak, pins.test_attn_mask_is_on_positions_not_buffer_order_and_sees_gaps]),
    ("scores scaled by 1/d", "double inv_sqrt_d = 1.0 / sqrt((double)d);\n    long pairs = (long)nq * Hq;\n#ifdef _OPENMP\n#pragma omp parallel for schedule(dynamic, 4) num_threads(g_threads)\n#endif\n    for (long w = 0; w < pairs; ++w) {\n        int q = (int)(w / Hq), h = (int)(w % Hq);\n        int kvh = h / group;\n        double *qrot",
     "double inv_sqrt_d = 1.0 / (double)d;\n    long pairs = (long)nq * Hq;\n#ifdef _OPENMP\n#pragma omp parallel for schedule(dynamic, 4) num_threads(g_threads)\n#endif\n    for (long w = 0; w < pairs; ++w) {\n        int q = (int)(w / Hq), h = (int)(w % Hq);\n        int kvh = h / group;\n        double *qrot",
     [pins.test_attn_scale_is_one_over_sqrt_d, pins.test_attn_contiguous_positions_is_textbook_causal_attention]),
    ("query heads mapped to kv heads round-robin", "int kvh = h / group;\n        double *qrot", "int kvh = h % Hkv;\n        double *qrot",
     [pins.test_attn_gqa_equals_mha_with_repeated_kv_heads]),
    ("queries not rotated", "orc_rope(qrot, 1, 1, d, q_pos + q, base);", ";",
     [pins.test_attn_rotates_queries_with_the_same_convention_as_keys, pins.test_attn_contiguous_positions_is_textbook_causal_attention]),
    ("values always taken from kv head 0", "softmax_times_v(s, nkv, V + (size_t)kvh * d, Hkv * d, d, out + ((size_t)q * Hq + h) * d);\n        free(s);\n        free(qrot);",
     "softmax_times_v(s, nkv, V, Hkv * d, d, out + ((size_t)q * Hq + h) * d);\n        free(s);\n        free(qrot);",
     [pins.test_attn_gqa_equals_mha_with_repeated_kv_heads, pins.test_attn_contiguous_positions_is_textbook_causal_attention]),
    ("softmax not normalised", "double p = exp(s[j] - top) / denom;", "double p = exp(s[j] - top);",
     [pins.test_attn_identical_keys_average_the_visible_values, pins.test_attn_contiguous_positions_is_textbook_causal_attention]),
    ("bias slopes start one step early", "slopes[i] = pow(2.0, -8.0 * (double)(i + 1) / (double)p);", "slopes[i] = pow(2.0, -8.0 * (double)i / (double)p);",
     [pins.test_alibi_slopes_match_the_published_sequence]),
    ("bias slopes for other head counts taken consecutively", "pow(2.0, -8.0 * (double)(2 * i + 1) / (double)(2 * p))", "pow(2.0, -8.0 * (double)(i + 1) / (double)(2 * p))",
     [pins.test_alibi_slopes_match_the_published_sequence]),
    ("bias rewards distance", "s[j] = dot * inv_sqrt_d - slope[h] * (double)(q_pos[q] - k_pos[j]);", "s[j] = dot * inv_sqrt_d + slope[h] * (double)(q_pos[q] - k_pos[j]);",
     [pins.test_alibi_zero_queries_give_the_geometric_closed_form, pins.test_alibi_matches_library_attention_with_an_additive_mask]),
    ("bias measured in buffer rows", "s[j] = dot * inv_sqrt_d - slope[h] * (double)(q_pos[q] - k_pos[j]);", "s[j] = dot * inv_sqrt_d - slope[h] * (double)(q_pos[q] - j);",
     [pins.test_alibi_distance_is_measured_in_position_ids_not_buffer_rows]),
    ("bias uses the slope of head 0", "s[j] = dot * inv_sqrt_d - slope[h] * (double)(q_pos[q] - k_pos[j]);", "s[j] = dot * inv_sqrt_d - slope[0] * (double)(q_pos[q] - k_pos[j]);",
     [pins.test_alibi_matches_library_attention_with_an_additive_mask, pins.test_alibi_zero_queries_give_the_geometric_closed_form]),
    ("module tokens see other modules", "(module_of[a] == module_of[b] || module_of[a] < 0)", "(1)",
     [pins.test_cached_attention_equals_full_recompute_under_module_local_mask]),
    ("uncached tokens confined like module tokens", "(module_of[a] == module_of[b] || module_of[a] < 0)", "(module_of[a] == module_of[b])",
     [pins.test_cached_attention_equals_full_recompute_under_module_local_mask]),
    ("argument keys not rotated", "orc_rope(k, 1, n_heads, d, &pos[row0 + i], base);", ";",
     [pins.test_param_full_length_argument_equals_module_encoded_with_the_argument_in_place]),
    ("unused placeholders stay tokens", "for (int i = n_arg; i < len; ++i) pos[row0 + i] = ORC_POS_NONE;", ";",
     [lambda: pins.test_param_shorter_argument_trailing_placeholders_stop_being_tokens(1)]),
    ("argument values not replaced", "v[c] = V_arg[(size_t)i * row + c];", ";",
     [pins.test_param_full_length_argument_equals_module_encoded_with_the_argument_in_place]),
    ("longer argument accepted", "if (n_arg < 0 || len < 0 || n_arg > len) return -1;", "if (n_arg < 0 || len < 0) return -1;",
     [pins.test_param_argument_longer_than_parameter_is_rejected]),
    ("bytes per token counts one tensor", "return 2L * n_layers * n_kv_heads * head_dim * elem_bytes;", "return 1L * n_layers * n_kv_heads * head_dim * elem_bytes;",
     [pins.test_bytes_per_token_matches_table2]),
]


def test_pins_pass_on_the_committed_oracle():
    """The control: every pin used below passes against the oracle as committed."""
    seen = set()
    for _, _, _, checks in MUTANTS:
        for check in checks:
            if getattr(check, "__name__", "<lambda>") in seen:
                continue
            seen.add(getattr(check, "__name__", "<lambda>"))
            check()


@pytest.mark.parametrize("what,old,new,checks", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(what, old, new, checks):
    with planted(old, new):
        caught = [getattr(c, "__name__", "pin") for c in checks if _fails(c)]
    assert caught, f"no pin noticed: {what}"
