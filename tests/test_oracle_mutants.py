"""Plant plausible mistakes in copies of the oracle's source (on the CPU) and show that the pins
catch every one: a dropped term, a wrong sign or index, a missing mask, a swapped operand."""
import os
import subprocess

import pytest

import oracle
import pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "oracle_attn.c")

# (name, text in oracle_attn.c, replacement)
MUTANTS = [
    ("gqa_modulo_mapping", "Lv, h / G, n_kv_heads, head_dim,\n                     (double)scale, out +",
     "Lv, h % n_kv_heads, n_kv_heads, head_dim,\n                     (double)scale, out +"),
    ("no_causal_mask", "const int Lv = kv_lens[b] - q_len + t + 1;\n            attn_row",
     "const int Lv = kv_lens[b];\n            attn_row"),
    ("causal_off_by_one", "const int Lv = kv_lens[b] - q_len + t + 1;\n            attn_row",
     "const int Lv = kv_lens[b] - q_len + t + (t > 0);\n            attn_row"),
    ("no_max_subtraction", "scratch[j] = exp(scratch[j] - m);", "scratch[j] = exp(scratch[j]);"),
    ("min_instead_of_max", "if (scratch[j] > m) m = scratch[j];", "if (j == 0 || scratch[j] < m) m = scratch[j];"),
    ("dropped_scale", "scratch[j] = scale * dot;", "scratch[j] = dot;"),
    ("dropped_normalisation", "for (int d = 0; d < D; ++d) out_row[d] /= Z;", ""),
    ("lse_without_max", "*lse_out = m + log(Z);", "*lse_out = log(Z);"),
    ("lse_without_log", "*lse_out = m + log(Z);", "*lse_out = m + Z;"),
    ("k_head_offset", "K + (size_t)j * row_stride + (size_t)g * D;", "K + (size_t)j * row_stride + (size_t)g;"),
    ("v_head_offset", "V + (size_t)j * row_stride + (size_t)g * D;", "V + (size_t)j * row_stride;"),
    ("v_rows_reversed", "V + (size_t)j * row_stride + (size_t)g * D;",
     "V + (size_t)(Lv - 1 - j) * row_stride + (size_t)g * D;"),
    ("unnormalised_weights", "weights[j] = scratch[j] / Z;", "weights[j] = scratch[j];"),
    ("merge_weight_vs_max", "const double w = exp(l - L);", "const double w = exp(l - M);"),
    ("merge_lse_without_max", "const double L = M + log(Z);", "const double L = log(Z);"),
    ("merge_counts_empty_parts", "if (l > -INFINITY) Z += exp(l - M);", "Z += 1.0;"),
    ("page_div_mod_swapped", "*page_idx = (va - va_start) / page_size;", "*page_idx = (va - va_start) % page_size;"),
    ("write_kvcache_row_off_by_one", "const size_t dst = (size_t)(kv_lens[b] - q_len + t) * (size_t)row_elems;",
     "const size_t dst = (size_t)(kv_lens[b] - q_len + t + 1) * (size_t)row_elems;"),
    ("write_kvcache_v_gets_k", "v_ptrs[b][dst + e] = v_new[src + e];", "v_ptrs[b][dst + e] = k_new[src + e];"),
    ("write_kvcache_source_ignores_token", "const size_t src = ((size_t)b * q_len + t) * (size_t)row_elems;",
     "const size_t src = ((size_t)b * q_len) * (size_t)row_elems;"),
    ("mla_value_uses_wrong_columns", "for (int d = 0; d < d_v; ++d) o[d] += p[j] * bf16_to_f64(C[(size_t)j * d_qk + d]);",
     "for (int d = 0; d < d_v; ++d) o[d] += p[j] * bf16_to_f64(C[(size_t)j * d_qk + d + (d_qk - d_v)]);"),
    ("mla_key_stops_at_value_width", "for (int d = 0; d < d_qk; ++d) dot += bf16_to_f64(q_row[d]) * bf16_to_f64(C[(size_t)j * d_qk + d]);",
     "for (int d = 0; d < d_v; ++d) dot += bf16_to_f64(q_row[d]) * bf16_to_f64(C[(size_t)j * d_qk + d]);"),
    ("mla_no_causal_mask", "const int Lv = kv_lens[b] - q_len + t + 1;\n            const uint16_t* q_row",
     "const int Lv = kv_lens[b];\n            const uint16_t* q_row"),
    ("mla_row_stride_is_value_width", "double dot = 0.0;\n                for (int d = 0; d < d_qk; ++d) dot += bf16_to_f64(q_row[d]) * bf16_to_f64(C[(size_t)j * d_qk + d]);",
     "double dot = 0.0;\n                for (int d = 0; d < d_qk; ++d) dot += bf16_to_f64(q_row[d]) * bf16_to_f64(C[(size_t)j * d_v + d]);"),
    ("token_order_in_q_index", "const int t = (int)((r / n_q_heads) % q_len);", "const int t = 0;"),
]


def _detects(lib_path):
    with oracle.use_library(lib_path):
        for check in pins.ALL_CHECKS:
            try:
                check()
            except Exception:          # AssertionError, ValueError from a rejected call, ...
                return check.__name__
    return None


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_mutant(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) >= 1, "mutation site not found: the oracle changed, update this test"
    mutated = text.replace(old, new)
    c = tmp_path / (name + ".c")
    so = tmp_path / (name + ".so")
    c.write_text(mutated)
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                           str(c), "-o", str(so), "-lm"])
    caught_by = _detects(str(so))
    assert caught_by is not None, "no pin notices mutant '%s'" % name


def test_unmutated_oracle_passes_all_pins():
    assert _detects(oracle.build()) is None
