"""Are the pins sharp?  Each case plants one plausible mistake in a *copy* of ``oracle.c`` (a dropped
term, a wrong index, a swapped operand), compiles it, and requires that at least one pin fails.
Runs on the CPU only; the committed oracle is never modified."""
import os

import pytest

import oracle
from oracle import build as obuild
import oracle_pins

MUTATIONS = {
    "gqa_mod_instead_of_div": ("const int kv_head = h / group;", "const int kv_head = h % n_kv;"),
    "causal_excludes_self": ("prefix_len + j + 1 : prefix_len", "prefix_len + j : prefix_len"),
    "causal_ignores_prefix": ("prefix_len + j + 1 : prefix_len", "j + 1 : prefix_len"),
    "cross_is_causal": ("prefix_len + j + 1 : prefix_len;", "prefix_len + j + 1 : (j + 1 < prefix_len ? j + 1 : prefix_len);"),
    "pool_layout_token_major": ("return ((page * n_kv + kv_head) * (int64_t)page_size + off) * d;",
                                "return ((page * (int64_t)page_size + off) * n_kv + kv_head) * d;"),
    "scale_dropped": ("scores[i] = scale * dot;", "scores[i] = dot;"),
    "no_max_subtraction": ("scores[i] = exp(scores[i] - m);", "scores[i] = exp(scores[i]);"),
    "scatter_ignores_prefix": ("const int pos = prefix_lens[r] + j;", "const int pos = j;"),
    "scatter_v_from_k": ("(const char *)v_new + src * elt_bytes", "(const char *)k_new + src * elt_bytes"),
    "lse_without_max": ("*lse = m + log(z);", "*lse = log(z);"),
    "values_read_from_keys": ("w * widen(v_cache, v_at + c, dtype)", "w * widen(k_cache, v_at + c, dtype)"),
    "page_offset_div": ("pool_index(page, kv_head, i % page_size, n_kv, page_size, d);\n        double dot",
                        "pool_index(page, kv_head, (i + 1) % page_size, n_kv, page_size, d);\n        double dot"),
    "packed_rows_ignore_cu": ("const int64_t src = ((int64_t)(cu_new_lens[r] + j) * n_kv + h) * d;",
                              "const int64_t src = ((int64_t)j * n_kv + h) * d;"),
    "unnormalised": ("const double w = scores[i] / z;", "const double w = scores[i];"),
}


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_mutant_is_caught(name, tmp_path):
    old, new = MUTATIONS[name]
    with open(obuild.SRC) as f:
        src = f.read()
    assert src.count(old) == 1, "mutation anchor must match the oracle source exactly once"
    mutated = tmp_path / "oracle_mutant.c"
    mutated.write_text(src.replace(old, new))
    lib_path = str(tmp_path / ("_mutant_%s.so" % name))
    obuild.build(force=True, src=str(mutated), lib=lib_path)
    lib = oracle.load(lib_path)
    caught = []
    for pin in oracle_pins.ALL_PINS:
        try:
            pin(lib)
        except (AssertionError, ValueError):
            caught.append(pin.__name__)
    assert caught, "no pin noticed the planted mistake %r" % name
