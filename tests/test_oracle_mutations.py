"""The pins must be able to fail: each plausible mistake planted in a COPY of the oracle's C source
(on the CPU, never in the HIP path) has to be caught by at least one pin of test_oracle_pins."""
import ctypes as C
import os
import subprocess

import pytest

from oracle import oracle
from tests import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "ukv_oracle.c")

MUTATIONS = {
    "gqa heads interleaved instead of grouped": (
        "uint32_t a = h * G + g; /* query head a reads kv head a / G */",
        "uint32_t a = g * H + h;"),
    "K and V swapped when reading": (
        "const uint16_t *kr = (const uint16_t *)(pool + a);\n"
        "            const uint16_t *vr = (const uint16_t *)(pool + a + 2ull * d);",
        "const uint16_t *vr = (const uint16_t *)(pool + a);\n"
        "            const uint16_t *kr = (const uint16_t *)(pool + a + 2ull * d);"),
    "scale dropped": ("s[t] = dot * scale;", "s[t] = dot;"),
    "second index taken modulo the token row": (
        "uint64_t second_index = stream % page_bytes;", "uint64_t second_index = stream % token_bytes;"),
    "page slot ignores the head offset": (
        "uint64_t slot = stream / page_bytes;", "uint64_t slot = (t * token_bytes) / page_bytes;"),
    "output not normalised": ("o[(uint64_t)a * d + j] /= l[a];", "o[(uint64_t)a * d + j] /= 1.0;"),
    "key matrix indexed transposed": ("dot += qf[j] * K[t * d + j];", "dot += qf[j] * K[j * n + t];"),
    "first token left out of the sum": (
        "for (uint64_t t = 0; t < n; ++t) {\n                double e = exp(s[t] - m);",
        "for (uint64_t t = 1; t < n; ++t) {\n                double e = exp(s[t] - m);"),
    "append stores V where K belongs": (
        "memcpy(pool + a, new_k + new_off[i] + h * d, 2ull * d);\n"
        "            memcpy(pool + a + 2ull * d, new_v + new_off[i] + h * d, 2ull * d);",
        "memcpy(pool + a, new_v + new_off[i] + h * d, 2ull * d);\n"
        "            memcpy(pool + a + 2ull * d, new_k + new_off[i] + h * d, 2ull * d);"),
    "append one token late": ("t = (uint64_t)ctx_len[i] - 1;", "t = (uint64_t)ctx_len[i];"),
    "merge weights inverted": ("double w = exp(m[c] - M);", "double w = exp(M - m[c]);"),
    "scatter writes head rows token-minor": (
        "memcpy(pool + a, k_in + (t * n_kv_heads + h) * head_dim, 2ull * head_dim);",
        "memcpy(pool + a, k_in + (h * n_tokens + t) * head_dim, 2ull * head_dim);"),
    "chunk scattered one token early": (
        "uint64_t a = head_row_address(page_bytes, n_pages, table, table_len, tok, row, first_token + t, h);\n"
        "            if (a == UINT64_MAX)\n                return ORC_ERANGE;\n"
        "            memcpy(pool + a, k_in",
        "uint64_t a = head_row_address(page_bytes, n_pages, table, table_len, tok, row, first_token + t - (first_token > 0), h);\n"
        "            if (a == UINT64_MAX)\n                return ORC_ERANGE;\n"
        "            memcpy(pool + a, k_in"),
    "prefill mask off by one (own token excluded)": (
        "head_dim, scale, 0, (uint64_t)pos[k] + 1, q_rows + (uint64_t)k * row, m,",
        "head_dim, scale, 0, (uint64_t)pos[k] + (pos[k] == 0), q_rows + (uint64_t)k * row, m,"),
    "prefill not causal (every position sees the whole context)": (
        "head_dim, scale, 0, (uint64_t)pos[k] + 1, q_rows + (uint64_t)k * row, m,",
        "head_dim, scale, 0, (uint64_t)ctx_len, q_rows + (uint64_t)k * row, m,"),
    "prefill uses the first query row for every position": (
        "head_dim, scale, 0, (uint64_t)pos[k] + 1, q_rows + (uint64_t)k * row, m,",
        "head_dim, scale, 0, (uint64_t)pos[k] + 1, q_rows, m,"),
    "gather reads V at the K offset": (
        "memcpy(v_out + (t * n_kv_heads + h) * head_dim, pool + a + 2ull * head_dim, 2ull * head_dim);",
        "memcpy(v_out + (t * n_kv_heads + h) * head_dim, pool + a, 2ull * head_dim);"),
}


def _run_pins():
    pins.test_address_map_matches_hand_worked_fixture()
    for shape, tpp in (("tiny", 8), ("7b", 1), ("8b", 4)):
        pins.test_integral_tokens_per_page_rule(shape, tpp)
    for si in range(len(pins.SMALL_SHAPES)):
        for n in (1, 7, 33):
            pins.test_oracle_equals_bruteforce_and_torch_on_small_shapes(si, n)
    pins.test_oracle_equals_bruteforce_on_service_shapes("13b")
    pins.test_explicit_scale_is_used()
    pins.test_constant_v_per_kv_head_returns_it_and_pins_gqa_mapping()
    pins.test_two_token_logistic_closed_form()
    pins.test_split_and_merge_equals_whole()
    pins.test_append_touches_exactly_the_new_token(5)
    pins.test_scatter_places_every_element_and_inverts_gather("13b")
    pins.test_scatter_of_a_chunk_is_a_bulk_append("13b")
    pins.test_prefill_equals_masked_matrix_and_torch_causal(1, 19)
    pins.test_prefill_closed_forms_and_causality()


def test_unmutated_copy_passes(tmp_path, monkeypatch):
    lib = _build(open(SRC).read(), tmp_path, "clean")
    monkeypatch.setattr(oracle, "_lib", lib)
    _run_pins()


def _build(text, tmp_path, tag):
    c = tmp_path / f"oracle_{tag}.c"
    so = tmp_path / f"liboracle_{tag}.so"
    c.write_text(text)
    subprocess.check_call(["gcc", "-O1", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", str(so), str(c), "-lm"])
    return oracle.bind(C.CDLL(str(so)))


@pytest.mark.parametrize("name", list(MUTATIONS))
def test_planted_mistake_is_caught(name, tmp_path, monkeypatch):
    old, new = MUTATIONS[name]
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation anchor for '{name}' not found exactly once"
    lib = _build(text.replace(old, new), tmp_path, "mut")
    monkeypatch.setattr(oracle, "_lib", lib)
    with pytest.raises((AssertionError, RuntimeError)):
        _run_pins()
