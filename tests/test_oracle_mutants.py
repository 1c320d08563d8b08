"""Planted mistakes in the oracle must be caught by its pins (CPU only).

Each mutant is the oracle's C source with one plausible slip (a dropped term, a wrong sign or
index, a transposed layout).  It is compiled to a temporary library, swapped in for the real
one, and the pin tests are run against it: at least one pin has to fail.
"""
import os
import subprocess

import numpy as np
import pytest

import test_oracle_pins as pins
from oracle import tetri_oracle

SRC = open(tetri_oracle._SRC).read()

MUTANTS = {
    "exp-sign": ("exp(scratch[j] - m)", "exp(m - scratch[j])"),
    "drop-diagonal": ("for (int j = 0; j <= p; ++j) {\n        const float *kv = ",
                      "for (int j = 0; j < p; ++j) {\n        const float *kv = "),
    "drop-context": ("    int p = ctx[s] + t;\n    int kh", "    int p = t;\n    int kh"),
    "gqa-mapping": ("h / (Hq / Hkv)", "h % Hkv"),
    "slot-index": ("which, kh, j % P, Hkv", "which, kh, j / P, Hkv"),
    "drop-segment-offset": ("(size_t)(cu[s] + (j - ctx[s])) * Hkv", "(size_t)(j - ctx[s]) * Hkv"),
    "drop-scale": ("scratch[j] = scale * dot;", "scratch[j] = dot;"),
    "drop-normalisation": ("(float)(acc[d] / l)", "(float)(acc[d])"),
    "pool-layout": ("(((size_t)page * 2 + (size_t)which) * (size_t)Hkv + (size_t)head)",
                    "(((size_t)page * (size_t)Hkv + (size_t)head) * 2 + (size_t)which)"),
    "append-slot": ("int slot = p % P;", "int slot = t % P;"),
    "append-row": ("int row = cu[s] + t;", "int row = t;"),
    "context-boundary": ("if (j < ctx[s]) {", "if (j <= ctx[s]) {"),
    "drop-query-head": ("(size_t)(cu[s] + t) * Hq + h) * (size_t)D;\n    double m",
                        "(size_t)(cu[s] + t) * Hq) * (size_t)D;\n    double m"),
    "pad-not-zero": ("++i) out[i] = 0.0f;", "++i) out[i] = 1.0f;"),
    "value-from-key": ("const float *src = which ? v_new : k_new;", "const float *src = k_new;"),
    "transposed-dot": ("dot += (double)qv[d] * (double)kv[d];", "dot += (double)qv[D - 1 - d] * (double)kv[d];"),
    "sample-head": ("attn_one_row(s, r - cu[s], heads[i],", "attn_one_row(s, r - cu[s], 0,"),
}


def _pin_calls():
    o = tetri_oracle
    calls = [
        lambda: pins.test_tiny_config_matches_brute_force(o),
        lambda: pins.test_packed_gqa_matches_brute_force(o),
        lambda: pins.test_unchunked_prompt_matches_library_sdpa(o),
        lambda: pins.test_hand_computed_two_and_three_tokens(o),
        lambda: pins.test_first_token_returns_its_own_value(o),
        lambda: pins.test_zero_keys_or_zero_scale_give_prefix_mean(o),
        lambda: pins.test_constant_values_pass_through(o),
        lambda: pins.test_dominant_key_selects_its_value(o),
        lambda: pins.test_softmax_rows_are_distributions(o),
        lambda: pins.test_sampled_rows_equal_full_rows(o),
        lambda: pins.test_chunked_equals_whole_prompt(o, 16),
        lambda: pins.test_result_independent_of_paging(o, 1),
        lambda: pins.test_requests_do_not_see_each_other(o),
        lambda: pins.test_padding_rows_are_inert_and_zero(o),
        lambda: pins.test_gqa_equals_mha_with_replicated_kv_heads(o),
        lambda: pins.test_append_closed_form(o, np.uint16),
    ]
    return calls


def test_every_mutation_site_exists():
    for name, (old, _new) in MUTANTS.items():
        assert SRC.count(old) == 1, f"mutation site for {name} not found exactly once"


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_mutant(name, tmp_path):
    old, new = MUTANTS[name]
    src = tmp_path / "mutant.c"
    lib = tmp_path / f"mutant_{name}.so"
    src.write_text(SRC.replace(old, new))
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-o", str(lib), str(src), "-lm"])
    real = tetri_oracle.load()
    caught = []
    try:
        tetri_oracle._lib = tetri_oracle.load(str(lib))
        for call in _pin_calls():
            try:
                call()
            except (AssertionError, RuntimeError):
                caught.append(call)
    finally:
        tetri_oracle._lib = real
    assert caught, f"no pin noticed the planted mistake '{name}'"


def test_unmutated_oracle_passes_the_same_calls():
    for call in _pin_calls():
        call()
