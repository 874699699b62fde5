"""Planted mistakes (CPU only): each mutant is a textual edit of the oracle's C source,
compiled to a temporary library.  At least one pin of test_oracle_pins must fail for
every mutant; otherwise the pins would not notice that mistake in the real oracle."""
import ctypes
import os
import subprocess

import pytest

from oracle import oracle as orc
from tests import test_oracle_pins as pins

MUTANTS = {
    "dropped_scale": ("scratch[j] = scale * acc;", "scratch[j] = acc;"),
    "no_max_subtraction_and_wrong_lse": ("if (lse) *lse = m + log(Z);", "if (lse) *lse = log(Z);"),
    "causal_off_by_one": ("const int n = p + 1;", "const int n = p > 0 ? p : 1;"),
    "gqa_interleaved_heads": ("const int h = g * G + hh;", "const int h = hh * Hkv + g;"),
    "slot_index": ("const int slot = p % bs;", "const int slot = (p + 1) % bs;"),
    "block_index": ("const int j = p / bs;", "const int j = (p + bs - 1) / bs;"),
    "v_gathered_from_k": ("rc = gather_dense(Vd, v_cache,", "rc = gather_dense(Vd, k_cache,"),
    "unnormalised": ("const double Pj = scratch[j] / Z;", "const double Pj = scratch[j];"),
    "append_swaps_k_v": ("memcpy((char *)v_cache + dst * es, (const char *)v_new + src * es",
                         "memcpy((char *)v_cache + dst * es, (const char *)k_new + src * es"),
    "decode_ignores_self": ("pos[b] = ctx_len[b] - 1;", "pos[b] = ctx_len[b] > 1 ? ctx_len[b] - 2 : 0;"),
    "prefill_ignores_prefix": ("pos[t] = ctx_before[b] + (t - cu_q[b]);", "pos[t] = (t - cu_q[b]);"),
    "head_stride": ("const size_t src = (t * (size_t)Hkv + (size_t)g) * (size_t)D;",
                    "const size_t src = (t * (size_t)Hkv) * (size_t)D;"),
}

PIN_FUNCS = [
    lambda: [pins.test_prefill_matches_dense_bruteforce(m, q) for m, q in pins.CASES],
    pins.test_chunked_appends_and_decode_match_dense_bruteforce,
    pins.test_two_key_softmax_by_hand,
    pins.test_default_scale_is_inverse_sqrt_head_dim,
    lambda: pins.test_single_token_context_returns_v_exactly("bf16"),
    pins.test_equal_keys_give_running_mean_of_values,
    pins.test_weights_sum_to_one_and_reproduce_output,
    pins.test_append_places_rows_bit_exactly_and_leaves_holes,
    pins.test_decode_equals_last_prefill_row,
]


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_planted_mistake(name, tmp_path, monkeypatch):
    old, new = MUTANTS[name]
    src = open(orc._SRC).read()
    assert src.count(old) == 1, f"mutation anchor for {name} not found exactly once"
    c = tmp_path / "mutant.c"
    so = tmp_path / "mutant.so"
    c.write_text(src.replace(old, new))
    subprocess.run(["gcc", "-O1", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", str(so), str(c), "-lm"], check=True)
    lib = ctypes.CDLL(str(so))
    lib.oracle_num_threads.restype = ctypes.c_int
    orc._load()
    monkeypatch.setattr(orc, "_lib", lib)
    caught = 0
    for f in PIN_FUNCS:
        try:
            f()
        except (AssertionError, ValueError):
            caught += 1
    assert caught >= 1, f"no pin noticed mutant {name}"
