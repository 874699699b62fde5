"""Pins of the byte/FLOP accounting against numbers and formulas the paper prints."""
import os

import numpy as np

from paper_2504_18154_amd import accounting as acc
from paper_2504_18154_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_kv_sizing.txt")


def _rows():
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        kind, model, layers, hkv, d, tps, val, unit = line.split()
        yield kind, model, int(layers), int(hkv), int(d), tps, float(val), unit


def test_kv_sizing_reproduces_printed_values():
    n = 0
    for kind, model, layers, hkv, d, tps, val, unit in _rows():
        per_tok = acc.kv_bytes_per_token(layers, hkv, d, 2)
        if kind == "per_token":
            assert abs(per_tok / 2**20 - val) < 0.005          # printed to 2 decimals
        elif kind == "batch":
            assert abs(round(per_tok / 2**20, 2) * float(tps) / 1000 - val) < 0.05
        else:
            digits = len(str(val).split(".")[1])
            assert abs(per_tok * float(tps) / 2**30 - val) < 0.6 * 10 ** (-digits), (model, tps)
        n += 1
    assert n == 6


def test_table2_flops_and_causal_count():
    # Table 2: decode QK^T = 2BSH, prefill = 2BS^2H, H = heads * D
    assert acc.table2_attention_flops("decode", 3, 100, 40, 128) == 2 * 3 * 100 * 40 * 128
    assert acc.table2_attention_flops("prefill", 3, 100, 40, 128) == 2 * 3 * 100 * 100 * 40 * 128
    # both matmuls of a decode step == 2 x the table row, for uniform lengths
    assert acc.decode_flops([100] * 3, 40, 128) == 2 * acc.table2_attention_flops("decode", 3, 100, 40, 128)
    # causal prefill credits S(S+1)/2 of the S^2 entries
    full = 2 * acc.table2_attention_flops("prefill", 1, 64, 8, 128)
    assert acc.prefill_flops_causal([64], 8, 128) * 64 * 2 == full * 65
    # brute-force count of (query, key) pairs with a cached prefix
    pairs = sum(c + i + 1 for S, c in [(5, 3), (7, 0)] for i in range(S))
    assert acc.prefill_flops_causal([5, 7], 2, 16, [3, 0]) == 4 * 2 * 16 * pairs


def test_bytes_per_token_of_bench_shapes():
    assert wl.M30B.kv_bytes_per_token_layer == 4096 and wl.M70B.kv_bytes_per_token_layer == 4096
    L = np.array([17, 32])
    b = acc.decode_bytes(L, 40, 8, 128, 16)
    assert b == 49 * 4096 + 2 * 2 * 40 * 128 * 2 + (2 + 2) * 4
    assert acc.append_bytes(10, 8, 128) == 2 * 10 * 4096


def test_workload_recipes_are_seeded_and_in_range():
    a, b = wl.config2_decode_30b(), wl.config2_decode_30b()
    assert np.array_equal(a.ctx_len, b.ctx_len) and np.array_equal(a.block_table, b.block_table)
    assert a.B == 128 and a.ctx_len.min() >= 512 and a.ctx_len.max() <= 4096
    used = a.block_table[a.block_table >= 0]
    assert len(np.unique(used)) == len(used) and used.max() < a.num_blocks
    assert a.num_blocks >= int(1.09 * len(used))
    nblk = (a.ctx_len + 15) // 16
    assert all((a.block_table[i, :n] >= 0).all() and (a.block_table[i, n:] == -1).all() for i, n in enumerate(nblk))
    p = wl.config3_prefill_30b()
    assert p.B == 16 and p.q_len.min() >= 128 and p.q_len.max() <= 4096
    d4 = wl.config4_decode_70b()
    assert d4.B == 256 and d4.ctx_len.min() >= 1024
    res, ql, table, nb = wl.config5_switch_70b()
    assert len(res) == 192 and list(ql) == [8192] * 8 and table.shape[0] == 200
    assert table.shape[1] >= (8192 + 64 + 15) // 16
    t = wl.config1_tiny()
    assert list(t.q_len) == [37, 100] and t.block_table.shape == (2, 7)


def test_table4_shaped_lengths_reproduce_the_table():
    """The synthetic stand-ins for the paper's datasets have Table 4's averages and medians
    (inputs are cut at 4096 tokens as in Section 4.1, which lowers ShareGPT's input average a little)."""
    for name, (in_avg, in_med, out_avg, out_med) in wl.TABLE4.items():
        n_in, n_out = wl.table4_lengths(name, wl.rng_for(5), 40000)
        assert n_in.min() >= 1 and n_in.max() <= 4096 and n_out.min() >= 1
        assert abs(np.median(n_in) - in_med) <= 0.03 * in_med + 1
        assert abs(np.median(n_out) - out_med) <= 0.03 * out_med + 1
        assert abs(n_out.mean() - out_avg) <= 0.10 * out_avg   # the cut at 4096 trims LongBench's heavy tail
        assert in_avg * (0.93 if name == "sharegpt" else 0.97) <= n_in.mean() <= 1.03 * in_avg
    db = wl.table4_decode_batch(wl.M30B, "sharegpt", 64, 9)
    assert db.B == 64 and db.ctx_len.min() >= 2
    used = db.block_table[db.block_table >= 0]
    assert len(np.unique(used)) == len(used) and used.max() < db.num_blocks
    assert all((db.block_table[i, :(n + 15) // 16] >= 0).all() for i, n in enumerate(db.ctx_len))
