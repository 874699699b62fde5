"""Pins of the fp64 CPU oracle against things that are not the oracle.

Each test fixes one way the oracle could be wrong (a dropped scale, a wrong
head->group map, a transposed operand, an off-by-one causal bound, a wrong block
or slot index) to something the paper and the mathematics determine:
  * an independent dense NumPy evaluation of Eq. 2 (Section 2.1) that never sees
    a block table: K/V are taken straight from the token stream;
  * a library SDPA routine on the case that reduces to it (no GQA, one sequence);
  * closed forms: single-token context, equal keys, a 2-key softmax by hand;
  * invariants: weights sum to one, physical block permutation changes nothing.
All CPU-only.
"""
import math

import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2504_18154_amd import workloads as wl


def _np64(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().to(torch.float64).numpy()


def _dense_reference(q, K, V, p, G):
    """Eq. 2 written densely and independently: q [Hq,D], K,V [L,Hkv,D] (float64),
    causal bound p.  No paging, no cache, one softmax per head via the textbook formula."""
    Hq, D = q.shape
    out = np.zeros((Hq, D))
    lse = np.zeros(Hq)
    for h in range(Hq):
        kk = K[: p + 1, h // G, :]
        vv = V[: p + 1, h // G, :]
        s = (kk @ q[h]) / math.sqrt(D)
        e = np.exp(s - s.max())
        out[h] = (e / e.sum()) @ vv
        lse[h] = s.max() + math.log(e.sum())
    return out, lse


def _setup(model, q_len, ctx_before=None, seed=7, grow=0):
    pb = wl.prefill_batch(model, q_len, seed, ctx_before=ctx_before, grow=grow)
    dt = orc.BF16 if model.dtype == "bf16" else orc.F32
    shape = orc.Shape(model.Hq, model.Hkv, model.D, model.bs, pb.num_blocks, dt)
    return pb, shape


CASES = [
    (wl.ModelShape("a", 4, 2, 64, 1, "f32"), [37, 100]),
    (wl.ModelShape("b", 6, 2, 32, 1, "bf16"), [1, 16, 17, 33]),
    (wl.ModelShape("c", 5, 5, 16, 1, "f32"), [15, 0, 31]),
    (wl.ModelShape("d", 8, 1, 128, 1, "bf16"), [48]),
    (wl.ModelShape("e", 3, 3, 8, 1, "f32", bs=4), [9, 2]),
]


@pytest.mark.parametrize("model,q_len", CASES)
def test_prefill_matches_dense_bruteforce(model, q_len):
    pb, shape = _setup(model, q_len)
    T = pb.T
    q = wl.randn((T, model.Hq, model.D), model.dtype, 11)
    k = wl.randn((T, model.Hkv, model.D), model.dtype, 12)
    v = wl.randn((T, model.Hkv, model.D), model.dtype, 13)
    kc, vc = orc.new_cache(shape)
    orc.kv_append(shape, kc, vc, wl.to_bits(k), wl.to_bits(v), pb.cu_q, pb.ctx_before, pb.block_table)
    out, lse = orc.attn_prefill(shape, wl.to_bits(q), kc, vc, pb.cu_q, pb.ctx_before, pb.block_table)
    q64, k64, v64 = _np64(q), _np64(k), _np64(v)
    for b in range(pb.B):
        a, e = int(pb.cu_q[b]), int(pb.cu_q[b + 1])
        for i in range(e - a):
            ref, ref_lse = _dense_reference(q64[a + i], k64[a:e], v64[a:e], i, model.G)
            np.testing.assert_allclose(out[a + i], ref, rtol=0, atol=1e-12)
            np.testing.assert_allclose(lse[a + i], ref_lse, rtol=0, atol=1e-12)


def test_chunked_appends_and_decode_match_dense_bruteforce():
    """Cache built by several appends (prefix, second chunk, single tokens); the dense
    reference is built from the concatenated token stream only."""
    model = wl.ModelShape("m", 4, 2, 32, 1, "bf16")
    lens0, lens1, steps = [21, 5, 40], [11, 30, 0], 3
    total = [a + b + steps for a, b in zip(lens0, lens1)]
    pb, shape = _setup(model, total)  # table sized for the final lengths
    B = 3
    kc, vc = orc.new_cache(shape)
    streams_k = [[] for _ in range(B)]
    streams_v = [[] for _ in range(B)]
    ctx = np.zeros(B, dtype=np.int32)
    seed = 100
    for lens in (lens0, lens1):
        cu = wl.cu_from_lengths(lens)
        T = int(cu[-1])
        k = wl.randn((T, model.Hkv, model.D), "bf16", seed); seed += 1
        v = wl.randn((T, model.Hkv, model.D), "bf16", seed); seed += 1
        q = wl.randn((T, model.Hq, model.D), "bf16", seed); seed += 1
        orc.kv_append(shape, kc, vc, wl.to_bits(k), wl.to_bits(v), cu, ctx, pb.block_table)
        for b in range(B):
            streams_k[b].append(_np64(k)[cu[b]:cu[b + 1]])
            streams_v[b].append(_np64(v)[cu[b]:cu[b + 1]])
        out, lse = orc.attn_prefill(shape, wl.to_bits(q), kc, vc, cu, ctx, pb.block_table)
        for b in range(B):
            K = np.concatenate(streams_k[b]); V = np.concatenate(streams_v[b])
            for i in range(lens[b]):
                ref, ref_lse = _dense_reference(_np64(q)[cu[b] + i], K, V, int(ctx[b]) + i, model.G)
                np.testing.assert_allclose(out[cu[b] + i], ref, rtol=0, atol=1e-12)
                np.testing.assert_allclose(lse[cu[b] + i], ref_lse, rtol=0, atol=1e-12)
        ctx = ctx + np.asarray(lens, dtype=np.int32)
    ones = wl.cu_from_lengths([1] * B)
    for _ in range(steps):
        k = wl.randn((B, model.Hkv, model.D), "bf16", seed); seed += 1
        v = wl.randn((B, model.Hkv, model.D), "bf16", seed); seed += 1
        q = wl.randn((B, model.Hq, model.D), "bf16", seed); seed += 1
        orc.kv_append(shape, kc, vc, wl.to_bits(k), wl.to_bits(v), ones, ctx, pb.block_table)
        ctx = ctx + 1
        out, lse = orc.attn_decode(shape, wl.to_bits(q), kc, vc, pb.block_table, ctx)
        for b in range(B):
            streams_k[b].append(_np64(k)[b:b + 1]); streams_v[b].append(_np64(v)[b:b + 1])
            K = np.concatenate(streams_k[b]); V = np.concatenate(streams_v[b])
            ref, ref_lse = _dense_reference(_np64(q)[b], K, V, int(ctx[b]) - 1, model.G)
            np.testing.assert_allclose(out[b], ref, rtol=0, atol=1e-12)
            np.testing.assert_allclose(lse[b], ref_lse, rtol=0, atol=1e-12)


def test_reduces_to_library_sdpa():
    """No GQA, one sequence, identity block table: ordinary causal SDPA (library routine, fp64)."""
    model = wl.ModelShape("s", 3, 3, 32, 1, "f32")
    S = 45
    nblk = (S + model.bs - 1) // model.bs
    shape = orc.Shape(3, 3, 32, 16, nblk, orc.F32)
    table = np.arange(nblk, dtype=np.int32)[None, :]
    q = wl.randn((S, 3, 32), "f32", 1); k = wl.randn((S, 3, 32), "f32", 2); v = wl.randn((S, 3, 32), "f32", 3)
    kc, vc = orc.new_cache(shape)
    cu = np.array([0, S], dtype=np.int32); cb = np.zeros(1, dtype=np.int32)
    orc.kv_append(shape, kc, vc, wl.to_bits(k), wl.to_bits(v), cu, cb, table)
    out, _ = orc.attn_prefill(shape, wl.to_bits(q), kc, vc, cu, cb, table)
    ref = torch.nn.functional.scaled_dot_product_attention(
        q.double().permute(1, 0, 2)[None], k.double().permute(1, 0, 2)[None], v.double().permute(1, 0, 2)[None],
        is_causal=True)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)


def test_two_key_softmax_by_hand():
    """D = 1, scale 1: scores (0, ln 3) give weights (1/4, 3/4); values (0, 4) give 3; lse = ln 4."""
    shape = orc.Shape(1, 1, 1, 16, 1, orc.F32)
    table = np.zeros((1, 1), dtype=np.int32)
    k = np.array([0.0, math.log(3.0)], dtype=np.float32).reshape(2, 1, 1)
    v = np.array([0.0, 4.0], dtype=np.float32).reshape(2, 1, 1)
    q = np.ones((1, 1, 1), dtype=np.float32)
    kc, vc = orc.new_cache(shape)
    orc.kv_append(shape, kc, vc, k, v, [0, 2], [0], table)
    out, lse, probs = orc.attn_rows(shape, q, kc, vc, table, [0, 1], [0], [1], scale=1.0, want_probs=True)
    s1 = float(np.float32(math.log(3.0)))
    w = math.exp(s1)
    assert abs(out[0, 0, 0] - 4.0 * w / (1 + w)) < 1e-14
    assert abs(out[0, 0, 0] - 3.0) < 1e-6
    assert abs(lse[0, 0] - math.log(1 + w)) < 1e-14
    np.testing.assert_allclose(probs[0, 0], [1 / (1 + w), w / (1 + w)], atol=1e-15)
    # causal bound: the same query at position 0 sees only the first key
    out0, lse0 = orc.attn_rows(shape, q, kc, vc, table, [0, 1], [0], [0], scale=1.0)
    assert out0[0, 0, 0] == 0.0 and lse0[0, 0] == 0.0


def test_default_scale_is_inverse_sqrt_head_dim():
    """Eq. 2's 1/sqrt(d_k): with q = k = ones(D), two keys, the second doubled: score gap = sqrt(D)."""
    D = 64
    shape = orc.Shape(1, 1, D, 16, 1, orc.F32)
    table = np.zeros((1, 1), dtype=np.int32)
    k = np.stack([np.ones(D), 2 * np.ones(D)]).astype(np.float32).reshape(2, 1, D)
    v = np.stack([np.zeros(D), np.ones(D)]).astype(np.float32).reshape(2, 1, D)
    q = np.ones((1, 1, D), dtype=np.float32)
    kc, vc = orc.new_cache(shape)
    orc.kv_append(shape, kc, vc, k, v, [0, 2], [0], table)
    out, lse = orc.attn_decode(shape, q, kc, vc, table, [2])
    gap = math.sqrt(D)  # (2D - D)/sqrt(D)
    expect = 1.0 / (1.0 + math.exp(-gap))
    np.testing.assert_allclose(out[0, 0], expect, atol=1e-14)
    assert abs(lse[0, 0] - (2 * D / math.sqrt(D) + math.log1p(math.exp(-gap)))) < 1e-12


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_single_token_context_returns_v_exactly(dtype):
    model = wl.ModelShape("one", 6, 3, 64, 1, dtype)
    pb, shape = _setup(model, [1, 1, 1])
    q = wl.randn((3, 6, 64), dtype, 1, scale=5.0)
    k = wl.randn((3, 3, 64), dtype, 2); v = wl.randn((3, 3, 64), dtype, 3)
    kc, vc = orc.new_cache(shape)
    orc.kv_append(shape, kc, vc, wl.to_bits(k), wl.to_bits(v), pb.cu_q, pb.ctx_before, pb.block_table)
    out, lse = orc.attn_decode(shape, wl.to_bits(q), kc, vc, pb.block_table, [1, 1, 1])
    v64 = _np64(v)
    for h in range(6):
        assert np.array_equal(out[:, h, :], v64[:, h // 2, :])
    out_p, _ = orc.attn_prefill(shape, wl.to_bits(q), kc, vc, pb.cu_q, pb.ctx_before, pb.block_table)
    assert np.array_equal(out_p, out)


def test_equal_keys_give_running_mean_of_values():
    model = wl.ModelShape("eq", 4, 2, 32, 1, "bf16")
    S = 53
    pb, shape = _setup(model, [S])
    q = wl.randn((S, 4, 32), "bf16", 1)
    k1 = wl.randn((1, 2, 32), "bf16", 2)
    k = k1.expand(S, 2, 32).contiguous()
    v = wl.randn((S, 2, 32), "bf16", 3)
    kc, vc = orc.new_cache(shape)
    orc.kv_append(shape, kc, vc, wl.to_bits(k), wl.to_bits(v), pb.cu_q, pb.ctx_before, pb.block_table)
    out, lse = orc.attn_prefill(shape, wl.to_bits(q), kc, vc, pb.cu_q, pb.ctx_before, pb.block_table)
    v64, q64, k64 = _np64(v), _np64(q), _np64(k1)
    run_mean = np.cumsum(v64, axis=0) / np.arange(1, S + 1)[:, None, None]
    for h in range(4):
        np.testing.assert_allclose(out[:, h, :], run_mean[:, h // 2, :], rtol=0, atol=1e-13)
        s = (q64[:, h, :] @ k64[0, h // 2, :]) / math.sqrt(32)
        np.testing.assert_allclose(lse[:, h], s + np.log(np.arange(1, S + 1)), rtol=0, atol=1e-12)


def test_weights_sum_to_one_and_reproduce_output():
    model = wl.ModelShape("p", 4, 2, 16, 1, "f32")
    pb, shape = _setup(model, [29, 18])
    T = pb.T
    q = wl.randn((T, 4, 16), "f32", 1, scale=3.0)
    k = wl.randn((T, 2, 16), "f32", 2); v = wl.randn((T, 2, 16), "f32", 3)
    kc, vc = orc.new_cache(shape)
    orc.kv_append(shape, kc, vc, wl.to_bits(k), wl.to_bits(v), pb.cu_q, pb.ctx_before, pb.block_table)
    pos = np.concatenate([np.arange(29), np.arange(18)]).astype(np.int32)
    out, lse, probs = orc.attn_rows(shape, wl.to_bits(q), kc, vc, pb.block_table, pb.cu_q,
                                    np.arange(T, dtype=np.int32), pos, want_probs=True)
    assert np.all(probs >= 0)
    np.testing.assert_allclose(probs.sum(-1), 1.0, rtol=0, atol=1e-12)
    v64 = _np64(v)
    for r in range(T):
        assert np.all(probs[r, :, pos[r] + 1:] == 0.0)   # nothing beyond the causal bound
        b = 0 if r < 29 else 1
        a = int(pb.cu_q[b])
        for h in range(4):
            ref = probs[r, h, : pos[r] + 1] @ v64[a: a + pos[r] + 1, h // 2, :]
            np.testing.assert_allclose(out[r, h], ref, rtol=0, atol=1e-13)


def test_invariant_under_physical_block_permutation():
    model = wl.ModelShape("perm", 4, 2, 32, 1, "bf16")
    q_len = [40, 7, 65]
    outs = []
    T = sum(q_len)
    q = wl.randn((T, 4, 32), "bf16", 1); k = wl.randn((T, 2, 32), "bf16", 2); v = wl.randn((T, 2, 32), "bf16", 3)
    for seed in (3, 4, 5):
        pb, shape = _setup(model, q_len, seed=seed)
        kc, vc = orc.new_cache(shape)
        orc.kv_append(shape, kc, vc, wl.to_bits(k), wl.to_bits(v), pb.cu_q, pb.ctx_before, pb.block_table)
        outs.append(orc.attn_prefill(shape, wl.to_bits(q), kc, vc, pb.cu_q, pb.ctx_before, pb.block_table))
        tables = pb.block_table
    assert not np.array_equal(tables, _setup(model, q_len, seed=3)[0].block_table)  # tables really differ
    for o, l in outs[1:]:
        assert np.array_equal(o, outs[0][0]) and np.array_equal(l, outs[0][1])


def test_append_places_rows_bit_exactly_and_leaves_holes():
    """Independent placement: for every token compute (block, slot) by hand and compare the
    whole pool, including sentinels in unwritten slots and unused blocks."""
    model = wl.ModelShape("ap", 2, 2, 8, 1, "bf16")
    q_len, cb = [19, 3, 0, 16], [5, 0, 7, 16]
    pb, shape = _setup(model, q_len, ctx_before=cb)
    T = pb.T
    k = wl.to_bits(wl.randn((T, 2, 8), "bf16", 2)); v = wl.to_bits(wl.randn((T, 2, 8), "bf16", 3))
    kc, vc = orc.new_cache(shape)
    exp_k, exp_v = kc.copy(), vc.copy()
    orc.kv_append(shape, kc, vc, k, v, pb.cu_q, pb.ctx_before, pb.block_table)
    written = np.zeros((pb.num_blocks, 16), dtype=bool)
    for b in range(4):
        for i in range(q_len[b]):
            p = cb[b] + i
            blk = pb.block_table[b, p // 16]
            exp_k[blk, :, p % 16, :] = k[pb.cu_q[b] + i]
            exp_v[blk, :, p % 16, :] = v[pb.cu_q[b] + i]
            written[blk, p % 16] = True
    assert np.array_equal(kc, exp_k) and np.array_equal(vc, exp_v)
    sentinel = 0x7FC1
    hole = ~written[:, None, :, None]   # broadcast over heads and elements of [blk, Hkv, slot, D]
    assert np.all((kc == sentinel) | ~hole) and np.all((vc == sentinel) | ~hole)
    assert np.all(kc[np.broadcast_to(hole, kc.shape)] == sentinel)
    assert written.sum() == T


def test_unwritten_slots_poison_the_result():
    """A read one slot past the context must be visible: sentinels are NaN."""
    model = wl.ModelShape("nan", 2, 1, 8, 1, "f32")
    pb, shape = _setup(model, [5])
    k = wl.to_bits(wl.randn((5, 1, 8), "f32", 2)); v = wl.to_bits(wl.randn((5, 1, 8), "f32", 3))
    q = wl.to_bits(wl.randn((1, 2, 8), "f32", 1))
    kc, vc = orc.new_cache(shape)
    orc.kv_append(shape, kc, vc, k, v, pb.cu_q, pb.ctx_before, pb.block_table)
    ok, _ = orc.attn_decode(shape, q, kc, vc, pb.block_table, [5])
    bad, _ = orc.attn_decode(shape, q, kc, vc, pb.block_table, [6])
    assert np.all(np.isfinite(ok)) and np.all(np.isnan(bad))


def test_decode_equals_last_prefill_row():
    model = wl.ModelShape("dl", 8, 2, 64, 1, "bf16")
    pb, shape = _setup(model, [33, 64])
    T = pb.T
    q = wl.randn((T, 8, 64), "bf16", 1); k = wl.randn((T, 2, 64), "bf16", 2); v = wl.randn((T, 2, 64), "bf16", 3)
    kc, vc = orc.new_cache(shape)
    orc.kv_append(shape, kc, vc, wl.to_bits(k), wl.to_bits(v), pb.cu_q, pb.ctx_before, pb.block_table)
    out_p, lse_p = orc.attn_prefill(shape, wl.to_bits(q), kc, vc, pb.cu_q, pb.ctx_before, pb.block_table)
    last = pb.cu_q[1:] - 1
    out_d, lse_d = orc.attn_decode(shape, wl.to_bits(q)[last], kc, vc, pb.block_table, pb.q_len)
    assert np.array_equal(out_d, out_p[last]) and np.array_equal(lse_d, lse_p[last])


def test_bf16_widening_is_exact():
    """Every bf16 bit pattern widens to the same double torch gives (NaNs aside)."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    t = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).double().numpy()
    shape = orc.Shape(1, 1, 8, 16, 1, orc.BF16)
    table = np.zeros((1, 1), dtype=np.int32)
    finite = np.isfinite(t)
    vals = bits[finite]
    ref = t[finite]
    # a single-token context returns V exactly: push every finite pattern through it, 8 at a time
    pad = (-len(vals)) % 8
    vals = np.concatenate([vals, np.zeros(pad, dtype=np.uint16)]); ref = np.concatenate([ref, np.zeros(pad)])
    q = np.zeros((1, 1, 8), dtype=np.uint16)
    for i in range(0, len(vals), 8 * 257):   # a spread sample keeps the test fast
        kc, vc = orc.new_cache(shape)
        row = vals[i:i + 8].reshape(1, 1, 8)
        orc.kv_append(shape, kc, vc, np.zeros_like(row), row, [0, 1], [0], table)
        out, _ = orc.attn_decode(shape, q, kc, vc, table, [1])
        assert np.array_equal(out[0, 0], ref[i:i + 8])


def test_errors_are_reported():
    shape = orc.Shape(2, 1, 8, 16, 2, orc.F32)
    kc, vc = orc.new_cache(shape)
    k = np.zeros((1, 1, 8), dtype=np.float32)
    with pytest.raises(ValueError):
        orc.kv_append(shape, kc, vc, k, k, [0, 1], [0], np.array([[5]], dtype=np.int32))   # block out of pool
    with pytest.raises(ValueError):
        orc.kv_append(shape, kc, vc, k, k, [0, 1], [16], np.array([[0]], dtype=np.int32))  # position beyond the table
    q = np.zeros((1, 2, 8), dtype=np.float32)
    with pytest.raises(ValueError):
        orc.attn_decode(shape, q, kc, vc, np.array([[0]], dtype=np.int32), [0])            # empty context
    with pytest.raises(ValueError):
        orc.attn_decode(shape, q, kc, vc, np.array([[-1]], dtype=np.int32), [1])           # unused table entry
