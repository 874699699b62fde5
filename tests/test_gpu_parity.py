"""GPU parity tests: the HIP library, called through the C ABI, against the fp64 CPU oracle
on the same seeded inputs, element by element.  Sizes here are ones the oracle finishes
in seconds but that span several tiles, splits and ragged tails."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2504_18154_amd import workloads as wl
from tests.parity_util import Layer, compare, compare_lse, dev_i32, say

pytestmark = pytest.mark.gpu

M30 = wl.ModelShape("30B-heads", 40, 8, 128, 1, "bf16")
M70 = wl.ModelShape("70B-heads", 64, 8, 128, 1, "bf16")


def _mk(model, q_len, ctx_before=None, seed=1, grow=0):
    pb = wl.prefill_batch(model, q_len, seed, ctx_before=ctx_before, grow=grow)
    layer = Layer(model, pb.num_blocks, max_batch=max(pb.B, 1), max_blocks_per_seq=pb.block_table.shape[1])
    return pb, layer


def _qkv(model, T, seed, qscale=1.0, vscale=1.0):
    q = wl.randn((T, model.Hq, model.D), model.dtype, seed, scale=qscale)
    k = wl.randn((T, model.Hkv, model.D), model.dtype, seed + 1)
    v = wl.randn((T, model.Hkv, model.D), model.dtype, seed + 2, scale=vscale)
    return q, k, v


def test_config1_tiny_padg_cycle_fp32():
    """Config 1: prefill-only batch (37 and 100 tokens) then 8 decode-only steps, fp32,
    full oracle at every step, cache compared bit for bit after every append."""
    say("config 1: tiny PaDG cycle fp32")
    pb = wl.config1_tiny()
    model = pb.model
    layer = Layer(model, pb.num_blocks, 2, pb.block_table.shape[1])
    q, k, v = _qkv(model, pb.T, wl.config_seed(1))
    layer.append(k, v, pb.cu_q, pb.ctx_before, pb.block_table)
    layer.assert_cache_bit_exact()
    out, lse = layer.prefill_gpu(q, pb.cu_q, pb.ctx_before, pb.block_table)
    ref, ref_lse = layer.prefill_oracle(q, pb.cu_q, pb.ctx_before, pb.block_table)
    compare("prefill", out, ref, "f32")
    compare_lse("prefill", lse, ref_lse, "f32", bf16_row_sum=True)
    ctx = pb.q_len.copy()
    ones = wl.cu_from_lengths([1, 1])
    for step in range(8):
        q, k, v = _qkv(model, 2, wl.config_seed(1) + 10 * (step + 1))
        layer.append(k, v, ones, ctx, pb.block_table)
        ctx = ctx + 1
        layer.assert_cache_bit_exact()
        out, lse = layer.decode_gpu(q, pb.block_table, ctx)
        ref, ref_lse = layer.decode_oracle(q, pb.block_table, ctx)
        compare(f"decode step {step}", out, ref, "f32")
        compare_lse(f"decode step {step}", lse, ref_lse, "f32")
    layer.close()


@pytest.mark.parametrize("model", [M30, M70], ids=["G5", "G8"])
def test_bf16_prefill_ragged_lengths(model):
    q_len = [1, 15, 16, 17, 127, 128, 129, 300, 0, 64, 513]
    say(f"bf16 prefill ragged {model.name} {q_len}")
    pb, layer = _mk(model, q_len, seed=5)
    q, k, v = _qkv(model, pb.T, 50)
    layer.append(k, v, pb.cu_q, pb.ctx_before, pb.block_table)
    layer.assert_cache_bit_exact()
    out, lse = layer.prefill_gpu(q, pb.cu_q, pb.ctx_before, pb.block_table)
    ref, ref_lse = layer.prefill_oracle(q, pb.cu_q, pb.ctx_before, pb.block_table)
    compare("prefill", out, ref, "bf16")
    compare_lse("prefill", lse, ref_lse, "bf16", bf16_row_sum=True)
    layer.close()


@pytest.mark.parametrize("heads", [(40, 8), (64, 8), (32, 2), (8, 2), (6, 6)], ids=["G5", "G8", "G16", "G4", "G1"])
def test_bf16_prefill_of_short_prompts_in_packed_tiles(heads):
    """Prompts that fit kTQ / G rows (25 new tokens for G = 5): the library packs the G query
    heads of a K/V head into one tile.  Lengths 0 .. P including both ends, with and without a cached prefix
    (then the packed rows sit behind hundreds of cached keys); a prompt that breaks the rule by one token and
    takes ordinary tiles beside packed ones; and sixty-three prompts of mixed lengths, one of them two tiles
    long.  The caller's bound on the lengths is exact, too small and generous in turn: it decides nothing."""
    model = wl.ModelShape("short", heads[0], heads[1], 128, 1, "bf16")
    G = heads[0] // heads[1]
    P = 128 // G
    rng = np.random.default_rng(77 + G)
    for name, new, prefix in (
            ("no prefix", np.r_[0, 1, P, P - 1, rng.integers(1, P + 1, size=37)], None),
            ("cached prefix", np.r_[P, 1, rng.integers(1, P + 1, size=10)], np.r_[300, 17, rng.integers(0, 400, size=10)]),
            ("one token too long", np.r_[3, P + 1, 5, min(P, 9)], None),
            ("short and longer prompts mixed", np.r_[rng.integers(1, 3 * P, size=60), 140, 1, P], np.r_[rng.integers(0, 90, size=60), 0, 5, 64])):
        new = new.astype(np.int32)
        prefix = np.zeros_like(new) if prefix is None else prefix.astype(np.int32)
        say(f"bf16 prefill of short prompts, G = {G} (P = {P}), {name}: new {new.tolist()}")
        pb, layer = _mk(model, np.maximum(prefix + new, 1), seed=80 + G)
        if prefix.sum() > 0:
            _, k1, v1 = _qkv(model, int(prefix.sum()), 800 + G)
            layer.append(k1, v1, wl.cu_from_lengths(prefix), np.zeros_like(prefix), pb.block_table)
        cu = wl.cu_from_lengths(new)
        q, k2, v2 = _qkv(model, int(new.sum()), 810 + G)
        layer.append(k2, v2, cu, prefix, pb.block_table)
        layer.assert_cache_bit_exact()
        ref, ref_lse = layer.prefill_oracle(q, cu, prefix, pb.block_table)
        for bound in (int(new.max()), min(P, int(new.max())), min(128, int(new.sum()))):   # exact, as small as packing needs, generous
            out, lse = layer.prefill_gpu(q, cu, prefix, pb.block_table, max_q_len=bound)
            compare(f"prefill, max_q_len = {bound}", out, ref, "bf16")
            compare_lse(f"prefill, max_q_len = {bound}", lse, ref_lse, "bf16", bf16_row_sum=True)
        layer.close()


def test_bf16_prefill_with_cached_prefix():
    """Second chunk of a prompt: queries sit at ctx_before + i and see the prefix too."""
    model = M30
    first, second = [70, 16, 200, 33], [90, 129, 1, 31]
    total = [a + b for a, b in zip(first, second)]
    say(f"bf16 prefill with prefix {first} + {second}")
    pb, layer = _mk(model, total, seed=6)
    cu1, cu2 = wl.cu_from_lengths(first), wl.cu_from_lengths(second)
    zero = np.zeros(4, dtype=np.int32)
    q1, k1, v1 = _qkv(model, int(cu1[-1]), 60)
    layer.append(k1, v1, cu1, zero, pb.block_table)
    q2, k2, v2 = _qkv(model, int(cu2[-1]), 70)
    cb = np.asarray(first, dtype=np.int32)
    layer.append(k2, v2, cu2, cb, pb.block_table)
    layer.assert_cache_bit_exact()
    out, lse = layer.prefill_gpu(q2, cu2, cb, pb.block_table)
    ref, ref_lse = layer.prefill_oracle(q2, cu2, cb, pb.block_table)
    compare("prefill chunk 2", out, ref, "bf16")
    compare_lse("prefill chunk 2", lse, ref_lse, "bf16", bf16_row_sum=True)
    layer.close()


DECODE_LENS = [1, 15, 16, 17, 63, 64, 65, 100, 513, 1000, 2047, 2048, 2049, 3000]


@pytest.mark.parametrize("model", [M30, M70], ids=["G5", "G8"])
def test_bf16_decode_split_plans(model):
    """Decode over ragged contexts with the automatic plan and forced split sizes
    (one split, many splits); every plan must meet the tolerance, the cache is shared."""
    from paper_2504_18154_amd import binding
    say(f"bf16 decode split plans {model.name}")
    pb, layer = _mk(model, DECODE_LENS, seed=7)
    T = pb.T
    _, k, v = _qkv(model, T, 80)
    layer.append(k, v, pb.cu_q, pb.ctx_before, pb.block_table)
    layer.assert_cache_bit_exact()
    B = pb.B
    q = wl.randn((B, model.Hq, model.D), "bf16", 81)
    ctx = pb.q_len
    ref, ref_lse = layer.decode_oracle(q, pb.block_table, ctx)
    outs = {}
    for split in (0, 64, 128, 448, 1024, 4096):
        layer.ctx.set_option(binding.OPT_DECODE_SPLIT_TOKENS, split)
        out, lse = layer.decode_gpu(q, pb.block_table, ctx)
        compare(f"decode split={split}", out, ref, "bf16")
        compare_lse(f"decode split={split}", lse, ref_lse, "bf16")
        out2, _ = layer.decode_gpu(q, pb.block_table, ctx)
        assert torch.equal(out.view(torch.int16), out2.view(torch.int16)), "decode is not run-to-run deterministic"
        outs[split] = out
    layer.close()


def test_bf16_multi_head_attention_no_kv_sharing():
    """52 query heads with a K/V head each (G = 1): the head shape of the multi-head model of the
    paper's evaluation (Section 4.1).  Prefill over ragged prompts, then decode steps on the grown
    contexts; decode arithmetic intensity is 1, the purest memory-bound case."""
    model = wl.ModelShape("mha", 52, 52, 128, 1, "bf16")
    q_len = [5, 130, 16, 257, 64, 1, 700]
    say(f"bf16 MHA (G = 1) prefill {q_len} then decode")
    pb, layer = _mk(model, q_len, seed=21, grow=3)
    q, k, v = _qkv(model, pb.T, 210)
    layer.append(k, v, pb.cu_q, pb.ctx_before, pb.block_table)
    layer.assert_cache_bit_exact()
    out, lse = layer.prefill_gpu(q, pb.cu_q, pb.ctx_before, pb.block_table)
    ref, ref_lse = layer.prefill_oracle(q, pb.cu_q, pb.ctx_before, pb.block_table)
    compare("MHA prefill", out, ref, "bf16")
    compare_lse("MHA prefill", lse, ref_lse, "bf16", bf16_row_sum=True)
    ctx = pb.q_len.copy()
    ones = wl.cu_from_lengths([1] * pb.B)
    for step in range(3):
        q, k, v = _qkv(model, pb.B, 220 + 10 * step)
        layer.append(k, v, ones, ctx, pb.block_table, max_new_len=1)
        ctx = ctx + 1
        out, lse = layer.decode_gpu(q, pb.block_table, ctx)
        ref, ref_lse = layer.decode_oracle(q, pb.block_table, ctx)
        compare(f"MHA decode step {step}", out, ref, "bf16")
        compare_lse(f"MHA decode step {step}", lse, ref_lse, "bf16")
    layer.assert_cache_bit_exact()
    layer.close()


def test_bf16_decode_adaptive_shares_small_and_ragged():
    """Per-XCD shares on launches that are too small to measure (shares must stay equal and
    results identical to the equal-share mode) and on ragged contexts over many calls."""
    from paper_2504_18154_amd import binding
    model = M30
    say("bf16 decode with per-XCD shares, ragged contexts")
    pb, layer = _mk(model, DECODE_LENS + [4000, 3500, 2222, 1234] * 6, seed=23)
    _, k, v = _qkv(model, pb.T, 230)
    layer.append(k, v, pb.cu_q, pb.ctx_before, pb.block_table)
    q = wl.randn((pb.B, model.Hq, model.D), "bf16", 231)
    ref, ref_lse = layer.decode_oracle(q, pb.block_table, pb.q_len)
    base, _ = layer.decode_gpu(q, pb.block_table, pb.q_len)
    layer.ctx.set_option(binding.OPT_DECODE_ADAPTIVE, 1)
    for call in range(20):
        out, lse = layer.decode_gpu(q, pb.block_table, pb.q_len)
        compare(f"adaptive call {call}", out, ref, "bf16")
        compare_lse(f"adaptive call {call}", lse, ref_lse, "bf16")
    layer.ctx.set_option(binding.OPT_DECODE_ADAPTIVE, 0)
    again, _ = layer.decode_gpu(q, pb.block_table, pb.q_len)
    assert torch.equal(base.view(torch.int16), again.view(torch.int16)), "equal-share mode is not reproducible"
    layer.close()


@pytest.mark.parametrize("hq,hkv", [(2, 1), (16, 1), (3, 3), (24, 6)], ids=["G2x1", "G16x1", "G1x3", "G4x6"])
def test_bf16_unusual_head_counts(hq, hkv):
    """Head counts that are not multiples of the XCD count, the largest supported group (16 query
    heads per K/V head) and a single K/V head: prefill (with a cached prefix on some sequences)
    and decode on the matrix-core path."""
    model = wl.ModelShape(f"h{hq}x{hkv}", hq, hkv, 128, 1, "bf16")
    first, second = [0, 40, 129, 0, 700, 16], [300, 1, 64, 65, 131, 500]
    say(f"bf16 {hq} query / {hkv} K/V heads: prefix {first} + new {second}")
    pb, layer = _mk(model, [a + b for a, b in zip(first, second)], seed=31, grow=2)
    cu1, cu2 = wl.cu_from_lengths(first), wl.cu_from_lengths(second)
    cb = np.asarray(first, dtype=np.int32)
    _, k1, v1 = _qkv(model, int(cu1[-1]), 310)
    layer.append(k1, v1, cu1, np.zeros(len(first), np.int32), pb.block_table)
    q2, k2, v2 = _qkv(model, int(cu2[-1]), 320)
    layer.append(k2, v2, cu2, cb, pb.block_table)
    layer.assert_cache_bit_exact()
    out, lse = layer.prefill_gpu(q2, cu2, cb, pb.block_table)
    ref, ref_lse = layer.prefill_oracle(q2, cu2, cb, pb.block_table)
    compare("prefill", out, ref, "bf16")
    compare_lse("prefill", lse, ref_lse, "bf16", bf16_row_sum=True)
    ctx = pb.q_len.copy()
    ones = wl.cu_from_lengths([1] * pb.B)
    for step in range(2):
        q, k, v = _qkv(model, pb.B, 330 + 10 * step)
        layer.append(k, v, ones, ctx, pb.block_table, max_new_len=1)
        ctx = ctx + 1
        out, lse = layer.decode_gpu(q, pb.block_table, ctx)
        ref, ref_lse = layer.decode_oracle(q, pb.block_table, ctx)
        compare(f"decode step {step}", out, ref, "bf16")
        compare_lse(f"decode step {step}", lse, ref_lse, "bf16")
    layer.close()


def test_bf16_large_batch_of_short_sequences():
    """1500 sequences of 0..70 tokens (the batch prefix sums take more than one entry per thread,
    most work items are a single key step, many sequences are empty in the prefill call), then a
    decode step over all of them."""
    model = wl.ModelShape("small-heads", 8, 2, 128, 1, "bf16")
    rng = np.random.default_rng(41)
    q_len = rng.integers(0, 71, size=1500)
    q_len[[0, 7, 1499]] = [0, 70, 0]
    say(f"bf16 batch of {len(q_len)} short sequences, {int(q_len.sum())} tokens")
    pb, layer = _mk(model, q_len, seed=42, grow=1)
    q, k, v = _qkv(model, pb.T, 410)
    layer.append(k, v, pb.cu_q, pb.ctx_before, pb.block_table)
    layer.assert_cache_bit_exact()
    out, lse = layer.prefill_gpu(q, pb.cu_q, pb.ctx_before, pb.block_table)
    ref, ref_lse = layer.prefill_oracle(q, pb.cu_q, pb.ctx_before, pb.block_table)
    compare("prefill", out, ref, "bf16")
    compare_lse("prefill", lse, ref_lse, "bf16", bf16_row_sum=True)
    ctx = pb.q_len + 1
    q, k, v = _qkv(model, pb.B, 420)
    layer.append(k, v, wl.cu_from_lengths([1] * pb.B), pb.q_len, pb.block_table, max_new_len=1)
    out, lse = layer.decode_gpu(q, pb.block_table, ctx)
    ref, ref_lse = layer.decode_oracle(q, pb.block_table, ctx)
    compare("decode", out, ref, "bf16")
    compare_lse("decode", lse, ref_lse, "bf16")
    layer.assert_cache_bit_exact()
    layer.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_append_at_the_largest_batch(dtype):
    """4096 sequences (the largest batch a context accepts) of 0..40 new tokens behind 0..20 cached
    ones: the append kernel's per-batch tables are at their largest; the cache is compared bit for bit."""
    model = wl.ModelShape("small-heads", 4, 2, 128, 1, dtype)
    rng = np.random.default_rng(43)
    first = rng.integers(0, 21, size=4096)
    second = rng.integers(0, 41, size=4096)
    second[[0, 4095]] = [40, 33]
    say(f"{dtype} append at batch 4096: {int(first.sum())} then {int(second.sum())} tokens")
    pb, layer = _mk(model, first + second, seed=44)
    cu1, cu2 = wl.cu_from_lengths(first), wl.cu_from_lengths(second)
    _, k1, v1 = _qkv(model, int(cu1[-1]), 430)
    layer.append(k1, v1, cu1, np.zeros(4096, np.int32), pb.block_table)
    layer.assert_cache_bit_exact()
    _, k2, v2 = _qkv(model, int(cu2[-1]), 440)
    layer.append(k2, v2, cu2, first.astype(np.int32), pb.block_table)
    layer.assert_cache_bit_exact()
    layer.close()


def test_bf16_decode_of_hundreds_of_short_sequences():
    """800 sequences of 1..150 tokens with 8 K/V heads: more than six (sequence, head) pieces per
    wavefront, so the block pipeline crosses piece boundaries all the time, the results leave through the
    LDS buffer in several batches, and nearly every (sequence, head) is written in final form by the
    decode kernel while the merge handles the few that a chunk boundary cuts.  Equal and measured per-XCD
    shares."""
    from paper_2504_18154_amd import binding
    model = M30
    rng = np.random.default_rng(47)
    lens = rng.integers(1, 151, size=800)
    lens[[0, 1, 799]] = [1, 300, 16]
    say(f"bf16 decode of {len(lens)} short sequences, {int(lens.sum())} tokens")
    pb, layer = _mk(model, lens, seed=48)
    _, k, v = _qkv(model, pb.T, 470)
    layer.append(k, v, pb.cu_q, pb.ctx_before, pb.block_table)
    layer.assert_cache_bit_exact()
    q = wl.randn((pb.B, model.Hq, model.D), "bf16", 471)
    ref, ref_lse = layer.decode_oracle(q, pb.block_table, pb.q_len)
    out, lse = layer.decode_gpu(q, pb.block_table, pb.q_len)
    compare("decode, equal shares", out, ref, "bf16")
    compare_lse("decode, equal shares", lse, ref_lse, "bf16")
    layer.ctx.set_option(binding.OPT_DECODE_ADAPTIVE, 1)
    for call in range(4):
        out, lse = layer.decode_gpu(q, pb.block_table, pb.q_len)
        compare(f"decode, measured shares, call {call}", out, ref, "bf16")
        compare_lse(f"decode, measured shares, call {call}", lse, ref_lse, "bf16")
    layer.close()


def test_bf16_decode_random_batches():
    """Sixteen seeded random decode batches: group sizes 1..16, 1..8 K/V heads, 1..47 sequences whose lengths
    mix a few tokens, a few hundred, about a thousand and up to five thousand, automatic and forced splits,
    equal and measured shares, the plain call and the fused append + decode call (the last token of every
    sequence wiped from the cache and handed in as the new one)."""
    from paper_2504_18154_amd import binding
    rng = np.random.default_rng(2025)
    for case in range(16):
        Hkv, G = int(rng.choice([1, 2, 8])), int(rng.choice([1, 4, 5, 8, 16]))
        model = wl.ModelShape("random", Hkv * G, Hkv, 128, 1, "bf16")
        B = int(rng.integers(1, 48))
        kind = rng.integers(0, 4, size=B)
        lens = np.where(kind == 0, rng.integers(1, 40, size=B),
                        np.where(kind == 1, rng.integers(40, 700, size=B),
                                 np.where(kind == 2, rng.integers(1000, 1100, size=B),
                                          rng.integers(1, 5000, size=B)))).astype(np.int32)
        while int(lens.sum()) * model.Hq > 2_000_000:   # keeps the oracle's share of the test short
            lens = np.maximum(lens // 2, 1)
        split, adaptive, fused = int(rng.choice([0, 0, 64, 256, 1024])), int(rng.integers(0, 2)), int(rng.integers(0, 2))
        say(f"random decode batch {case}: Hq {model.Hq} Hkv {Hkv} B {B} tokens {int(lens.sum())} max {int(lens.max())} "
            f"split {split} measured shares {adaptive} fused {fused}")
        pb, layer = _mk(model, lens, seed=900 + case)
        _, k, v = _qkv(model, pb.T, 910 + 3 * case)
        layer.append(k, v, pb.cu_q, pb.ctx_before, pb.block_table)
        layer.ctx.set_option(binding.OPT_DECODE_SPLIT_TOKENS, split)
        layer.ctx.set_option(binding.OPT_DECODE_ADAPTIVE, adaptive)
        q = wl.randn((B, model.Hq, model.D), "bf16", 990 + case)
        ref, ref_lse = layer.decode_oracle(q, pb.block_table, lens)
        table, ctx_dev = dev_i32(pb.block_table), dev_i32(lens)
        for rep in range(3 if adaptive else 1):
            if fused:
                last = torch.as_tensor(pb.cu_q[1:] - 1, dtype=torch.int64)
                kn, vn = k[last].contiguous().cuda(), v[last].contiguous().cuda()
                wipe = torch.full_like(kn, float("nan"))
                layer.ctx.kv_append(layer.kc, layer.vc, wipe, wipe, dev_i32(wl.cu_from_lengths([1] * B)),
                                    dev_i32(lens - 1), table, max_new_len=1)
                out = torch.full((B, model.Hq, model.D), float("nan"), dtype=torch.bfloat16, device="cuda")
                lse = torch.full((B, model.Hq), float("nan"), dtype=torch.float32, device="cuda")
                layer.ctx.attn_decode_append(q.cuda(), kn, vn, layer.kc, layer.vc, table, ctx_dev, out,
                                             int(lens.max()), lse)
                torch.cuda.synchronize()
                layer.assert_cache_bit_exact()
            else:
                out, lse = layer.decode_gpu(q, pb.block_table, lens)
            compare(f"batch {case} call {rep}", out, ref, "bf16")
            compare_lse(f"batch {case} call {rep}", lse, ref_lse, "bf16")
        layer.close()


def test_bf16_decode_passes_over_sequences_without_tokens():
    """A context length of zero is not a valid decode input (the step's own token counts), but a batch that
    holds one - first, last or in the middle, alone or several in a row - must not cost the other sequences
    their results: their rows are held to the oracle, the empty sequences' rows are left alone."""
    model = M30
    lens = np.asarray([0, 700, 0, 0, 33, 257, 0, 1500, 16, 0], dtype=np.int32)
    say(f"bf16 decode with empty sequences in the batch {lens.tolist()}")
    pb, layer = _mk(model, np.maximum(lens, 1), seed=51)
    _, k, v = _qkv(model, int(lens.sum()), 510)
    layer.append(k, v, wl.cu_from_lengths(lens), np.zeros(len(lens), np.int32), pb.block_table)
    q = wl.randn((len(lens), model.Hq, model.D), "bf16", 511)
    live = np.flatnonzero(lens > 0)
    ref, ref_lse = layer.decode_oracle(q[live], pb.block_table[live], lens[live])
    from paper_2504_18154_amd import binding
    for split in (0, 64):
        layer.ctx.set_option(binding.OPT_DECODE_SPLIT_TOKENS, split)
        out, lse = layer.decode_gpu(q, pb.block_table, lens, max_ctx_len=int(lens.max()))
        compare(f"decode split={split}, rows of the non-empty sequences", out, ref, "bf16", rows=live)
        compare_lse(f"decode split={split}", lse[torch.as_tensor(live, device=lse.device)], ref_lse, "bf16")
    layer.close()


@pytest.mark.parametrize("shape", ["bf16-G5", "bf16-mha", "bf16-many-short", "bf16-forced-split", "f32-plain"])
def test_decode_with_the_append_fused_in(shape):
    """ecoserve_attn_decode_append against the two separate calls on a copy of the same cache: cache and
    output must agree bit for bit, step after step (positions crossing block boundaries, contexts that end
    on a block boundary, a sequence whose first token is the appended one), and against the oracle."""
    from paper_2504_18154_amd import binding
    if shape == "f32-plain":
        model, lens = wl.ModelShape("small-f32", 4, 2, 64, 1, "f32"), [0, 15, 16, 17, 100]
    elif shape == "bf16-mha":
        model, lens = wl.ModelShape("mha", 6, 6, 128, 1, "bf16"), [0, 15, 16, 31, 32, 700]
    elif shape == "bf16-many-short":
        model, lens = M30, list(np.random.default_rng(49).integers(0, 100, size=800))   # many pieces per wavefront
    elif shape == "bf16-forced-split":      # fixed chunks of 256 tokens: the other merge kernel carries the stores
        model, lens = M30, [0, 1, 15, 16, 255, 256, 600, 2047]
    else:
        model, lens = M30, [0, 1, 14, 15, 16, 17, 255, 256, 1000, 2047, 3000]
    steps = 3
    say(f"fused append + decode, {shape}: {len(lens)} sequences, {steps} steps")
    lens = np.asarray(lens, dtype=np.int32)
    pb, layer = _mk(model, lens + steps, seed=62)
    if shape == "bf16-forced-split":
        layer.ctx.set_option(binding.OPT_DECODE_SPLIT_TOKENS, 256)
    table = dev_i32(pb.block_table)
    if lens.sum() > 0:
        _, k, v = _qkv(model, int(lens.sum()), 620)
        layer.append(k, v, wl.cu_from_lengths(lens), np.zeros(len(lens), np.int32), pb.block_table)
    kc2, vc2 = layer.kc.clone(), layer.vc.clone()     # the fused call works on its own copy
    B = len(lens)
    ones = dev_i32(wl.cu_from_lengths([1] * B))
    ctx = lens.copy()
    for step in range(steps):
        rows = wl.randn((B, (model.Hq + 2 * model.Hkv) * model.D), model.dtype, 630 + step, device="cuda")
        body = rows.unflatten(1, (model.Hq + 2 * model.Hkv, model.D))
        q, kn, vn = body[:, :model.Hq], body[:, model.Hq:model.Hq + model.Hkv], body[:, model.Hq + model.Hkv:]
        # separate calls (and the oracle's cache) ...
        layer.ctx.kv_append_strided(layer.kc, layer.vc, kn, vn, ones, dev_i32(ctx), table, max_new_len=1)
        orc.kv_append(layer.shape, layer.okc, layer.ovc, wl.to_bits(kn), wl.to_bits(vn), wl.cu_from_lengths([1] * B),
                      ctx, pb.block_table)
        ctx = ctx + 1
        want = torch.full((B, model.Hq, model.D), float("nan"), dtype=q.dtype, device="cuda")
        want_lse = torch.full((B, model.Hq), float("nan"), dtype=torch.float32, device="cuda")
        layer.ctx.attn_decode_strided(q, layer.kc, layer.vc, table, dev_i32(ctx), want, int(ctx.max()), want_lse)
        # ... against the fused call
        out, lse = torch.full_like(want, float("nan")), torch.full_like(want_lse, float("nan"))
        layer.ctx.attn_decode_append(q, kn, vn, kc2, vc2, table, dev_i32(ctx), out, int(ctx.max()), lse)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.uint8), want.view(torch.uint8)), f"step {step}: outputs differ"
        assert torch.equal(lse, want_lse), f"step {step}: log-sum-exp differs"
        assert torch.equal(kc2.view(torch.uint8), layer.kc.view(torch.uint8)), f"step {step}: K pools differ"
        assert torch.equal(vc2.view(torch.uint8), layer.vc.view(torch.uint8)), f"step {step}: V pools differ"
        layer.assert_cache_bit_exact()
        ref, ref_lse = layer.decode_oracle(q, pb.block_table, ctx)
        compare(f"fused decode step {step}", out, ref, model.dtype)
        compare_lse(f"fused decode step {step}", lse, ref_lse, model.dtype)
    layer.close()


def test_bf16_short_chunk_after_long_prefix():
    """A few new tokens behind thousands of cached ones (one query tile, many key steps) next to a
    long new prompt: the work items differ by two orders of magnitude."""
    model = M30
    first, second = [3001, 0, 4090, 777], [5, 1200, 3, 64]
    say(f"bf16 prefill: prefix {first} + new {second}")
    pb, layer = _mk(model, [a + b for a, b in zip(first, second)], seed=51)
    cu1, cu2 = wl.cu_from_lengths(first), wl.cu_from_lengths(second)
    cb = np.asarray(first, dtype=np.int32)
    _, k1, v1 = _qkv(model, int(cu1[-1]), 510)
    layer.append(k1, v1, cu1, np.zeros(4, np.int32), pb.block_table)
    q2, k2, v2 = _qkv(model, int(cu2[-1]), 520)
    layer.append(k2, v2, cu2, cb, pb.block_table)
    layer.assert_cache_bit_exact()
    out, lse = layer.prefill_gpu(q2, cu2, cb, pb.block_table)
    ref, ref_lse = layer.prefill_oracle(q2, cu2, cb, pb.block_table)
    compare("prefill", out, ref, "bf16")
    compare_lse("prefill", lse, ref_lse, "bf16", bf16_row_sum=True)
    layer.close()


@pytest.mark.parametrize("heads, n_seq, lo, hi, with_prefix", [((24, 6), 64, 200, 1200, False), ((40, 8), 40, 300, 1500, True),
                                                               ((16, 1), 24, 800, 2200, False)])
def test_bf16_prefill_results_do_not_depend_on_the_queue_shares(heads, n_seq, lo, hi, with_prefix):
    """Batches large enough (3072 work items or more) for the prefill kernel to move its queues' shares of the
    items with the busy times of the launch before: seven launches on one batch, every one bit for bit the first
    (whose shares are equal), with and without cached prefixes, for group sizes 4, 5 and 16 (the last with a
    single K/V head: all queues then share one head's K/V); sampled rows of the first against the oracle."""
    model = wl.ModelShape(f"h{heads[0]}x{heads[1]}", heads[0], heads[1], 128, 1, "bf16")
    rng = wl.rng_for(700 + heads[0])
    q_len = rng.integers(lo, hi, n_seq).astype(np.int32)
    ctx_before = rng.integers(0, 700, n_seq).astype(np.int32) if with_prefix else None
    say(f"bf16 prefill, queue shares: {n_seq} prompts of {lo}..{hi} tokens, heads {heads}, prefixes {with_prefix}")
    pb, layer = _mk(model, q_len, ctx_before=ctx_before, seed=71)
    if with_prefix:
        _, kp, vp = _qkv(model, int(pb.ctx_before.sum()), 720)
        layer.append(kp, vp, wl.cu_from_lengths(pb.ctx_before), np.zeros(pb.B, np.int32), pb.block_table)
    q, k, v = _qkv(model, pb.T, 710)
    layer.append(k, v, pb.cu_q, pb.ctx_before, pb.block_table)
    first, first_lse = layer.prefill_gpu(q, pb.cu_q, pb.ctx_before, pb.block_table)
    assert layer.ctx.debug_prefill_queue_shares() == [1.0] * 8
    moved = False
    for launch in range(1, 7):
        out, lse = layer.prefill_gpu(q, pb.cu_q, pb.ctx_before, pb.block_table)
        shares = layer.ctx.debug_prefill_queue_shares()
        moved = moved or any(abs(x - 1.0) > 1e-4 for x in shares)
        assert torch.equal(out.view(torch.int16), first.view(torch.int16)), f"launch {launch}: shares {shares}"
        assert torch.equal(lse.view(torch.int32), first_lse.view(torch.int32)), f"launch {launch}: lse, shares {shares}"
    say("  shares of the last launch: " + " ".join(f"{x:.3f}" for x in shares))
    assert moved, "the shares never left 1.0: the batch is too small for the measured path"
    # a few hundred rows of the first launch against the oracle
    rows = np.sort(wl.rng_for(73).choice(pb.T, size=min(pb.T, 300), replace=False)).astype(np.int64)
    seq = np.searchsorted(pb.cu_q, rows, side="right") - 1
    pos = pb.ctx_before[seq] + (rows - pb.cu_q[seq])
    start = np.searchsorted(seq, np.arange(pb.B + 1), side="left").astype(np.int32)  # rows of sequence b: start[b] .. start[b+1]-1
    ref, ref_lse = orc.attn_rows(layer.shape, wl.to_bits(q), layer.okc, layer.ovc, pb.block_table, start,
                                 rows.astype(np.int32), pos.astype(np.int32))
    compare("prefill with queue shares (sampled rows)", first, ref, "bf16", rows=rows)
    compare_lse("prefill with queue shares (sampled rows)", first_lse, ref_lse, "bf16", rows=rows, bf16_row_sum=True)
    layer.close()


def test_bf16_prefill_reuses_the_tile_list_across_layers():
    """Several 'layers' (different caches and queries, the same batch arrays) with the tile list
    built once and reused, against the oracle and bit for bit against the mode that rebuilds it;
    then another batch through the same context, which must get a list of its own."""
    from paper_2504_18154_amd import binding
    model = M30
    q_len = [700, 130, 1, 257, 0, 64, 2100]
    say(f"bf16 prefill, tile list reused over 3 layers: {q_len}")
    pb, layer = _mk(model, q_len, seed=61)
    cu, cb, bt = dev_i32(pb.cu_q), dev_i32(pb.ctx_before), dev_i32(pb.block_table)
    layers = []
    for l in range(3):
        q, k, v = _qkv(model, pb.T, 610 + 10 * l)
        kc, vc = layer.ctx.new_cache()
        layer.ctx.kv_append(kc, vc, k.cuda(), v.cuda(), cu, cb, bt)
        layers.append((q.cuda(), kc, vc))
    # layer 0 also lives in the Layer object, for the oracle
    q0, k0, v0 = _qkv(model, pb.T, 610)
    layer.append(k0, v0, pb.cu_q, pb.ctx_before, pb.block_table)
    ref, ref_lse = layer.prefill_oracle(q0, pb.cu_q, pb.ctx_before, pb.block_table)

    def run_all():
        outs = []
        for qd, kc, vc in layers:
            out = torch.full_like(qd, float("nan"))
            lse = torch.full(qd.shape[:2], float("nan"), dtype=torch.float32, device="cuda")
            layer.ctx.attn_prefill(qd, kc, vc, cu, cb, bt, out, lse, max_q_len=int(pb.q_len.max()))
            outs.append((out, lse))
        torch.cuda.synchronize()
        return outs

    fresh = run_all()
    layer.ctx.set_option(binding.OPT_PREFILL_REUSE_PLAN, 1)
    for rep in range(2):
        reused = run_all()
        for (a, al), (b, bl) in zip(fresh, reused):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16)) and torch.equal(al, bl), "reused tile list changed the result"
    compare("layer 0 with reused list", reused[0][0], ref, "bf16")
    compare_lse("layer 0 with reused list", reused[0][1], ref_lse, "bf16", bf16_row_sum=True)
    # the same batch through other arrays: a list of its own, same result
    cu2, cb2, bt2 = cu.clone(), cb.clone(), bt.clone()
    qd, kc, vc = layers[1]
    out = torch.full_like(qd, float("nan"))
    layer.ctx.attn_prefill(qd, kc, vc, cu2, cb2, bt2, out, max_q_len=int(pb.q_len.max()))
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), fresh[1][0].view(torch.int16))
    # the same arrays but one sequence fewer: B and T differ, so the list is rebuilt
    Bs, Ts = pb.B - 1, int(pb.cu_q[pb.B - 1])
    qd, kc, vc = layers[0]
    out = torch.full((Ts,) + tuple(qd.shape[1:]), float("nan"), dtype=qd.dtype, device="cuda")
    lse = torch.full((Ts, model.Hq), float("nan"), dtype=torch.float32, device="cuda")
    layer.ctx.attn_prefill(qd[:Ts], kc, vc, cu[:Bs + 1], cb[:Bs], bt, out, lse, max_q_len=int(pb.q_len[:Bs].max()))
    torch.cuda.synchronize()
    ref_s, ref_s_lse = layer.prefill_oracle(q0[:Ts], pb.cu_q[:Bs + 1], pb.ctx_before[:Bs], pb.block_table[:Bs])
    compare("one sequence fewer", out, ref_s, "bf16")
    compare_lse("one sequence fewer", lse, ref_s_lse, "bf16", bf16_row_sum=True)
    layer.close()


@pytest.mark.parametrize("seed", [101, 102, 103, 104, 105, 106])
def test_bf16_seeded_random_batches(seed):
    """Seeded random shapes: head counts, batch size, prefixes, prompt lengths (zeros, one token,
    around the 16/64/128 boundaries, a few long ones), then two decode steps with per-XCD shares
    on and off.  Everything against the oracle."""
    from paper_2504_18154_amd import binding
    rng = np.random.default_rng(seed)
    hkv = int(rng.choice([1, 2, 4, 8]))
    G = int(rng.choice([1, 2, 4, 5, 8]))
    model = wl.ModelShape(f"rnd{seed}", hkv * G, hkv, 128, 1, "bf16")
    B = int(rng.integers(1, 24))
    pool = np.array([0, 1, 2, 15, 16, 17, 63, 64, 65, 127, 128, 129, 191, 200, 255, 256, 257, 600, 1100])
    first = rng.choice(pool, size=B) * (rng.random(B) < 0.4)
    second = rng.choice(pool, size=B)
    first, second = first.astype(np.int64), second.astype(np.int64)
    second[rng.integers(0, B)] = max(1, int(second.max()))      # at least one non-empty sequence
    say(f"seed {seed}: {model.Hq}/{model.Hkv} heads, B={B}, prefix {first.tolist()}, new {second.tolist()}")
    pb, layer = _mk(model, first + second, seed=seed, grow=2)
    cu1, cu2 = wl.cu_from_lengths(first), wl.cu_from_lengths(second)
    cb = first.astype(np.int32)
    if int(cu1[-1]) > 0:
        _, k1, v1 = _qkv(model, int(cu1[-1]), seed * 10)
        layer.append(k1, v1, cu1, np.zeros(B, np.int32), pb.block_table)
    q2, k2, v2 = _qkv(model, int(cu2[-1]), seed * 10 + 3)
    layer.append(k2, v2, cu2, cb, pb.block_table)
    layer.assert_cache_bit_exact()
    out, lse = layer.prefill_gpu(q2, cu2, cb, pb.block_table)
    ref, ref_lse = layer.prefill_oracle(q2, cu2, cb, pb.block_table)
    compare("prefill", out, ref, "bf16")
    compare_lse("prefill", lse, ref_lse, "bf16", bf16_row_sum=True)
    ctx = (first + second).astype(np.int32)
    ones = wl.cu_from_lengths([1] * B)
    for step in range(2):
        q, k, v = _qkv(model, B, seed * 10 + 6 + step)
        layer.append(k, v, ones, ctx, pb.block_table, max_new_len=1)
        ctx = ctx + 1
        layer.ctx.set_option(binding.OPT_DECODE_ADAPTIVE, step)
        out, lse = layer.decode_gpu(q, pb.block_table, ctx)
        ref, ref_lse = layer.decode_oracle(q, pb.block_table, ctx)
        compare(f"decode step {step}", out, ref, "bf16")
        compare_lse(f"decode step {step}", lse, ref_lse, "bf16")
    layer.assert_cache_bit_exact()
    layer.close()


def test_bf16_decode_after_growth_steps():
    """Decode-only phase: several steps, each appending one token per sequence (crossing
    block boundaries) before attending."""
    model = M30
    lens = [14, 15, 16, 31, 47, 250, 1023]
    say(f"bf16 decode growth {lens}")
    pb, layer = _mk(model, lens, seed=8, grow=4)
    _, k, v = _qkv(model, pb.T, 90)
    layer.append(k, v, pb.cu_q, pb.ctx_before, pb.block_table)
    ctx = pb.q_len.copy()
    ones = wl.cu_from_lengths([1] * pb.B)
    for step in range(4):
        q, k, v = _qkv(model, pb.B, 100 + 10 * step)
        layer.append(k, v, ones, ctx, pb.block_table, max_new_len=1)
        ctx = ctx + 1
        layer.assert_cache_bit_exact()
        out, lse = layer.decode_gpu(q, pb.block_table, ctx)
        ref, ref_lse = layer.decode_oracle(q, pb.block_table, ctx)
        compare(f"decode step {step}", out, ref, "bf16")
        compare_lse(f"decode step {step}", lse, ref_lse, "bf16")
    layer.close()


@pytest.mark.parametrize("model", [M30, wl.ModelShape("d64", 8, 2, 64, 1, "bf16"),
                                   wl.ModelShape("f32-d128", 6, 3, 128, 1, "f32")], ids=["bf16-d128", "bf16-d64", "f32-d128"])
def test_plain_kernels(model):
    """The plain (non matrix-core) kernels on shapes the fast path also/never covers."""
    from paper_2504_18154_amd import binding
    lens = [1, 17, 64, 130, 333]
    say(f"plain kernels {model.name}")
    pb, layer = _mk(model, lens, seed=9)
    layer.ctx.set_option(binding.OPT_FORCE_PLAIN, 1)
    q, k, v = _qkv(model, pb.T, 110)
    layer.append(k, v, pb.cu_q, pb.ctx_before, pb.block_table)
    layer.assert_cache_bit_exact()
    out, lse = layer.prefill_gpu(q, pb.cu_q, pb.ctx_before, pb.block_table)
    ref, ref_lse = layer.prefill_oracle(q, pb.cu_q, pb.ctx_before, pb.block_table)
    compare("prefill", out, ref, model.dtype)
    compare_lse("prefill", lse, ref_lse, model.dtype)   # (the plain kernels sum the weights in fp32)
    qd = wl.randn((pb.B, model.Hq, model.D), model.dtype, 111)
    ref, ref_lse = layer.decode_oracle(qd, pb.block_table, pb.q_len)
    for split in (0, 64, 4096):
        layer.ctx.set_option(binding.OPT_DECODE_SPLIT_TOKENS, split)
        out, lse = layer.decode_gpu(qd, pb.block_table, pb.q_len)
        compare(f"decode split={split}", out, ref, model.dtype)
        compare_lse(f"decode split={split}", lse, ref_lse, model.dtype)
    layer.close()


@pytest.mark.parametrize("vscale", [0.25, 1.0], ids=["V-quarter-scale", "V-full-scale"])
def test_bf16_peaky_softmax(vscale):
    """Queries scaled x8: near one-hot weights exercise max tracking and rescaling.  With V
    scaled x0.25 every output stays below 2, where a bf16 spacing is under the max-abs bound, so
    the stated 1e-2 holds for every element.  With V at full scale an output is close to one V
    entry, thousands of them are 2 or larger, and those are held to half a bf16 spacing plus
    2^-9 |o| (see compare): the adversarial case for that bound."""
    model = M30
    lens = [200, 1000, 77]
    say(f"bf16 peaky softmax, V x {vscale}")
    pb, layer = _mk(model, lens, seed=10)
    q, k, v = _qkv(model, pb.T, 120, qscale=8.0, vscale=vscale)
    layer.append(k, v, pb.cu_q, pb.ctx_before, pb.block_table)
    out, lse = layer.prefill_gpu(q, pb.cu_q, pb.ctx_before, pb.block_table)
    ref, ref_lse = layer.prefill_oracle(q, pb.cu_q, pb.ctx_before, pb.block_table)
    compare("prefill", out, ref, "bf16")
    compare_lse("prefill", lse, ref_lse, "bf16", bf16_row_sum=True)
    last = pb.cu_q[1:] - 1
    qd = q[torch.as_tensor(last, dtype=torch.long)]
    out_d, lse_d = layer.decode_gpu(qd, pb.block_table, pb.q_len)
    compare("decode", out_d, ref[last], "bf16")
    compare_lse("decode", lse_d, ref_lse[last], "bf16")
    layer.close()


def test_single_token_context_is_exact():
    """L = 1: the only weight is 1, so the output must equal V bit for bit (both kernels)."""
    model = M70
    say("single-token contexts")
    pb, layer = _mk(model, [1] * 5, seed=11)
    q, k, v = _qkv(model, 5, 130, qscale=4.0)
    layer.append(k, v, pb.cu_q, pb.ctx_before, pb.block_table)
    expect = v.cuda().repeat_interleave(model.G, dim=1).view(torch.int16)
    out_d, lse = layer.decode_gpu(q, pb.block_table, pb.q_len)
    out_p, _ = layer.prefill_gpu(q, pb.cu_q, pb.ctx_before, pb.block_table)
    assert torch.equal(out_d.view(torch.int16), expect)
    assert torch.equal(out_p.view(torch.int16), expect)
    layer.close()


def test_unwritten_slots_and_unused_blocks_are_never_read_or_written():
    """Pools start as NaN sentinels.  Outputs must be finite (no stray read reaches them)
    and every unaddressed slot must keep its sentinel (covered by the whole-pool compare)."""
    model = M30
    lens = [3, 18, 50, 129, 1000]
    say("poison test")
    pb, layer = _mk(model, lens, seed=12, grow=20)   # spare table entries stay -1
    q, k, v = _qkv(model, pb.T, 140)
    layer.append(k, v, pb.cu_q, pb.ctx_before, pb.block_table)
    layer.assert_cache_bit_exact()
    out, _ = layer.prefill_gpu(q, pb.cu_q, pb.ctx_before, pb.block_table)
    assert torch.isfinite(out.float()).all()
    qd = wl.randn((pb.B, model.Hq, model.D), "bf16", 141)
    out_d, _ = layer.decode_gpu(qd, pb.block_table, pb.q_len)
    assert torch.isfinite(out_d.float()).all()
    ref, _ = layer.decode_oracle(qd, pb.block_table, pb.q_len)
    compare("decode", out_d, ref, "bf16")
    layer.close()


def test_empty_batches_and_host_side_errors():
    from paper_2504_18154_amd import binding
    model = M30
    say("empty batches / error codes")
    pb, layer = _mk(model, [40, 0, 7], seed=13)
    c = layer.ctx
    q, k, v = _qkv(model, pb.T, 150)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    cu, cb, bt = dev_i32(pb.cu_q), dev_i32(pb.ctx_before), dev_i32(pb.block_table)
    # T == 0 and B == 0 are no-ops
    empty = torch.empty((0, model.Hkv, model.D), dtype=torch.bfloat16, device="cuda")
    c.kv_append(layer.kc, layer.vc, empty, empty, cu, cb, bt)
    c.attn_decode(qd[:0], layer.kc, layer.vc, bt, cb[:0], qd[:0], 1)
    # batch larger than the context was created for
    with pytest.raises(binding.EcoserveError) as e:
        big = dev_i32(np.zeros(8))
        c.attn_decode(qd[:8], layer.kc, layer.vc, bt, big, qd[:8].clone(), 16)
    assert e.value.status == binding.EINVAL
    # max_ctx_len beyond the block table
    with pytest.raises(binding.EcoserveError) as e:
        c.attn_decode(qd[:3], layer.kc, layer.vc, bt, cb, qd[:3].clone(), 16 * pb.block_table.shape[1] + 1)
    assert e.value.status == binding.EINVAL
    # misaligned pointer
    with pytest.raises(binding.EcoserveError) as e:
        mis = torch.empty(qd.numel() + 8, dtype=torch.bfloat16, device="cuda")[1:1 + qd.numel()].view_as(qd)
        c.attn_prefill(mis, layer.kc, layer.vc, cu, cb, bt, torch.empty_like(qd))
    assert e.value.status == binding.EINVAL
    # more new tokens than the pool holds: the prefill tile list has no room (checked before any launch)
    with pytest.raises(binding.EcoserveError) as e:
        T_big = 128 * (pb.num_blocks // 8 + 3 + 1)
        huge = torch.empty((T_big, model.Hq, model.D), dtype=torch.bfloat16, device="cuda")
        c.attn_prefill(huge, layer.kc, layer.vc, cu, cb, bt, torch.empty_like(huge), max_q_len=T_big)
    assert e.value.status == binding.EINVAL
    # device-resident contents: the debug validator sees what the hot calls do not check
    total = dev_i32(pb.q_len)
    assert c.debug_validate(cu, total, bt) == binding.OK
    bad = pb.block_table.copy(); bad[0, 1] = pb.num_blocks
    assert c.debug_validate(cu, total, dev_i32(bad)) == binding.ECONTENT
    dup = pb.block_table.copy(); dup[2, 0] = dup[0, 0]
    assert c.debug_validate(cu, total, dev_i32(dup)) == binding.ECONTENT
    assert c.debug_validate(None, dev_i32([40, 0, 7]), bt) == binding.ECONTENT   # decode needs ctx_len >= 1
    layer.close()


@pytest.mark.parametrize("dtype,pad", [("bf16", 0), ("f32", 0), ("bf16", 24)])
def test_fused_projection_rows_are_read_in_place(dtype, pad):
    """Q, K and V as slices of one row [Hq + 2 Hkv (+ padding)][D] per token, the shape in which a fused
    projection (Eq. 1) leaves them: the strided calls read them where they are.  Append bit-exact, prefill
    and decode against the oracle and bit-identical to the packed calls on copies of the same slices; a
    prefix chunk first so that the second append starts inside a block."""
    from paper_2504_18154_amd import binding
    model = M30 if dtype == "bf16" else wl.ModelShape("small-f32", 4, 2, 64, 1, "f32")
    Hq, Hkv, D = model.Hq, model.Hkv, model.D
    first, second = [70, 0, 203, 5], [130, 257, 1, 64]
    say(f"{dtype} fused rows, {pad} padding elements per row: prefix {first} + new {second}")
    pb, layer = _mk(model, [a + b + 1 for a, b in zip(first, second)], seed=61)
    cu1, cu2 = wl.cu_from_lengths(first), wl.cu_from_lengths(second)
    cb = np.asarray(first, dtype=np.int32)
    table = dev_i32(pb.block_table)

    def fused(T, seed):
        rows = wl.randn((T, (Hq + 2 * Hkv) * D + pad), dtype, seed, device="cuda")
        body = rows[:, :(Hq + 2 * Hkv) * D].unflatten(1, (Hq + 2 * Hkv, D))
        return body[:, :Hq], body[:, Hq:Hq + Hkv], body[:, Hq + Hkv:]

    _, k1, v1 = fused(int(cu1[-1]), 610)
    layer.ctx.kv_append_strided(layer.kc, layer.vc, k1, v1, dev_i32(cu1), dev_i32(np.zeros(4, np.int32)), table)

    def orc_append(k, v, cu, before):
        orc.kv_append(layer.shape, layer.okc, layer.ovc, wl.to_bits(k), wl.to_bits(v), cu, before, pb.block_table)

    orc_append(k1, v1, cu1, np.zeros(4, np.int32))
    q2, k2, v2 = fused(int(cu2[-1]), 620)
    assert not q2.is_contiguous() and not k2.is_contiguous()
    layer.ctx.kv_append_strided(layer.kc, layer.vc, k2, v2, dev_i32(cu2), dev_i32(cb), table)
    orc_append(k2, v2, cu2, cb)
    layer.assert_cache_bit_exact()

    out = torch.full((q2.shape[0], Hq, D), float("nan"), dtype=q2.dtype, device="cuda")
    lse = torch.full((q2.shape[0], Hq), float("nan"), dtype=torch.float32, device="cuda")
    layer.ctx.attn_prefill_strided(q2, layer.kc, layer.vc, dev_i32(cu2), dev_i32(cb), table, out, lse,
                                   max_q_len=max(second))
    ref, ref_lse = layer.prefill_oracle(q2, cu2, cb, pb.block_table)
    compare("prefill on fused rows", out, ref, dtype)
    compare_lse("prefill on fused rows", lse, ref_lse, dtype, bf16_row_sum=True)
    packed, _ = layer.prefill_gpu(q2.contiguous(), cu2, cb, pb.block_table)
    assert torch.equal(out.view(torch.uint8), packed.view(torch.uint8)), "strided and packed prefill differ"

    ctx = cb + np.asarray(second, dtype=np.int32)
    qd, kd, vd = fused(4, 630)
    layer.ctx.kv_append_strided(layer.kc, layer.vc, kd, vd, dev_i32(wl.cu_from_lengths([1] * 4)), dev_i32(ctx), table,
                                max_new_len=1)
    orc_append(kd, vd, wl.cu_from_lengths([1] * 4), ctx)
    layer.assert_cache_bit_exact()
    ctx = ctx + 1
    out = torch.full((4, Hq, D), float("nan"), dtype=qd.dtype, device="cuda")
    lse = torch.full((4, Hq), float("nan"), dtype=torch.float32, device="cuda")
    layer.ctx.attn_decode_strided(qd, layer.kc, layer.vc, table, dev_i32(ctx), out, int(ctx.max()), lse)
    ref, ref_lse = layer.decode_oracle(qd, pb.block_table, ctx)
    compare("decode on fused rows", out, ref, dtype)
    compare_lse("decode on fused rows", lse, ref_lse, dtype)
    packed, _ = layer.decode_gpu(qd.contiguous(), pb.block_table, ctx)
    assert torch.equal(out.view(torch.uint8), packed.view(torch.uint8)), "strided and packed decode differ"

    # strides the library must refuse: shorter than a packed row, not a multiple of 16 bytes, 2^31 or more
    lib, h, vp = binding._lib, layer.ctx._h, binding._ptr
    for bad in (Hkv * D - 8, Hkv * D + 1, 1 << 31):
        st = lib.ecoserve_kv_append_strided(h, vp(layer.kc), vp(layer.vc), vp(kd), vp(vd), bad,
                                            vp(dev_i32(wl.cu_from_lengths([1] * 4))), vp(dev_i32(ctx)), vp(table),
                                            pb.block_table.shape[1], 4, 4, 1, None)
        assert st == binding.EINVAL, bad
    for bad in (Hq * D - 8, Hq * D + 1, 1 << 31):
        st = lib.ecoserve_attn_decode_strided(h, vp(qd), bad, vp(layer.kc), vp(layer.vc), vp(table),
                                              pb.block_table.shape[1], vp(dev_i32(ctx)), vp(out), None, 4,
                                              int(ctx.max()), None)
        assert st == binding.EINVAL, bad
    layer.close()


def test_hot_calls_can_be_captured_in_a_hip_graph():
    """One decode step of three layers (append one token, decode; one of them as the fused call) and one prefill call recorded into a HIP
    graph and replayed three times with new input contents and the program's own eager work in between:
    every replay must give exactly what the eager calls give on the same inputs.  The hot calls neither
    allocate nor synchronise, so a capturing stream can take them (default options: equal decode shares, a
    tile list per prefill call)."""
    model = M30
    layers = 3
    lens = [700, 33, 1500, 64, 257]
    say("HIP graph capture of append + decode (3 layers) and of prefill")
    pb = wl.prefill_batch(model, [n + 1 for n in lens], 71)
    Ls = [Layer(model, pb.num_blocks, pb.B, pb.block_table.shape[1], oracle_cache=False) for _ in range(layers)]
    table = dev_i32(pb.block_table)
    cu = dev_i32(wl.cu_from_lengths(lens))
    zero = dev_i32(np.zeros(pb.B))
    for i, L in enumerate(Ls):
        _, k, v = _qkv(model, sum(lens), 710 + 10 * i)
        L.ctx.kv_append(L.kc, L.vc, k.cuda(), v.cuda(), cu, zero, table)
    ones = dev_i32(wl.cu_from_lengths([1] * pb.B))
    before, ctx = dev_i32(np.asarray(lens)), dev_i32(np.asarray(lens) + 1)
    B, T = pb.B, sum(lens)
    q = torch.empty((B, model.Hq, model.D), dtype=torch.bfloat16, device="cuda")
    kn, vn = (torch.empty((B, model.Hkv, model.D), dtype=torch.bfloat16, device="cuda") for _ in range(2))
    qp = torch.empty((T, model.Hq, model.D), dtype=torch.bfloat16, device="cuda")
    out = torch.empty((layers, B, model.Hq, model.D), dtype=torch.bfloat16, device="cuda")
    outp = torch.empty_like(qp)

    def work():
        for i, L in enumerate(Ls):
            if i == 1:          # the middle layer through the fused call
                L.ctx.attn_decode_append(q, kn, vn, L.kc, L.vc, table, ctx, out[i], max(lens) + 1)
                continue
            L.ctx.kv_append(L.kc, L.vc, kn, vn, ones, before, table, max_new_len=1)
            L.ctx.attn_decode(q, L.kc, L.vc, table, ctx, out[i], max(lens) + 1)
        Ls[0].ctx.attn_prefill(qp, Ls[0].kc, Ls[0].vc, cu, zero, table, outp, max_q_len=max(lens))

    def new_inputs(seed):
        q.copy_(wl.randn(q.shape, "bf16", seed, device="cuda"))
        kn.copy_(wl.randn(kn.shape, "bf16", seed + 1, device="cuda"))
        vn.copy_(wl.randn(vn.shape, "bf16", seed + 2, device="cuda"))
        qp.copy_(wl.randn(qp.shape, "bf16", seed + 3, device="cuda"))

    new_inputs(720)
    work()                      # warm: nothing is created lazily inside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        work()
    for r in range(3):
        new_inputs(730 + 10 * r)
        work()
        torch.cuda.synchronize()
        want, wantp = out.clone(), outp.clone()
        out.fill_(float("nan"))
        outp.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), want.view(torch.int16)), f"decode: replay {r} differs from eager"
        assert torch.equal(outp.view(torch.int16), wantp.view(torch.int16)), f"prefill: replay {r} differs from eager"
    for L in Ls:
        L.close()


def test_machine_ceiling_probes_report_plausible_rates():
    """The two measurement helpers run, return rates of the right order for this class of device (between
    a quarter of and the whole published peak: 8 TB/s, 2.5 PFLOP/s) and reject bad arguments."""
    from paper_2504_18154_amd import binding
    say("machine ceiling probes")
    bw = binding.probe_hbm_read(1 << 30, reps=3)
    smooth = binding.probe_mfma_bf16(False, reps=2)
    rand = binding.probe_mfma_bf16(True, reps=2)
    say(f"  read {bw:.0f} GB/s, bf16 MFMA {smooth:.0f} TFLOP/s (smooth operands), {rand:.0f} (random)")
    assert 2000 < bw < 8000
    assert 625 < rand <= smooth * 1.02 and smooth < 2520
    for bad in (lambda: binding.probe_hbm_read(1000), lambda: binding.probe_hbm_read(1 << 30, reps=0),
                lambda: binding.probe_hbm_read(1 << 30, device=99), lambda: binding.probe_mfma_bf16(True, reps=0)):
        with pytest.raises(binding.EcoserveError) as ei:
            bad()
        assert ei.value.status == binding.EINVAL


def test_profile_events_report_kernel_time():
    from paper_2504_18154_amd import binding
    model = M30
    pb, layer = _mk(model, [300, 500], seed=14)
    q, k, v = _qkv(model, pb.T, 160)
    layer.ctx.set_option(binding.OPT_PROFILE, 1)
    layer.append(k, v, pb.cu_q, pb.ctx_before, pb.block_table)
    for _ in range(3):
        layer.prefill_gpu(q, pb.cu_q, pb.ctx_before, pb.block_table)
    ms, n = layer.ctx.profile_read(binding.KERNEL_PREFILL)
    assert n == 3 and 0 < ms < 1000
    ms, n = layer.ctx.profile_read(binding.KERNEL_APPEND)
    assert n == 1 and ms > 0
    layer.ctx.profile_reset()
    assert layer.ctx.profile_read(binding.KERNEL_PREFILL) == (0.0, 0)
    # every third call of a kind: calls 0, 3 and 6 of seven are bracketed, the appends count on their own
    layer.ctx.set_option(binding.OPT_PROFILE, 3)
    layer.ctx.profile_reset()
    for i in range(7):
        layer.prefill_gpu(q, pb.cu_q, pb.ctx_before, pb.block_table)
        if i < 2:
            layer.append(k, v, pb.cu_q, pb.ctx_before, pb.block_table)
    ms, n = layer.ctx.profile_read(binding.KERNEL_PREFILL)
    assert n == 3 and 0 < ms < 1000
    assert layer.ctx.profile_read(binding.KERNEL_APPEND)[1] == 1
    with pytest.raises(binding.EcoserveError):
        layer.ctx.set_option(binding.OPT_PROFILE, -1)
    layer.close()
