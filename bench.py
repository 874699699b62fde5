#!/usr/bin/env python3
"""Benchmark of the paged-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline]

One "step" is one pass of the whole hot path over one phase-pure batch pair of the
30B-scale model (40 query heads, 8 K/V heads, head size 128, block size 16, 64 layers,
bf16), with every input resident in HBM before the timed region starts:

  * prefill-only batch (BASELINE config index 2): 16 prompts, lengths lognormal(mean 1024)
    clipped to [128, 4096]; per layer kv_append of all prompt tokens, then causal prefill
    attention over the paged cache;
  * decode-only batch (BASELINE config index 1): 128 resident sequences, contexts uniform in
    [512, 4096], physical blocks randomly permuted; per layer kv_append of one token per
    sequence, then split-context decode attention.  64 independent layer caches.

It prints ONE JSON line.  `value` is the decode phase's algorithmic HBM traffic rate (GB/s),
the headline metric; the prefill phase's causal TFLOP/s and the append rates ride along.
`roofline` is for the dominant kernel (decode partial attention): algorithmic bytes per
launch / its average launch duration, measured with HIP events recorded by the library on
the launch stream around every 7th launch inside the timed region.  `cpu_baseline` is the fp64
oracle on the host cores, on one layer of the decode batch.

    python bench.py --sweep

times the kernels alone on the other batch shapes (the 70B-scale decode and phase-switch
configurations, a multi-head model, longer contexts, uniform prompt lengths) over a few layer
caches each and prints one JSON line {"sweep": [...]}: the source of the table in the benchmark spec.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def sweep() -> int:
    """Kernel time and rate on other batch shapes, a few layer caches each, all launches bracketed."""
    import numpy as np
    import torch

    from paper_2504_18154_amd import accounting as acc
    from paper_2504_18154_amd import binding, build
    from paper_2504_18154_amd import workloads as wl

    if not os.path.exists(binding.LIB_PATH):
        build.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(0)
    i32 = lambda a: torch.as_tensor(np.ascontiguousarray(a, dtype=np.int32), device=dev)
    rows = []

    def pools(n_elems, layers, seed):
        g = torch.Generator(device=dev)
        g.manual_seed(seed)
        mk = lambda: torch.randn(n_elems, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
        return [(mk(), mk()) for _ in range(layers)]

    def run_passes(ctx, one_pass, warm_ms=60.0, timed_ms=60.0):
        """Untimed passes until the chip has been busy for warm_ms (clocks settle), then bracketed passes."""
        for phase_ms, bracket in ((warm_ms, False), (timed_ms, True)):
            if bracket:
                ctx.set_option(binding.OPT_PROFILE, 1)
                ctx.profile_reset()
            t0, n = time.perf_counter(), 0
            while n < 3 or (time.perf_counter() - t0) * 1e3 < phase_ms:
                one_pass()
                torch.cuda.synchronize()
                n += 1

    def decode(name, db, layers=4):
        m = db.model
        ctx = binding.Context(m.Hq, m.Hkv, m.D, db.num_blocks, "bf16", db.B, db.block_table.shape[1])
        ctx.set_option(binding.OPT_DECODE_ADAPTIVE, 1)
        caches = pools(db.num_blocks * m.Hkv * m.bs * m.D, layers, db.seed)
        q = wl.randn((db.B, m.Hq, m.D), "bf16", db.seed + 3, device=dev)
        out = torch.empty_like(q)
        bt, cl = i32(db.block_table), i32(db.ctx_len)

        def one_pass():
            for kc, vc in caches:
                ctx.attn_decode(q, kc, vc, bt, cl, out, db.max_ctx_len)

        run_passes(ctx, one_pass)
        ms, n = ctx.profile_read(binding.KERNEL_DECODE)
        by = acc.decode_bytes(db.ctx_len, m.Hq, m.Hkv, m.D, m.bs)
        rate = by / (ms / n * 1e-3) / 1e9
        rows.append({"workload": name, "kernel": "decode_mfma_kernel", "avg_launch_us": ms / n * 1e3, "launches": n,
                     "algorithmic_bytes_per_launch": by, "GBps": rate, "frac_of_hbm_peak": rate / acc.PEAK_HBM_GBPS})
        ctx.close()

    def prefill(name, m, q_len, layers=2):
        pb = wl.prefill_batch(m, q_len, 3)
        ctx = binding.Context(m.Hq, m.Hkv, m.D, pb.num_blocks, "bf16", pb.B, pb.block_table.shape[1])
        ctx.set_option(binding.OPT_PREFILL_REUSE_PLAN, 1)
        q = wl.randn((pb.T, m.Hq, m.D), "bf16", 11, device=dev)
        k = wl.randn((pb.T, m.Hkv, m.D), "bf16", 12, device=dev)
        v = wl.randn((pb.T, m.Hkv, m.D), "bf16", 13, device=dev)
        out = torch.empty_like(q)
        cu, cb, bt = i32(pb.cu_q), i32(pb.ctx_before), i32(pb.block_table)
        caches = [ctx.new_cache(fill_bits=0) for _ in range(layers)]

        def one_pass():
            ctx.set_option(binding.OPT_PREFILL_REUSE_PLAN, 1)   # one list of query tiles per pass over the layers
            for kc, vc in caches:
                ctx.kv_append(kc, vc, k, v, cu, cb, bt, max_new_len=pb.max_q_len)
                ctx.attn_prefill(q, kc, vc, cu, cb, bt, out, max_q_len=pb.max_q_len)

        run_passes(ctx, one_pass)
        ms, n = ctx.profile_read(binding.KERNEL_PREFILL)
        ams, an = ctx.profile_read(binding.KERNEL_APPEND)
        fl = acc.prefill_flops_causal(pb.q_len, m.Hq, m.D)
        tf = fl / (ms / n * 1e-3) / 1e12
        ab = acc.append_bytes(pb.T, m.Hkv, m.D)
        rows.append({"workload": name, "kernel": "prefill_mfma_kernel", "avg_launch_us": ms / n * 1e3, "launches": n,
                     "algorithmic_flops_per_launch": fl, "TFLOPs": tf, "frac_of_bf16_peak": tf / acc.PEAK_BF16_TFLOPS,
                     "append_us": ams / an * 1e3, "append_GBps": ab / (ams / an * 1e-3) / 1e9})
        ctx.close()

    decode("30B decode: 128 seqs, ctx U[512,4096] (BASELINE config 1)", wl.config2_decode_30b())
    decode("70B decode: 256 seqs, ctx U[1024,4096], 64 q heads (BASELINE config 3)", wl.config4_decode_70b())
    resident, new, table, nb = wl.config5_switch_70b()
    decode("70B phase switch, decode side: 192 resident + 8 new x 8192 (BASELINE config 4)",
           wl.DecodeBatch(wl.M70B, np.concatenate([resident, new]).astype(np.int32), table, nb, 0), layers=2)
    decode("30B, 128 seqs, every context 8192", wl.decode_batch(wl.M30B, 128, 8192, 8192, 5))
    decode("multi-head model (52 q = 52 kv heads), 128 seqs, ctx U[512,4096]",
           wl.decode_batch(wl.M30B_MHA, 128, 512, 4096, 7), layers=2)
    decode("30B, 16 seqs, ctx U[512,4096] (small batch)", wl.decode_batch(wl.M30B, 16, 512, 4096, 6))

    def consecutive(db):
        """The same batch over a block table that gives every sequence consecutive physical blocks (a fresh allocator)."""
        table = np.array(db.block_table)
        first = 0
        for b, n in enumerate((np.asarray(db.ctx_len) + db.model.bs - 1) // db.model.bs):
            table[b, :n] = np.arange(first, first + n)
            first += n
        return wl.DecodeBatch(db.model, db.ctx_len, table.astype(np.int32), db.num_blocks, db.seed)

    decode("30B decode batch of config 1 over consecutive physical blocks", consecutive(wl.config2_decode_30b()))
    decode("30B, 128 seqs, every context 8192, over consecutive physical blocks",
           consecutive(wl.decode_batch(wl.M30B, 128, 8192, 8192, 5)))
    decode("30B, 512 seqs, contexts shaped like ShareGPT (Table 4)", wl.table4_decode_batch(wl.M30B, "sharegpt", 512, 21))
    decode("30B, 1024 seqs, contexts shaped like Alpaca (Table 4)", wl.table4_decode_batch(wl.M30B, "alpaca", 1024, 22))
    decode("30B, 64 seqs, contexts shaped like LongBench (Table 4)", wl.table4_decode_batch(wl.M30B, "longbench", 64, 23))
    prefill("30B prefill: 16 prompts lognormal in [128,4096] (BASELINE config 2)", wl.M30B,
            wl.config3_prefill_30b().q_len)
    prefill("70B phase switch, prefill side: 8 x 8192, 64 q heads (BASELINE config 4)", wl.M70B, [8192] * 8)
    prefill("30B, 16 x 1024", wl.M30B, [1024] * 16)
    prefill("30B, 64 x 256", wl.M30B, [256] * 64)
    prefill("30B, 4 x 4096", wl.M30B, [4096] * 4)
    prefill("multi-head model (52/52), 16 x 1024", wl.M30B_MHA, [1024] * 16)
    prefill("30B, 64 prompts shaped like ShareGPT (Table 4)", wl.M30B, wl.table4_lengths("sharegpt", wl.rng_for(31), 64)[0])
    prefill("30B, 512 prompts shaped like Alpaca (Table 4)", wl.M30B, wl.table4_lengths("alpaca", wl.rng_for(32), 512)[0])
    prefill("30B, 8 prompts shaped like LongBench (Table 4)", wl.M30B, wl.table4_lengths("longbench", wl.rng_for(33), 8)[0])
    print(json.dumps({"sweep": rows, "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
                      "note": "kernel time alone from HIP events around every launch; decode with per-XCD shares"}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debugging only; invalid as a result)")
    ap.add_argument("--split-tokens", type=int, default=0, help="force the decode split size (tuning)")
    ap.add_argument("--prefill-chunk", type=int, default=0,
                    help="process every prompt in chunks of this many tokens (each chunk attends to the cached prefix "
                         "of its prompt): quantifies the repeated K/V reads of chunked prefill; 0 = whole prompts")
    ap.add_argument("--equal-shares", action="store_true",
                    help="decode with equal chunks per wavefront instead of per-XCD shares that follow measured speeds")
    ap.add_argument("--phase", choices=["both", "decode", "prefill"], default="both",
                    help="run only one phase (profiling runs; the default is the full step)")
    ap.add_argument("--fused-qkv", action="store_true",
                    help="Q, K and V are slices of one row [Hq + 2 Hkv][D] per token (the output of a fused projection, "
                         "Eq. 1) and are read in place through the strided calls; default: three packed arrays")
    ap.add_argument("--separate-append", action="store_true",
                    help="decode phase: kv_append and attn_decode as two calls per layer (default: one call, "
                         "ecoserve_attn_decode_append, which takes the new tokens from the new rows and stores them "
                         "with its merge launch; same bits in cache and output)")
    ap.add_argument("--event-every", type=int, default=7,
                    help="bracket every n-th launch of each kernel with HIP events inside the timed region (an event pair "
                         "per launch delays the stream by several microseconds per layer; 1 = every launch)")
    ap.add_argument("--no-probes", action="store_true",
                    help="skip the two machine-ceiling probes (streaming read, matrix-core loop) after the timed region")
    ap.add_argument("--sweep", action="store_true",
                    help="time the kernels alone on the other batch shapes and print {\"sweep\": [...]} instead")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also launch one plain 1 GiB device copy (known traffic, for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the path has no cross-GPU exchange step); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    if args.sweep:
        return sweep()
    if args.fused_qkv and args.prefill_chunk:
        print("bench.py: --fused-qkv and --prefill-chunk are separate experiments; give one of them", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2504_18154_amd import accounting as acc
    from paper_2504_18154_amd import binding, build
    from paper_2504_18154_amd import workloads as wl

    if not os.path.exists(binding.LIB_PATH):
        build.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda", 0)
    model = wl.M30B
    layers = args.layers or model.layers
    do_dec = args.phase in ("both", "decode")
    do_pre = args.phase in ("both", "prefill")

    def i32(a):
        return torch.as_tensor(np.ascontiguousarray(a, dtype=np.int32), device=dev)

    def fill_randn_(t: torch.Tensor, seed: int):
        g = torch.Generator(device=dev)
        g.manual_seed(seed)
        chunk = 1 << 26
        flat = t.view(-1)
        for o in range(0, flat.numel(), chunk):
            n = min(chunk, flat.numel() - o)
            flat[o:o + n] = torch.randn(n, generator=g, device=dev, dtype=torch.float32).to(t.dtype)

    # ---------------- decode-only batch (config index 1) ---------------------------------
    db = wl.config2_decode_30b()
    dctx = binding.Context(model.Hq, model.Hkv, model.D, db.num_blocks, "bf16", db.B, db.block_table.shape[1])
    if args.split_tokens:
        dctx.set_option(binding.OPT_DECODE_SPLIT_TOKENS, args.split_tokens)
    if not args.equal_shares:
        dctx.set_option(binding.OPT_DECODE_ADAPTIVE, 1)
    pool_elems = db.num_blocks * model.Hkv * model.bs * model.D
    d_bt, d_len = i32(db.block_table), i32(db.ctx_len)
    d_before = i32(db.ctx_len - 1)
    d_cu = i32(np.arange(db.B + 1))
    d_pools = []
    stream_k = stream_v = None
    if do_dec:
        for l in range(layers):
            if l == 0:
                # layer 0 is built through kv_append from a token stream the oracle can replay
                kc, vc = dctx.new_cache()
                T0 = int(db.ctx_len.sum())
                stream_k = wl.randn((T0, model.Hkv, model.D), "bf16", db.seed + 1, device=dev)
                stream_v = wl.randn((T0, model.Hkv, model.D), "bf16", db.seed + 2, device=dev)
                dctx.kv_append(kc, vc, stream_k, stream_v, i32(wl.cu_from_lengths(db.ctx_len)),
                               i32(np.zeros(db.B)), d_bt)
            else:
                kc = torch.empty(pool_elems, dtype=torch.bfloat16, device=dev)
                vc = torch.empty(pool_elems, dtype=torch.bfloat16, device=dev)
                fill_randn_(kc, db.seed + 10 * l)
                fill_randn_(vc, db.seed + 10 * l + 1)
            d_pools.append((kc, vc))
    d_q = wl.randn((db.B, model.Hq, model.D), "bf16", db.seed + 3, device=dev)
    d_knew = wl.randn((db.B, model.Hkv, model.D), "bf16", db.seed + 4, device=dev)
    d_vnew = wl.randn((db.B, model.Hkv, model.D), "bf16", db.seed + 5, device=dev)
    if do_dec:
        # the new token of layer 0 is the last token of its stream, so the cache stays replayable
        last = torch.as_tensor(np.cumsum(db.ctx_len) - 1, device=dev, dtype=torch.long)
        d_knew0, d_vnew0 = stream_k[last].contiguous(), stream_v[last].contiguous()
    d_out = torch.empty((layers, db.B, model.Hq, model.D), dtype=torch.bfloat16, device=dev)

    def fuse(q, k, v):
        """The same bits as slices of one [tokens, Hq + 2 Hkv, D] array."""
        rows = torch.cat([q, k, v], dim=1)
        return rows[:, :model.Hq], rows[:, model.Hq:model.Hq + model.Hkv], rows[:, model.Hq + model.Hkv:]

    if args.fused_qkv:
        if do_dec:
            _, d_knew0, d_vnew0 = fuse(d_q, d_knew0, d_vnew0)
        d_q, d_knew, d_vnew = fuse(d_q, d_knew, d_vnew)

    # ---------------- prefill-only batch (config index 2) --------------------------------
    pb = wl.config3_prefill_30b()
    pctx = binding.Context(model.Hq, model.Hkv, model.D, pb.num_blocks, "bf16", pb.B, pb.block_table.shape[1])
    p_bt, p_cu, p_before = i32(pb.block_table), i32(pb.cu_q), i32(pb.ctx_before)
    # the 64 layers of a step pass the same batch arrays: the list of query tiles is built once per step
    pctx.set_option(binding.OPT_PREFILL_REUSE_PLAN, 1)
    p_pools = [pctx.new_cache(fill_bits=0) for _ in range(layers)] if do_pre else []
    p_q = wl.randn((pb.T, model.Hq, model.D), "bf16", pb.seed + 3, device=dev)
    p_k = wl.randn((pb.T, model.Hkv, model.D), "bf16", pb.seed + 4, device=dev)
    p_v = wl.randn((pb.T, model.Hkv, model.D), "bf16", pb.seed + 5, device=dev)
    p_out = torch.empty_like(p_q)
    if args.fused_qkv:
        p_q, p_k, p_v = fuse(p_q, p_k, p_v)
    append = (lambda c: c.kv_append_strided) if args.fused_qkv else (lambda c: c.kv_append)
    prefill = pctx.attn_prefill_strided if args.fused_qkv else pctx.attn_prefill
    decode = dctx.attn_decode_strided if args.fused_qkv else dctx.attn_decode
    # chunked prefill: chunk ci holds tokens [ci C, ci C + C) of every prompt that is that long
    p_chunks = []
    if args.prefill_chunk > 0:
        C = args.prefill_chunk
        for ci in range((pb.max_q_len + C - 1) // C):
            lens = np.clip(pb.q_len.astype(np.int64) - ci * C, 0, C)
            idx = np.concatenate([np.arange(pb.cu_q[b] + ci * C, pb.cu_q[b] + ci * C + lens[b]) for b in range(pb.B)])
            sel = torch.as_tensor(idx, device=dev, dtype=torch.long)
            before = np.minimum(pb.q_len, ci * C) + pb.ctx_before
            p_chunks.append(dict(q=p_q[sel].contiguous(), k=p_k[sel].contiguous(), v=p_v[sel].contiguous(),
                                 out=torch.empty((len(idx), model.Hq, model.D), dtype=torch.bfloat16, device=dev),
                                 cu=i32(wl.cu_from_lengths(lens)), before=i32(before), max_len=int(lens.max())))

    ev = lambda: torch.cuda.Event(enable_timing=True)

    def step(timers=None):
        t = [ev() for _ in range(3)]
        t[0].record()
        if do_pre:
            # a step brings a new batch: its list of query tiles is built once, by the first layer's call
            pctx.set_option(binding.OPT_PREFILL_REUSE_PLAN, 1)
            for l in range(layers):
                kc, vc = p_pools[l]
                if not p_chunks:
                    append(pctx)(kc, vc, p_k, p_v, p_cu, p_before, p_bt, max_new_len=pb.max_q_len)
                    prefill(p_q, kc, vc, p_cu, p_before, p_bt, p_out, max_q_len=pb.max_q_len)
                for ch in p_chunks:
                    pctx.kv_append(kc, vc, ch["k"], ch["v"], ch["cu"], ch["before"], p_bt, max_new_len=ch["max_len"])
                    pctx.attn_prefill(ch["q"], kc, vc, ch["cu"], ch["before"], p_bt, ch["out"], max_q_len=ch["max_len"])
        t[1].record()
        if do_dec:
            for l in range(layers):
                kc, vc = d_pools[l]
                kn, vn = (d_knew0, d_vnew0) if l == 0 else (d_knew, d_vnew)
                if not args.separate_append:
                    dctx.attn_decode_append(d_q, kn, vn, kc, vc, d_bt, d_len, d_out[l], db.max_ctx_len)
                else:
                    append(dctx)(kc, vc, kn, vn, d_cu, d_before, d_bt, max_new_len=1)
                    decode(d_q, kc, vc, d_bt, d_len, d_out[l], db.max_ctx_len)
        t[2].record()
        if timers is not None:
            timers.append(t)

    for _ in range(args.warmup):
        step()
    if args.calibration_copy:
        src = torch.empty(1 << 29, dtype=torch.bfloat16, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)   # 1 GiB read + 1 GiB written by a plain copy kernel
        torch.cuda.synchronize()
        del src, dst
    for c in (dctx, pctx):
        # chunked prefill makes calls of different sizes per layer: bracket them all
        c.set_option(binding.OPT_PROFILE, 1 if args.prefill_chunk else max(1, args.event_every))
        c.profile_reset()
    timers = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(timers)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    pre_ms = sum(t[0].elapsed_time(t[1]) for t in timers) / args.steps
    dec_ms = sum(t[1].elapsed_time(t[2]) for t in timers) / args.steps
    k_dec_ms, k_dec_n = dctx.profile_read(binding.KERNEL_DECODE)
    k_dapp_ms, k_dapp_n = dctx.profile_read(binding.KERNEL_APPEND)
    k_pre_ms, k_pre_n = pctx.profile_read(binding.KERNEL_PREFILL)
    k_papp_ms, k_papp_n = pctx.profile_read(binding.KERNEL_APPEND)

    # ---------------- algorithmic work --------------------------------------------------
    dec_bytes_layer = acc.decode_bytes(db.ctx_len, model.Hq, model.Hkv, model.D, model.bs)
    dec_app_bytes_layer = acc.append_bytes(db.B, model.Hkv, model.D)
    pre_flops_layer = acc.prefill_flops_causal(pb.q_len, model.Hq, model.D)
    pre_app_bytes_layer = acc.append_bytes(pb.T, model.Hkv, model.D)

    def rate(x, ms):
        return x / (ms * 1e-3) if ms and ms > 0 else None

    res = {
        "metric": "decode attn HBM GB/s + prefill attn TFLOP/s, % of MI355X roofline",
        "value": None, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall_ms / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {
            "workload": "30B-scale PaDG step: prefill-only batch (16 prompts, lognormal mean 1024 in [128,4096]) "
                        "then decode-only batch (128 seqs, ctx U[512,4096]); 40 q heads / 8 kv heads / D 128 / "
                        "block 16; append + attention per layer",
            "layers": layers, "phase": args.phase, "decode_shares": "equal" if args.equal_shares else "per-XCD, measured",
            "prefill_tile_list": "built once per step, shared by the layers",
            "decode_append": "a launch of its own" if args.separate_append else "fused into the decode call",
            "qkv_rows": "slices of fused rows [tokens, Hq + 2 Hkv, D], read in place" if args.fused_qkv
                        else "three packed arrays",
            "kernel_events": "every launch" if args.prefill_chunk or args.event_every <= 1
                             else f"every {args.event_every}th launch of each kernel",
            "decode_batch": db.B, "decode_ctx_tokens": int(db.ctx_len.sum()),
            "prefill_prompts": pb.B, "prefill_tokens": pb.T, "prefill_lengths": [int(x) for x in pb.q_len],
        },
    }
    def measured_traffic(kernel):
        """HBM bytes per launch from the committed rocprofv3 --pmc runs (profiles/traffic.json), or None."""
        try:
            with open(os.path.join(ROOT, "profiles", "traffic.json")) as f:
                t = json.load(f).get(kernel)
            return None if t is None else t["fetch_bytes_per_launch"] + t["write_bytes_per_launch"]
        except (OSError, ValueError, KeyError):
            return None

    if do_dec:
        # phase time includes the one-token appends (fused or not) and the merge kernels: whole decode phase
        res["value"] = rate(dec_bytes_layer * layers, dec_ms) / 1e9
        res["decode"] = {
            "ms_per_layer": dec_ms / layers, "phase_ms": dec_ms, "GBps": res["value"],
            "frac_of_hbm_peak": res["value"] / acc.PEAK_HBM_GBPS,
            "append_us_per_layer": 1e3 * k_dapp_ms / k_dapp_n if k_dapp_n else None,
        }
        avg_ms = k_dec_ms / max(k_dec_n, 1)
        a = rate(dec_bytes_layer, avg_ms) / 1e9
        res["roofline"] = {"kernel": "decode_mfma_kernel", "bound": "hbm", "achieved": a, "peak": acc.PEAK_HBM_GBPS,
                           "unit": "GB/s", "frac": a / acc.PEAK_HBM_GBPS,
                           "traffic": measured_traffic("decode_mfma_kernel") if layers == model.layers else None,
                           "avg_launch_us": avg_ms * 1e3, "launches": k_dec_n,
                           "algorithmic_bytes_per_launch": dec_bytes_layer}
    if do_pre:
        tf = rate(pre_flops_layer * layers, pre_ms) / 1e12
        calls = max(1, len(p_chunks))  # hot calls per layer (chunked prefill: one per chunk)
        avg_ms = calls * k_pre_ms / max(k_pre_n, 1)      # kernel time per layer
        ktf = rate(pre_flops_layer, avg_ms) / 1e12
        app_ms = calls * k_papp_ms / max(k_papp_n, 1)
        res["prefill"] = {
            "value": tf, "unit": "TFLOP/s", "ms_per_layer": pre_ms / layers, "phase_ms": pre_ms,
            "frac_of_bf16_peak": tf / acc.PEAK_BF16_TFLOPS,
            "roofline": {"kernel": "prefill_mfma_kernel", "bound": "mfma", "achieved": ktf,
                         "peak": acc.PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": ktf / acc.PEAK_BF16_TFLOPS,
                         "traffic": measured_traffic("prefill_mfma_kernel") if layers == model.layers and calls == 1 else None,
                         "avg_launch_us": avg_ms * 1e3 / calls, "launches": k_pre_n,
                         "algorithmic_flops_per_launch": pre_flops_layer},
            "chunk_tokens": args.prefill_chunk, "calls_per_layer": calls,
            "append": {"GBps": rate(pre_app_bytes_layer, app_ms) / 1e9, "avg_launch_us": app_ms * 1e3 / calls,
                       "frac_of_hbm_peak": rate(pre_app_bytes_layer, app_ms) / 1e9 / acc.PEAK_HBM_GBPS},
        }
        if not do_dec:
            res["value"], res["unit"] = tf, "TFLOP/s"

    # ---------------- CPU baseline: the oracle on one decode layer ------------------------
    if do_dec and not args.no_cpu_baseline:
        from oracle import oracle as orc
        shape = orc.Shape(model.Hq, model.Hkv, model.D, model.bs, db.num_blocks, orc.BF16)
        okc, ovc = orc.new_cache(shape)
        orc.kv_append(shape, okc, ovc, wl.to_bits(stream_k), wl.to_bits(stream_v), wl.cu_from_lengths(db.ctx_len),
                      np.zeros(db.B, dtype=np.int32), db.block_table)
        qh = wl.to_bits(d_q)
        reps, t0 = 0, time.perf_counter()
        while reps < 3 or time.perf_counter() - t0 < 1.5:   # ~1.5 s on all host cores
            ref, _ = orc.attn_decode(shape, qh, okc, ovc, db.block_table, db.ctx_len)
            reps += 1
        cpu_s = (time.perf_counter() - t0) / reps
        err = np.abs(d_out[0].double().cpu().numpy() - ref)
        res["cpu_baseline"] = {
            "value": dec_bytes_layer / cpu_s / 1e9, "unit": "GB/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"one full layer of the decode batch (128 seqs, {int(db.ctx_len.sum())} cached tokens), "
                      f"fp64, {reps} repetitions, {cpu_s:.3f} s each",
            "seconds": cpu_s,
            "gpu_vs_oracle_layer0_max_abs": float(err.max()), "gpu_vs_oracle_layer0_mean_abs": float(err.mean()),
        }
    # ---------------- what this device sustains on the two rooflines' resources ------------
    if not args.no_probes:
        res["machine"] = {
            "hbm_read_GBps": binding.probe_hbm_read(4 << 30, reps=5),
            "hbm_read_same_bytes_GBps": binding.probe_hbm_read(int(dec_bytes_layer) // 8192 * 8192, reps=20),
            "mfma_bf16_TFLOPs": binding.probe_mfma_bf16(False, reps=5),
            "mfma_bf16_random_operands_TFLOPs": binding.probe_mfma_bf16(True, reps=5),
            "how": "after the timed region: 4 GiB (and as many bytes as one decode launch reads) read in 8 KiB pieces per "
                   "wavefront, 16-byte non-temporal loads; register-only 32x32x16 bf16 loop, "
                   "4 wavefronts per SIMD, smooth and pseudo-random operands; 5 launches each after one untimed",
        }
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
