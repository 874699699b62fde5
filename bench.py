#!/usr/bin/env python3
"""Benchmark of the paged-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--only SECTIONS] [--no-cpu-baseline]

It prints ONE JSON line.

The timed "step" (W warm-up steps, then K timed ones) is one pass of the whole hot path over one
phase-pure batch pair of the 30B-scale model (40 query heads, 8 K/V heads, head size 128, block size
16, 64 layers, bf16), every input resident in HBM before the timed region starts:

  * prefill-only batch (BASELINE config index 2): 16 prompts, lengths lognormal(mean 1024) clipped to
    [128, 4096]; per layer kv_append of all prompt tokens, then causal prefill attention over the paged
    cache;
  * decode-only batch (BASELINE config index 1): 128 resident sequences, contexts uniform in
    [512, 4096], physical blocks randomly permuted; per layer one new token per sequence appended and
    split-context decode attention, 64 independent layer caches.

`value` is the decode phase's algorithmic HBM traffic rate (GB/s), `prefill_value` the prefill phase's
causal TFLOP/s.  `roofline` is the kernel with the largest share of the timed region and the other
attention kernel stands beside it (`roofline_decode` or `roofline_prefill`), each with its algorithmic
work per launch / its average launch duration, measured with HIP events the library records on the
launch stream around every 7th launch inside the timed region.

After the timed region the other BASELINE configurations run at their stated sizes (`configs`):
the 70B-scale decode batch (index 3: 256 sequences, 80 distinct layer caches), the 70B-scale phase
switch (index 4: prefill burst of 8 x 8192 tokens into the pool of 192 resident sequences, then 64
decode steps of all 200, per-phase time over 80 layers) and the tiny fp32 cycle (index 0), each with
its roofline figures and the fp64 oracle timed on the host cores on a bounded sample; then decode
batches shaped like the paper's chat workloads (`table4_decode`) and the machine-ceiling probes
(`machine`).  `--only` takes a comma-separated subset of 30b,70b-decode,70b-switch,tiny,table4,machine
(the profiling commands under profiles/ use it).

    python bench.py --sweep

times the kernels alone on further batch shapes over a few layer caches each and prints one JSON line
{"sweep": [...]}.
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

SECTIONS = ("30b", "70b-decode", "70b-switch", "tiny", "table4", "machine")


class Env:
    """Imports, the device and small helpers shared by the sections."""

    def __init__(self):
        import numpy as np
        import torch

        from paper_2504_18154_amd import accounting, binding, build
        from paper_2504_18154_amd import workloads

        if not os.path.exists(binding.LIB_PATH):
            build.build()
        assert torch.cuda.is_available(), "bench.py needs a GPU"
        torch.cuda.set_device(0)
        self.np, self.torch, self.acc, self.binding, self.wl = np, torch, accounting, binding, workloads
        self.dev = torch.device("cuda", 0)
        self._traffic = None

    def i32(self, a):
        return self.torch.as_tensor(self.np.ascontiguousarray(a, dtype=self.np.int32), device=self.dev)

    def fill_randn_(self, t, seed: int):
        g = self.torch.Generator(device=self.dev)
        g.manual_seed(int(seed))
        chunk = 1 << 26
        flat = t.view(-1)
        for o in range(0, flat.numel(), chunk):
            n = min(chunk, flat.numel() - o)
            flat[o:o + n] = self.torch.randn(n, generator=g, device=self.dev, dtype=self.torch.float32).to(t.dtype)

    def event(self):
        return self.torch.cuda.Event(enable_timing=True)

    def free(self):
        import gc
        gc.collect()
        self.torch.cuda.empty_cache()

    def traffic(self, workload: str, kernel: str):
        """HBM bytes per launch from the committed rocprofv3 --pmc runs (profiles/traffic.json), or None."""
        if self._traffic is None:
            try:
                with open(os.path.join(ROOT, "profiles", "traffic.json")) as f:
                    self._traffic = json.load(f)
            except (OSError, ValueError):
                self._traffic = {}
        t = self._traffic.get(workload, {}).get(kernel)
        return None if t is None else t["fetch_bytes_per_launch"] + t["write_bytes_per_launch"]

    def roofline(self, kernel, bound, work, ms_total, launches, workload=None):
        """`work` algorithmic bytes (bound hbm) or FLOPs (bound mfma) per launch; ms_total / launches from HIP events."""
        acc = self.acc
        avg_ms = ms_total / max(launches, 1)
        if bound == "hbm":
            a, peak, unit, key = work / (avg_ms * 1e-3) / 1e9, acc.PEAK_HBM_GBPS, "GB/s", "algorithmic_bytes_per_launch"
        else:
            a, peak, unit, key = work / (avg_ms * 1e-3) / 1e12, acc.PEAK_BF16_TFLOPS, "TFLOP/s", "algorithmic_flops_per_launch"
        tr = self.traffic(workload, kernel) if workload else None
        return {"kernel": kernel, "bound": bound, "achieved": a, "peak": peak, "unit": unit, "frac": a / peak,
                "traffic": tr,
                "traffic_source": ("profiles/traffic.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this workload, "
                                   "committed; not measured in this run") if tr is not None else None,
                "avg_launch_us": avg_ms * 1e3, "launches": launches, key: work}


def time_oracle(fn, min_s: float, min_reps: int = 2):
    """Mean seconds per call of fn over at least min_reps calls and min_s seconds; also fn's last result."""
    reps, t0, out = 0, time.perf_counter(), None
    while reps < min_reps or time.perf_counter() - t0 < min_s:
        out = fn()
        reps += 1
    return (time.perf_counter() - t0) / reps, reps, out


def sample_rows(wl, np, rng, q_len, extra):
    """Query rows {0, 1, 15, 16, S/2, S-2, S-1} plus `extra` random ones per sequence, grouped by sequence."""
    start, tok, pos = [0], [], []
    cu = wl.cu_from_lengths(q_len)
    for b, S in enumerate(q_len):
        S = int(S)
        rows = {0, 1, 15, 16, S // 2, S - 2, S - 1} | set(rng.integers(0, S, size=extra).tolist())
        rows = sorted(r for r in rows if 0 <= r < S)
        tok += [int(cu[b]) + r for r in rows]
        pos += rows
        start.append(len(tok))
    return np.asarray(start, np.int32), np.asarray(tok, np.int32), np.asarray(pos, np.int32)


def max_mean_err(got, ref):
    import numpy as np
    err = np.abs(got.double().cpu().numpy() - ref)
    return float(err.max()), float(err.mean())


# ------------------------------------------------------------------------------------------------
# the timed step: 30B-scale prefill-only batch, then decode-only batch (BASELINE configs index 2, 1)
# ------------------------------------------------------------------------------------------------
def run_30b(E: Env, args, res: dict):
    np, torch, acc, binding, wl = E.np, E.torch, E.acc, E.binding, E.wl
    dev, i32 = E.dev, E.i32
    model = wl.M30B
    layers = args.layers or model.layers
    do_dec = args.phase in ("both", "decode")
    do_pre = args.phase in ("both", "prefill")

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
                E.fill_randn_(kc, db.seed + 10 * l)
                E.fill_randn_(vc, db.seed + 10 * l + 1)
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
    p_out = torch.empty((pb.T, model.Hq, model.D), dtype=torch.bfloat16, device=dev)
    if args.fused_qkv:
        p_q, p_k, p_v = fuse(p_q, p_k, p_v)
    append = (lambda c: c.kv_append_strided) if args.fused_qkv else (lambda c: c.kv_append)
    prefill = pctx.attn_prefill_strided if args.fused_qkv else pctx.attn_prefill
    decode = dctx.attn_decode_strided if args.fused_qkv else dctx.attn_decode
    # chunked prefill: chunk ci holds tokens [ci C, ci C + C) of every prompt that is that long
    p_chunks = []
    reread_tokens = 0     # cached K/V tokens a chunk's queries read again (summed over chunks, one layer)
    if args.prefill_chunk > 0:
        C = args.prefill_chunk
        for ci in range((pb.max_q_len + C - 1) // C):
            lens = np.clip(pb.q_len.astype(np.int64) - ci * C, 0, C)
            idx = np.concatenate([np.arange(pb.cu_q[b] + ci * C, pb.cu_q[b] + ci * C + lens[b]) for b in range(pb.B)])
            sel = torch.as_tensor(idx, device=dev, dtype=torch.long)
            before = np.minimum(pb.q_len, ci * C) + pb.ctx_before
            reread_tokens += int(before[lens > 0].sum())
            p_chunks.append(dict(q=p_q[sel].contiguous(), k=p_k[sel].contiguous(), v=p_v[sel].contiguous(),
                                 out=torch.empty((len(idx), model.Hq, model.D), dtype=torch.bfloat16, device=dev),
                                 cu=i32(wl.cu_from_lengths(lens)), before=i32(before), max_len=int(lens.max())))

    def step(timers=None):
        t = [E.event() for _ in range(3)]
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
    for c in (dctx, pctx):
        c.set_option(binding.OPT_PROFILE, 0)

    # ---------------- algorithmic work --------------------------------------------------
    dec_bytes_layer = acc.decode_bytes(db.ctx_len, model.Hq, model.Hkv, model.D, model.bs)
    pre_flops_layer = acc.prefill_flops_causal(pb.q_len, model.Hq, model.D)
    pre_app_bytes_layer = acc.append_bytes(pb.T, model.Hkv, model.D)

    def rate(x, ms):
        return x / (ms * 1e-3) if ms and ms > 0 else None

    res.update({
        "ms_per_step": wall_ms / args.steps,
        "config": {
            "workload": "30B-scale PaDG step (BASELINE configs index 2 then 1): prefill-only batch (16 prompts, lognormal "
                        "mean 1024 in [128,4096]) then decode-only batch (128 seqs, ctx U[512,4096]); 40 q heads / 8 kv "
                        "heads / D 128 / block 16; append + attention per layer; the other BASELINE configurations "
                        "follow under `configs`",
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
    })
    roofs = {}
    if do_dec:
        # phase time includes the one-token appends (fused or not) and the merge kernels: whole decode phase
        res["value"] = rate(dec_bytes_layer * layers, dec_ms) / 1e9
        res["decode"] = {
            "ms_per_layer": dec_ms / layers, "phase_ms": dec_ms, "GBps": res["value"],
            "frac_of_hbm_peak": res["value"] / acc.PEAK_HBM_GBPS,
            "append_us_per_layer": 1e3 * k_dapp_ms / k_dapp_n if k_dapp_n else None,
        }
        roofs["decode"] = E.roofline("decode_mfma_kernel", "hbm", dec_bytes_layer, k_dec_ms, k_dec_n,
                                     "30b_step" if layers == model.layers else None)
        roofs["decode"]["kernel_ms_per_step"] = k_dec_ms / max(k_dec_n, 1) * layers
    if do_pre:
        tf = rate(pre_flops_layer * layers, pre_ms) / 1e12
        calls = max(1, len(p_chunks))  # hot calls per layer (chunked prefill: one per chunk)
        res["prefill_value"], res["prefill_unit"] = tf, "TFLOP/s"
        r = E.roofline("prefill_mfma_kernel", "mfma", pre_flops_layer / calls, k_pre_ms, k_pre_n,
                       "30b_step" if layers == model.layers and calls == 1 else None)
        r["kernel_ms_per_step"] = k_pre_ms / max(k_pre_n, 1) * calls * layers
        roofs["prefill"] = r
        a = E.roofline("kv_append_kernel", "hbm", pre_app_bytes_layer / calls, k_papp_ms, k_papp_n,
                       "30b_step" if layers == model.layers and calls == 1 else None)
        res["prefill"] = {
            "value": tf, "unit": "TFLOP/s", "ms_per_layer": pre_ms / layers, "phase_ms": pre_ms,
            "frac_of_bf16_peak": tf / acc.PEAK_BF16_TFLOPS,
            "chunk_tokens": args.prefill_chunk, "calls_per_layer": calls,
            "kernel_us_per_layer": calls * 1e3 * k_pre_ms / max(k_pre_n, 1),
            "append": {"GBps": a["achieved"], "avg_launch_us": a["avg_launch_us"], "frac_of_hbm_peak": a["frac"],
                       "us_per_layer": calls * a["avg_launch_us"]},
        }
        if p_chunks:
            # chunked prefill reads the cached prefix of every prompt again with every chunk (Section 2.4.1)
            res["prefill"]["kv_bytes_reread_per_layer"] = reread_tokens * model.kv_bytes_per_token_layer
            res["prefill"]["kv_bytes_new_per_layer"] = pb.T * model.kv_bytes_per_token_layer
        roofs["append"] = a
        if not do_dec:
            res["value"], res["unit"] = tf, "TFLOP/s"
    # the kernel with the largest share of the timed region leads; the other attention kernel stands beside it
    order = sorted((k for k in ("prefill", "decode") if k in roofs), key=lambda k: -roofs[k]["kernel_ms_per_step"])
    for k in order:
        roofs[k]["share_of_timed_region"] = roofs[k]["kernel_ms_per_step"] / (wall_ms / args.steps)
    if order:
        res["roofline"] = roofs[order[0]]
        for k in order[1:]:
            res["roofline_" + k] = roofs[k]
    if "append" in roofs:
        res["roofline_append"] = roofs["append"]

    # ---------------- CPU baseline: the oracle on one decode layer, and on sampled prefill rows ------
    if not args.no_cpu_baseline and (do_dec or do_pre):
        from oracle import oracle as orc
        if do_dec:
            shape = orc.Shape(model.Hq, model.Hkv, model.D, model.bs, db.num_blocks, orc.BF16)
            okc, ovc = orc.new_cache(shape)
            orc.kv_append(shape, okc, ovc, wl.to_bits(stream_k), wl.to_bits(stream_v), wl.cu_from_lengths(db.ctx_len),
                          np.zeros(db.B, dtype=np.int32), db.block_table)
            qh = wl.to_bits(d_q.contiguous())
            cpu_s, reps, (ref, _) = time_oracle(lambda: orc.attn_decode(shape, qh, okc, ovc, db.block_table, db.ctx_len), 1.5, 3)
            mx, mean = max_mean_err(d_out[0], ref)
            res["cpu_baseline"] = {
                "value": dec_bytes_layer / cpu_s / 1e9, "unit": "GB/s", "cores": orc.num_threads(), "kind": "oracle",
                "sample": f"one full layer of the decode batch (128 seqs, {int(db.ctx_len.sum())} cached tokens), "
                          f"fp64, {reps} repetitions, {cpu_s:.3f} s each",
                "seconds": cpu_s, "gpu_vs_oracle_layer0_max_abs": mx, "gpu_vs_oracle_layer0_mean_abs": mean,
            }
            del okc, ovc
        if do_pre and not p_chunks and not args.fused_qkv:
            shape = orc.Shape(model.Hq, model.Hkv, model.D, model.bs, pb.num_blocks, orc.BF16)
            okc, ovc = orc.new_cache(shape)
            orc.kv_append(shape, okc, ovc, wl.to_bits(p_k), wl.to_bits(p_v), pb.cu_q, pb.ctx_before, pb.block_table)
            start, tok, pos = sample_rows(wl, np, wl.rng_for(1), pb.q_len, 16)
            qh = wl.to_bits(p_q)
            cpu_s, reps, (ref, _) = time_oracle(
                lambda: orc.attn_rows(shape, qh, okc, ovc, pb.block_table, start, tok, pos), 1.0, 2)
            sample_flops = 4 * model.Hq * model.D * int((pos.astype(np.int64) + 1).sum())
            sel = torch.as_tensor(tok, dtype=torch.long, device=dev)
            mx, mean = max_mean_err(p_out[sel], ref)
            res["prefill"]["cpu_baseline"] = {
                "value": sample_flops / cpu_s / 1e12, "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
                "sample": f"{len(tok)} sampled query rows of the {pb.B} prompts (all heads), fp64, {reps} repetitions, "
                          f"{cpu_s:.3f} s each = {sample_flops / 1e9:.2f} GFLOP of the layer's {pre_flops_layer / 1e9:.1f}",
                "extrapolated": True, "seconds_one_layer_extrapolated": cpu_s * pre_flops_layer / sample_flops,
                "gpu_vs_oracle_sampled_rows_max_abs": mx, "gpu_vs_oracle_sampled_rows_mean_abs": mean,
            }
    dctx.close()
    pctx.close()
    return dec_bytes_layer


# ------------------------------------------------------------------------------------------------
# BASELINE config index 3: 70B-scale decode-only batch, 80 distinct layer caches
# ------------------------------------------------------------------------------------------------
def run_70b_decode(E: Env, args):
    np, torch, acc, binding, wl = E.np, E.torch, E.acc, E.binding, E.wl
    dev, i32 = E.dev, E.i32
    db = wl.config4_decode_70b()
    m = db.model
    layers = args.layers or m.layers
    pool_elems = db.num_blocks * m.Hkv * m.bs * m.D
    need = layers * 2 * pool_elems * 2
    free_b, _ = torch.cuda.mem_get_info()
    # all layer caches at once if they fit beside the inputs; else two halves with distinct data, one after the other
    groups = 1 if need + (6 << 30) <= free_b else 2
    per_group = (layers + groups - 1) // groups
    ctx = binding.Context(m.Hq, m.Hkv, m.D, db.num_blocks, "bf16", db.B, db.block_table.shape[1])
    if not args.equal_shares:
        ctx.set_option(binding.OPT_DECODE_ADAPTIVE, 1)
    bt, cl = i32(db.block_table), i32(db.ctx_len)
    q = wl.randn((db.B, m.Hq, m.D), "bf16", db.seed + 3, device=dev)
    kn = wl.randn((db.B, m.Hkv, m.D), "bf16", db.seed + 4, device=dev)
    vn = wl.randn((db.B, m.Hkv, m.D), "bf16", db.seed + 5, device=dev)
    out = torch.empty((per_group, db.B, m.Hq, m.D), dtype=torch.bfloat16, device=dev)
    pools = [(torch.empty(pool_elems, dtype=torch.bfloat16, device=dev), torch.empty(pool_elems, dtype=torch.bfloat16, device=dev))
             for _ in range(per_group)]
    # layer 0 comes from a token stream the oracle can replay; its new token is the stream's last one
    T0 = int(db.ctx_len.sum())
    stream_k = wl.randn((T0, m.Hkv, m.D), "bf16", db.seed + 1, device=dev)
    stream_v = wl.randn((T0, m.Hkv, m.D), "bf16", db.seed + 2, device=dev)
    last = torch.as_tensor(np.cumsum(db.ctx_len) - 1, device=dev, dtype=torch.long)
    kn0, vn0 = stream_k[last].contiguous(), stream_v[last].contiguous()
    phase_ms, k_ms, k_n, out0 = 0.0, 0.0, 0, None
    passes = max(2, args.steps // 2)
    for g in range(groups):
        n_l = min(per_group, layers - g * per_group)
        for l in range(n_l):
            E.fill_randn_(pools[l][0], db.seed + 1000 * g + 10 * l)
            E.fill_randn_(pools[l][1], db.seed + 1000 * g + 10 * l + 1)
        if g == 0:
            ctx.kv_append(pools[0][0], pools[0][1], stream_k, stream_v, i32(wl.cu_from_lengths(db.ctx_len)),
                          i32(np.zeros(db.B)), bt)

        def one_pass():
            for l in range(n_l):
                k1, v1 = (kn0, vn0) if g == 0 and l == 0 else (kn, vn)
                ctx.attn_decode_append(q, k1, v1, pools[l][0], pools[l][1], bt, cl, out[l], db.max_ctx_len)

        one_pass()   # warm-up
        torch.cuda.synchronize()
        ctx.set_option(binding.OPT_PROFILE, max(1, args.event_every))
        ctx.profile_reset()
        e0, e1 = E.event(), E.event()
        e0.record()
        for _ in range(passes):
            one_pass()
        e1.record()
        torch.cuda.synchronize()
        phase_ms += e0.elapsed_time(e1) / passes
        ms, n = ctx.profile_read(binding.KERNEL_DECODE)
        k_ms, k_n = k_ms + ms, k_n + n
        ctx.set_option(binding.OPT_PROFILE, 0)
        if g == 0:
            out0 = out[0].clone()
    by = acc.decode_bytes(db.ctx_len, m.Hq, m.Hkv, m.D, m.bs)
    gbps = by * layers / (phase_ms * 1e-3) / 1e9
    r = {
        "workload": "BASELINE config index 3: 70B-scale decode-only batch, 256 seqs, ctx U[1024,4096], 64 q / 8 kv heads, "
                    "one decode step across all layers (fused append + decode call per layer)",
        "layers": layers, "layer_caches": "all distinct and resident at once" if groups == 1 else
                  f"{groups} groups of {per_group} distinct caches timed one after the other (all {layers} do not fit beside the inputs)",
        "kv_cache_GB": need / 1e9, "decode_ctx_tokens": T0,
        "ms_per_step": phase_ms, "ms_per_layer": phase_ms / layers, "GBps": gbps, "frac_of_hbm_peak": gbps / acc.PEAK_HBM_GBPS,
        "passes_timed": passes,
        "roofline": E.roofline("decode_mfma_kernel", "hbm", by, k_ms, k_n, "70b_decode" if layers == m.layers else None),
    }
    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        shape = orc.Shape(m.Hq, m.Hkv, m.D, m.bs, db.num_blocks, orc.BF16)
        okc, ovc = orc.new_cache(shape)
        orc.kv_append(shape, okc, ovc, wl.to_bits(stream_k), wl.to_bits(stream_v), wl.cu_from_lengths(db.ctx_len),
                      np.zeros(db.B, dtype=np.int32), db.block_table)
        qh = wl.to_bits(q)
        cpu_s, reps, (ref, _) = time_oracle(lambda: orc.attn_decode(shape, qh, okc, ovc, db.block_table, db.ctx_len), 1.0, 2)
        mx, mean = max_mean_err(out0, ref)
        r["cpu_baseline"] = {"value": by / cpu_s / 1e9, "unit": "GB/s", "cores": orc.num_threads(), "kind": "oracle",
                             "sample": f"one full layer of the batch ({T0} cached tokens), fp64, {reps} repetitions, {cpu_s:.3f} s each; "
                                       f"x {layers} layers (identical in shape) = {cpu_s * layers:.1f} s per step, extrapolated",
                             "seconds": cpu_s, "gpu_vs_oracle_layer0_max_abs": mx, "gpu_vs_oracle_layer0_mean_abs": mean}
    ctx.close()
    return r


# ------------------------------------------------------------------------------------------------
# BASELINE config index 4: 70B-scale temporal-disaggregation switch
# ------------------------------------------------------------------------------------------------
def run_70b_switch(E: Env, args):
    np, torch, acc, binding, wl = E.np, E.torch, E.acc, E.binding, E.wl
    dev, i32 = E.dev, E.i32
    m = wl.M70B
    layers = args.layers or m.layers
    n_steps = args.decode_steps
    resident, q_len, table, nb = wl.config5_switch_70b()
    nres, nnew = len(resident), len(q_len)
    B = nres + nnew
    pool_elems = nb * m.Hkv * m.bs * m.D
    ctx = binding.Context(m.Hq, m.Hkv, m.D, nb, "bf16", B, table.shape[1])
    ctx.set_option(binding.OPT_PREFILL_REUSE_PLAN, 1)
    if not args.equal_shares:
        ctx.set_option(binding.OPT_DECODE_ADAPTIVE, 1)
    pools = []
    for l in range(layers):
        kc = torch.empty(pool_elems, dtype=torch.bfloat16, device=dev)
        vc = torch.empty(pool_elems, dtype=torch.bfloat16, device=dev)
        E.fill_randn_(kc, 7000 + 10 * l)     # the resident sequences' contexts: whatever their blocks hold
        E.fill_randn_(vc, 7001 + 10 * l)
        pools.append((kc, vc))
    # layer 0's resident contexts come from a token stream the oracle can replay
    Tres = int(resident.sum())
    res_k = wl.randn((Tres, m.Hkv, m.D), "bf16", 501, device=dev)
    res_v = wl.randn((Tres, m.Hkv, m.D), "bf16", 502, device=dev)
    ctx.kv_append(pools[0][0], pools[0][1], res_k, res_v, i32(wl.cu_from_lengths(resident)), i32(np.zeros(nres)), i32(table[:nres]))
    # the prefill-only burst
    cu = wl.cu_from_lengths(q_len)
    T = int(cu[-1])
    p_q = wl.randn((T, m.Hq, m.D), "bf16", 505, device=dev)
    p_k = wl.randn((T, m.Hkv, m.D), "bf16", 503, device=dev)
    p_v = wl.randn((T, m.Hkv, m.D), "bf16", 504, device=dev)
    p_out = torch.empty_like(p_q)
    p_cu, p_zero, p_bt = i32(cu), i32(np.zeros(nnew)), i32(table[nres:])
    max_q = int(q_len.max())
    # the decode-only steps: all sequences, contexts one longer with every step
    ctx0 = np.concatenate([resident, q_len]).astype(np.int64)
    lens = torch.as_tensor(np.stack([ctx0 + s + 1 for s in range(n_steps)]).astype(np.int32), device=dev)
    d_bt = i32(table)
    d_q = wl.randn((B, m.Hq, m.D), "bf16", 605, device=dev)
    d_k = wl.randn((B, m.Hkv, m.D), "bf16", 600, device=dev)
    d_v = wl.randn((B, m.Hkv, m.D), "bf16", 601, device=dev)
    d_out = torch.empty((B, m.Hq, m.D), dtype=torch.bfloat16, device=dev)
    d_out_l0 = torch.empty_like(d_out)
    max_ctx = int(ctx0.max()) + n_steps

    def prefill_phase(n_layers):
        ctx.set_option(binding.OPT_PREFILL_REUSE_PLAN, 1)
        for l in range(n_layers):
            kc, vc = pools[l]
            ctx.kv_append(kc, vc, p_k, p_v, p_cu, p_zero, p_bt, max_new_len=max_q)
            ctx.attn_prefill(p_q, kc, vc, p_cu, p_zero, p_bt, p_out, max_q_len=max_q)

    def decode_step(s, n_layers):
        for l in range(n_layers):
            kc, vc = pools[l]
            ctx.attn_decode_append(d_q, d_k, d_v, kc, vc, d_bt, lens[s], d_out_l0 if (s == 0 and l == 0) else d_out, max_ctx)

    # warm-up on a few layers (the timed pass redoes them: same tokens into the same slots)
    prefill_phase(min(4, layers))
    decode_step(0, min(4, layers))
    torch.cuda.synchronize()
    ctx.set_option(binding.OPT_PROFILE, max(1, args.event_every))
    ctx.profile_reset()
    e = [E.event() for _ in range(3)]
    e[0].record()
    prefill_phase(layers)
    e[1].record()
    for s in range(n_steps):
        decode_step(s, layers)
    e[2].record()
    torch.cuda.synchronize()
    pre_ms, dec_ms = e[0].elapsed_time(e[1]), e[1].elapsed_time(e[2])
    k_pre_ms, k_pre_n = ctx.profile_read(binding.KERNEL_PREFILL)
    k_app_ms, k_app_n = ctx.profile_read(binding.KERNEL_APPEND)
    k_dec_ms, k_dec_n = ctx.profile_read(binding.KERNEL_DECODE)
    ctx.set_option(binding.OPT_PROFILE, 0)
    flops = acc.prefill_flops_causal(q_len, m.Hq, m.D)
    app_bytes = acc.append_bytes(T, m.Hkv, m.D)
    dec_bytes = [acc.decode_bytes(ctx0 + s + 1, m.Hq, m.Hkv, m.D, m.bs) for s in range(n_steps)]
    dec_bytes_mean = float(np.mean(dec_bytes))
    pre_kernel_ms = k_pre_ms / max(k_pre_n, 1) * layers
    app_kernel_ms = k_app_ms / max(k_app_n, 1) * layers
    dec_kernel_ms = k_dec_ms / max(k_dec_n, 1) * layers * n_steps
    r = {
        "workload": f"BASELINE config index 4: 70B-scale temporal-disaggregation switch; {nres} resident seqs (ctx U[1024,4096]), "
                    f"prefill-only burst of {nnew} x {int(q_len[0])} tokens appended into the same paged pools, then {n_steps} "
                    f"decode-only steps of all {B}; 64 q / 8 kv heads",
        "layers": layers, "kv_cache_GB": layers * 2 * pool_elems * 2 / 1e9, "layer_caches": "all distinct and resident at once",
        "kernel_events": f"every {max(1, args.event_every)}th launch of each kernel; kernel times below = average launch x launches",
        "phases": {
            "prefill_append": {"kernel_ms_all_layers": app_kernel_ms, "us_per_layer": app_kernel_ms / layers * 1e3,
                               "GBps": app_bytes * layers / (app_kernel_ms * 1e-3) / 1e9,
                               "frac_of_hbm_peak": app_bytes * layers / (app_kernel_ms * 1e-3) / 1e9 / acc.PEAK_HBM_GBPS},
            "prefill_attention": {"kernel_ms_all_layers": pre_kernel_ms, "ms_per_layer": pre_kernel_ms / layers,
                                  "TFLOPs": flops * layers / (pre_kernel_ms * 1e-3) / 1e12,
                                  "frac_of_bf16_peak": flops * layers / (pre_kernel_ms * 1e-3) / 1e12 / acc.PEAK_BF16_TFLOPS},
            "prefill_phase_wall": {"ms_all_layers": pre_ms, "TFLOPs": flops * layers / (pre_ms * 1e-3) / 1e12,
                                   "frac_of_bf16_peak": flops * layers / (pre_ms * 1e-3) / 1e12 / acc.PEAK_BF16_TFLOPS},
            "decode_attention": {"kernel_ms_all_layers_all_steps": dec_kernel_ms, "us_per_layer_per_step": dec_kernel_ms / layers / n_steps * 1e3,
                                 "GBps": dec_bytes_mean * layers * n_steps / (dec_kernel_ms * 1e-3) / 1e9,
                                 "frac_of_hbm_peak": dec_bytes_mean * layers * n_steps / (dec_kernel_ms * 1e-3) / 1e9 / acc.PEAK_HBM_GBPS},
            "decode_phase_wall": {"ms_all_layers_all_steps": dec_ms, "ms_per_step": dec_ms / n_steps, "steps": n_steps,
                                  "GBps": dec_bytes_mean * layers * n_steps / (dec_ms * 1e-3) / 1e9,
                                  "frac_of_hbm_peak": dec_bytes_mean * layers * n_steps / (dec_ms * 1e-3) / 1e9 / acc.PEAK_HBM_GBPS},
        },
        "roofline": E.roofline("prefill_mfma_kernel", "mfma", flops, k_pre_ms, k_pre_n, "70b_switch" if layers == m.layers else None),
        "roofline_decode": E.roofline("decode_mfma_kernel", "hbm", dec_bytes_mean, k_dec_ms, k_dec_n,
                                      "70b_switch" if layers == m.layers else None),
        "roofline_append": E.roofline("kv_append_kernel", "hbm", app_bytes, k_app_ms, k_app_n,
                                      "70b_switch" if layers == m.layers else None),
    }
    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        shape = orc.Shape(m.Hq, m.Hkv, m.D, m.bs, nb, orc.BF16)
        okc, ovc = orc.new_cache(shape)
        orc.kv_append(shape, okc, ovc, wl.to_bits(res_k), wl.to_bits(res_v), wl.cu_from_lengths(resident), np.zeros(nres, np.int32), table[:nres])
        orc.kv_append(shape, okc, ovc, wl.to_bits(p_k), wl.to_bits(p_v), cu, np.zeros(nnew, np.int32), table[nres:])
        # prefill: sampled rows of the burst, extrapolated by FLOP ratio
        start, tok, pos = sample_rows(wl, np, wl.rng_for(2), q_len, 4)
        qh = wl.to_bits(p_q)
        cpu_s, reps, (ref, _) = time_oracle(lambda: orc.attn_rows(shape, qh, okc, ovc, table[nres:], start, tok, pos), 1.0, 1)
        sample_flops = 4 * m.Hq * m.D * int((pos.astype(np.int64) + 1).sum())
        # (p_out holds the last layer's output; layer 0 saw the same q and the same burst, and keys of other sequences do not matter)
        ctx.attn_prefill(p_q, pools[0][0], pools[0][1], p_cu, p_zero, p_bt, p_out, max_q_len=max_q)
        torch.cuda.synchronize()
        mx, mean = max_mean_err(p_out[torch.as_tensor(tok, dtype=torch.long, device=dev)], ref)
        r["cpu_baseline_prefill"] = {
            "value": sample_flops / cpu_s / 1e12, "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"{len(tok)} sampled query rows of the burst (all heads), fp64, {reps} repetitions, {cpu_s:.3f} s each = "
                      f"{sample_flops / 1e9:.2f} GFLOP of the layer's {flops / 1e9:.0f}",
            "extrapolated": True, "seconds_one_layer_extrapolated": cpu_s * flops / sample_flops,
            "gpu_vs_oracle_sampled_rows_max_abs": mx, "gpu_vs_oracle_sampled_rows_mean_abs": mean}
        # decode: step 0 of layer 0 in full
        ones = wl.cu_from_lengths([1] * B)
        orc.kv_append(shape, okc, ovc, wl.to_bits(d_k), wl.to_bits(d_v), ones, ctx0.astype(np.int32), table)
        l1 = (ctx0 + 1).astype(np.int32)
        qh = wl.to_bits(d_q)
        cpu_s, reps, (ref, _) = time_oracle(lambda: orc.attn_decode(shape, qh, okc, ovc, table, l1), 1.0, 2)
        mx, mean = max_mean_err(d_out_l0, ref)
        r["cpu_baseline_decode"] = {
            "value": dec_bytes[0] / cpu_s / 1e9, "unit": "GB/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"one decode step of one layer in full ({B} seqs, {int(l1.sum())} cached tokens), fp64, {reps} repetitions, {cpu_s:.3f} s each",
            "seconds": cpu_s, "gpu_vs_oracle_layer0_step0_max_abs": mx, "gpu_vs_oracle_layer0_step0_mean_abs": mean}
    ctx.close()
    return r


# ------------------------------------------------------------------------------------------------
# BASELINE config index 0: the tiny fp32 PaDG cycle (a correctness configuration: launch-bound)
# ------------------------------------------------------------------------------------------------
def run_tiny(E: Env, args):
    np, torch, binding, wl = E.np, E.torch, E.binding, E.wl
    dev, i32 = E.dev, E.i32
    pb = wl.config1_tiny()
    m = pb.model
    ctx = binding.Context(m.Hq, m.Hkv, m.D, pb.num_blocks, m.dtype, pb.B, pb.block_table.shape[1])
    bt = i32(pb.block_table)
    q, k, v = (wl.randn((pb.T, h, m.D), m.dtype, wl.config_seed(1) + i) for i, h in enumerate((m.Hq, m.Hkv, m.Hkv)))
    steps = [tuple(wl.randn((2, h, m.D), m.dtype, wl.config_seed(1) + 10 * (s + 1) + i) for i, h in enumerate((m.Hq, m.Hkv, m.Hkv)))
             for s in range(8)]
    gq, gk, gv = q.to(dev), k.to(dev), v.to(dev)
    gsteps = [tuple(t.to(dev) for t in st) for st in steps]
    cu, cb = i32(pb.cu_q), i32(pb.ctx_before)
    ones = i32(wl.cu_from_lengths([1, 1]))
    lens = [i32(pb.q_len + s) for s in range(9)]
    out_p = torch.empty_like(gq)
    outs = [torch.empty_like(gsteps[0][0]) for _ in range(8)]

    def cycle():
        kc, vc = cache
        ctx.kv_append(kc, vc, gk, gv, cu, cb, bt)
        ctx.attn_prefill(gq, kc, vc, cu, cb, bt, out_p, max_q_len=pb.max_q_len)
        for s in range(8):
            ctx.kv_append(kc, vc, gsteps[s][1], gsteps[s][2], ones, lens[s], bt, max_new_len=1)
            ctx.attn_decode(gsteps[s][0], kc, vc, bt, lens[s + 1], outs[s], int(pb.q_len.max()) + s + 1)

    cache = ctx.new_cache()
    cycle()
    torch.cuda.synchronize()
    e0, e1 = E.event(), E.event()
    reps = 20
    e0.record()
    for _ in range(reps):
        cycle()
    e1.record()
    torch.cuda.synchronize()
    gpu_ms = e0.elapsed_time(e1) / reps
    r = {"workload": "BASELINE config index 0: tiny PaDG cycle, fp32, 4 q / 2 kv heads, D 64: prefill-only batch (37 + 100 tokens), "
                     "then 8 decode-only steps (plain kernels; 18 launches, launch-bound by construction)",
         "gpu_ms_per_cycle": gpu_ms, "launches_per_cycle": 18, "roofline": None}
    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        shape = orc.Shape(m.Hq, m.Hkv, m.D, m.bs, pb.num_blocks, orc.F32)

        def oracle_cycle():
            okc, ovc = orc.new_cache(shape)
            orc.kv_append(shape, okc, ovc, wl.to_bits(k), wl.to_bits(v), pb.cu_q, pb.ctx_before, pb.block_table)
            ref = [orc.attn_prefill(shape, wl.to_bits(q), okc, ovc, pb.cu_q, pb.ctx_before, pb.block_table)[0]]
            for s in range(8):
                orc.kv_append(shape, okc, ovc, wl.to_bits(steps[s][1]), wl.to_bits(steps[s][2]), wl.cu_from_lengths([1, 1]),
                              pb.q_len + s, pb.block_table)
                ref.append(orc.attn_decode(shape, wl.to_bits(steps[s][0]), okc, ovc, pb.block_table, pb.q_len + s + 1)[0])
            return ref

        cpu_s, n, ref = time_oracle(oracle_cycle, 0.5, 3)
        errs = [max_mean_err(out_p, ref[0])[0]] + [max_mean_err(outs[s], ref[s + 1])[0] for s in range(8)]
        r["cpu_baseline"] = {"value": cpu_s * 1e3, "unit": "ms per cycle", "cores": orc.num_threads(), "kind": "oracle",
                             "sample": f"the whole cycle in full, fp64, {n} repetitions", "gpu_vs_oracle_max_abs": max(errs)}
    ctx.close()
    return r


# ------------------------------------------------------------------------------------------------
# decode batches shaped like the paper's chat workloads (Table 4) and a small batch
# ------------------------------------------------------------------------------------------------
def time_decode_batch(E: Env, name, db, layers=4, warm_ms=60.0, timed_ms=60.0):
    np, torch, acc, binding, wl = E.np, E.torch, E.acc, E.binding, E.wl
    m = db.model
    ctx = binding.Context(m.Hq, m.Hkv, m.D, db.num_blocks, "bf16", db.B, db.block_table.shape[1])
    ctx.set_option(binding.OPT_DECODE_ADAPTIVE, 1)
    g = torch.Generator(device=E.dev)
    g.manual_seed(db.seed)
    n_elems = db.num_blocks * m.Hkv * m.bs * m.D
    mk = lambda: torch.randn(n_elems, generator=g, device=E.dev, dtype=torch.float32).to(torch.bfloat16)
    caches = [(mk(), mk()) for _ in range(layers)]
    q = wl.randn((db.B, m.Hq, m.D), "bf16", db.seed + 3, device=E.dev)
    out = torch.empty_like(q)
    bt, cl = E.i32(db.block_table), E.i32(db.ctx_len)

    def one_pass():
        for kc, vc in caches:
            ctx.attn_decode(q, kc, vc, bt, cl, out, db.max_ctx_len)

    for phase_ms, bracket in ((warm_ms, False), (timed_ms, True)):
        if bracket:
            ctx.set_option(binding.OPT_PROFILE, 1)
            ctx.profile_reset()
        t0, n = time.perf_counter(), 0
        while n < 3 or (time.perf_counter() - t0) * 1e3 < phase_ms:
            one_pass()
            torch.cuda.synchronize()
            n += 1
    ms, n = ctx.profile_read(binding.KERNEL_DECODE)
    by = acc.decode_bytes(db.ctx_len, m.Hq, m.Hkv, m.D, m.bs)
    rate = by / (ms / n * 1e-3) / 1e9
    ctx.close()
    return {"workload": name, "kernel": "decode_mfma_kernel", "avg_launch_us": ms / n * 1e3, "launches": n,
            "algorithmic_bytes_per_launch": by, "GBps": rate, "frac_of_hbm_peak": rate / acc.PEAK_HBM_GBPS}


def run_table4(E: Env, args):
    wl = E.wl
    return [
        time_decode_batch(E, "30B heads, 1024 seqs, contexts shaped like Alpaca (Table 4)", wl.table4_decode_batch(wl.M30B, "alpaca", 1024, 22)),
        time_decode_batch(E, "30B heads, 512 seqs, contexts shaped like ShareGPT (Table 4)", wl.table4_decode_batch(wl.M30B, "sharegpt", 512, 21)),
        time_decode_batch(E, "30B heads, 64 seqs, contexts shaped like LongBench (Table 4)", wl.table4_decode_batch(wl.M30B, "longbench", 64, 23)),
        time_decode_batch(E, "30B heads, 16 seqs, ctx U[512,4096] (small batch)", wl.decode_batch(wl.M30B, 16, 512, 4096, 6)),
    ]


def run_machine(E: Env, dec_bytes_layer):
    b = E.binding
    m = {
        "hbm_read_GBps": b.probe_hbm_read(4 << 30, reps=5),
        "mfma_bf16_TFLOPs": b.probe_mfma_bf16(False, reps=5),
        "mfma_bf16_random_operands_TFLOPs": b.probe_mfma_bf16(True, reps=5),
        "how": "after the timed region: 4 GiB (and as many bytes as one decode launch reads) read in 8 KiB pieces per "
               "wavefront, 16-byte non-temporal loads; register-only 32x32x16 bf16 loop, "
               "4 wavefronts per SIMD, smooth and pseudo-random operands; 5 launches each after one untimed",
    }
    if dec_bytes_layer:
        m["hbm_read_same_bytes_GBps"] = b.probe_hbm_read(int(dec_bytes_layer) // 8192 * 8192, reps=20)
    # what a plain device copy moves (read + written bytes per second) at the two sizes kv_append handles in the
    # prefill workloads: the append is such a pass (every new K/V byte read once and written once) plus a scatter.
    # As in the benchmark, the source is the same every time and the destination never (a ring of buffers larger
    # than the 256 MB last-level cache).
    torch = E.torch
    for tag, T in (("30b_prefill_batch", 15385), ("8x8192_burst", 65536)):
        n = T * 8 * 128 * 2          # elements of K and V rows together (bf16)
        src = torch.empty(n, dtype=torch.bfloat16, device=E.dev).normal_()
        ring = [torch.empty_like(src) for _ in range(max(3, (1 << 30) // (2 * n) + 1))]
        for dst in ring[:3]:
            dst.copy_(src)
        e0, e1 = E.event(), E.event()
        reps = max(20, len(ring))
        e0.record()
        for i in range(reps):
            ring[i % len(ring)].copy_(src)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / reps * 1e3
        m["plain_copy_" + tag] = {"bytes_read_plus_written": 4 * n, "us": us, "GBps": 4 * n / (us * 1e-6) / 1e9}
        del src, ring
    # how much vector work the matrix cores hide: ns one SIMD spends per slot of one matrix instruction plus the
    # given v_fma_f32 / v_exp_f32 (two wavefronts per SIMD, registers only); the prefill kernel's softmax is
    # about 3.5 plain vector instructions and one v_exp_f32 per matrix instruction
    rows = []
    for mf, f, e in ((1, 0, 0), (1, 2, 0), (1, 4, 0), (1, 8, 0), (1, 0, 2), (1, 2, 2), (1, 4, 2), (0, 4, 2), (0, 8, 0)):
        clocks, ghz = b.probe_mfma_valu(bool(mf), f, e, 2)
        rows.append({"mfma": mf, "fma": f, "exp": e, "clocks_per_slot": clocks, "ghz": ghz, "ns_per_slot": clocks / ghz if ghz else None})
    m["mfma_valu_slots"] = rows
    base = rows[0]["ns_per_slot"]
    m["matrix_core_share_with_softmax_like_work"] = base / rows[6]["ns_per_slot"] if base and rows[6]["ns_per_slot"] else None
    return m


def sweep() -> int:
    """Kernel time and rate on other batch shapes, a few layer caches each, all launches bracketed."""
    E = Env()
    np, torch, acc, binding, wl = E.np, E.torch, E.acc, E.binding, E.wl
    dev, i32 = E.dev, E.i32
    rows = []

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
        rows.append(time_decode_batch(E, name, db, layers))

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
    ap.add_argument("--only", default=",".join(SECTIONS),
                    help="comma-separated sections to run: " + ", ".join(SECTIONS) + " (default: all; the JSON line keeps its "
                         "top-level contract fields only if 30b is among them)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debugging only; invalid as a result)")
    ap.add_argument("--decode-steps", type=int, default=64, help="decode-only steps of the 70B phase switch (64 is the configuration's)")
    ap.add_argument("--split-tokens", type=int, default=0, help="force the decode split size (tuning)")
    ap.add_argument("--prefill-chunk", type=int, default=0,
                    help="process every prompt in chunks of this many tokens (each chunk attends to the cached prefix "
                         "of its prompt): quantifies the repeated K/V reads of chunked prefill; 0 = whole prompts")
    ap.add_argument("--equal-shares", action="store_true",
                    help="decode with equal chunks per wavefront instead of per-XCD shares that follow measured speeds")
    ap.add_argument("--phase", choices=["both", "decode", "prefill"], default="both",
                    help="30b section: run only one phase (profiling runs; the default is the full step)")
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
    ap.add_argument("--no-probes", action="store_true", help="same as leaving `machine` out of --only")
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
    only = [s.strip() for s in args.only.split(",") if s.strip()]
    bad = [s for s in only if s not in SECTIONS]
    if bad:
        print(f"bench.py: unknown section(s) {bad}; choose from {SECTIONS}", file=sys.stderr)
        return 2
    if args.no_probes and "machine" in only:
        only.remove("machine")
    special = args.prefill_chunk or args.fused_qkv or args.phase != "both" or args.layers
    if special and args.only == ",".join(SECTIONS):
        only = ["30b"]      # an experiment on the timed step: the other sections would only take time

    E = Env()
    if args.calibration_copy:
        src = E.torch.empty(1 << 29, dtype=E.torch.bfloat16, device=E.dev).normal_()
        dst = E.torch.empty_like(src)
        dst.copy_(src)   # 1 GiB read + 1 GiB written by a plain copy kernel
        E.torch.cuda.synchronize()
        del src, dst
        E.free()
    res = {
        "metric": "decode attn HBM GB/s + prefill attn TFLOP/s, % of MI355X roofline",
        "value": None, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": None, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic", "sections": only,
    }
    dec_bytes_layer = None
    if "30b" in only:
        dec_bytes_layer = run_30b(E, args, res)
        E.free()
    configs = {}
    if "70b-decode" in only:
        configs["3_70b_decode"] = run_70b_decode(E, args)
        E.free()
    if "70b-switch" in only:
        configs["4_70b_switch"] = run_70b_switch(E, args)
        E.free()
    if "tiny" in only:
        configs["0_tiny_fp32"] = run_tiny(E, args)
    if configs:
        res["configs"] = configs
    if "table4" in only:
        res["table4_decode"] = run_table4(E, args)
        E.free()
    if "machine" in only:
        res["machine"] = run_machine(E, dec_bytes_layer)
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
