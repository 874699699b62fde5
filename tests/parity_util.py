"""Shared plumbing of the GPU parity tests: run one layer's cache through both the HIP
library (via the C ABI binding) and the CPU oracle on the same seeded inputs."""
from __future__ import annotations

import sys

import numpy as np
import torch

from oracle import oracle as orc
from paper_2504_18154_amd import workloads as wl

# Tolerances (outputs, GPU vs fp64 oracle).  bf16 inputs, fp32 accumulation: the stated
# bar.  fp32: derived from fp32 accumulation over a few hundred keys plus exp2 error,
# with two orders of magnitude of headroom.
TOL = {"bf16": (1e-2, 1e-3), "f32": (1e-4, 1e-5)}
# log-sum-exp (natural log).  The prefill kernel sums the bf16-rounded weights (the same
# values the second product consumes), so the row sum carries a relative error of at most
# half a bf16 spacing, 2^-9 = 1.95e-3, which is also the bound on the error of its log.
LSE_TOL = {"bf16": 2.5e-3, "f32": 1e-4}


def say(msg: str):
    print(msg, flush=True)
    sys.stdout.flush()


def dev_i32(a):
    return torch.as_tensor(np.ascontiguousarray(a, dtype=np.int32), device="cuda")


class Layer:
    """One layer's paged cache held twice: by the HIP library (device) and by the oracle (host)."""

    def __init__(self, model: wl.ModelShape, num_blocks: int, max_batch: int, max_blocks_per_seq: int,
                 oracle_cache: bool = True):
        from paper_2504_18154_amd import binding
        self.model = model
        self.ctx = binding.Context(model.Hq, model.Hkv, model.D, num_blocks, model.dtype, max_batch,
                                   max_blocks_per_seq)
        self.kc, self.vc = self.ctx.new_cache()
        dt = orc.BF16 if model.dtype == "bf16" else orc.F32
        self.shape = orc.Shape(model.Hq, model.Hkv, model.D, model.bs, num_blocks, dt)
        if oracle_cache:
            self.okc, self.ovc = orc.new_cache(self.shape)

    def append(self, k_new: torch.Tensor, v_new: torch.Tensor, cu_q, ctx_before, table, max_new_len=None):
        """k_new/v_new: tensors on any device; the same bits go to both sides."""
        kd, vd = k_new.cuda(), v_new.cuda()
        self.ctx.kv_append(self.kc, self.vc, kd, vd, dev_i32(cu_q), dev_i32(ctx_before), dev_i32(table),
                           max_new_len=max_new_len)
        orc.kv_append(self.shape, self.okc, self.ovc, wl.to_bits(k_new), wl.to_bits(v_new), cu_q, ctx_before, table)

    def assert_cache_bit_exact(self):
        torch.cuda.synchronize()
        gk = wl.to_bits(self.ctx.k_logical(self.kc))
        gv = wl.to_bits(self.ctx.v_logical(self.vc))
        if self.model.dtype == "f32":
            assert np.array_equal(gk.view(np.uint32), self.okc.view(np.uint32)), "K pool differs from the oracle's"
            assert np.array_equal(gv.view(np.uint32), self.ovc.view(np.uint32)), "V pool differs from the oracle's"
        else:
            assert np.array_equal(gk, self.okc), "K pool differs from the oracle's"
            assert np.array_equal(gv, self.ovc), "V pool differs from the oracle's"

    def prefill_gpu(self, q: torch.Tensor, cu_q, ctx_before, table, max_q_len=None):
        qd = q.cuda()
        out = torch.full_like(qd, float("nan"))
        lse = torch.full(qd.shape[:2], float("nan"), dtype=torch.float32, device="cuda")
        if max_q_len is None:
            max_q_len = int(np.max(np.diff(cu_q))) if len(cu_q) > 1 else 0
        self.ctx.attn_prefill(qd, self.kc, self.vc, dev_i32(cu_q), dev_i32(ctx_before), dev_i32(table), out, lse,
                              max_q_len=max_q_len)
        torch.cuda.synchronize()
        return out, lse

    def decode_gpu(self, q: torch.Tensor, table, ctx_len, max_ctx_len=None):
        qd = q.cuda()
        out = torch.full_like(qd, float("nan"))
        lse = torch.full(qd.shape[:2], float("nan"), dtype=torch.float32, device="cuda")
        if max_ctx_len is None:
            max_ctx_len = int(np.max(ctx_len))
        self.ctx.attn_decode(qd, self.kc, self.vc, dev_i32(table), dev_i32(ctx_len), out, max_ctx_len, lse)
        torch.cuda.synchronize()
        return out, lse

    def prefill_oracle(self, q, cu_q, ctx_before, table):
        return orc.attn_prefill(self.shape, wl.to_bits(q), self.okc, self.ovc, cu_q, ctx_before, table)

    def decode_oracle(self, q, table, ctx_len):
        return orc.attn_decode(self.shape, wl.to_bits(q), self.okc, self.ovc, table, ctx_len)

    def close(self):
        self.ctx.close()


def bf16_ulp(x: np.ndarray) -> np.ndarray:
    """Spacing of bf16 numbers (8 significant bits) at |x|."""
    ax = np.maximum(np.abs(x), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(ax)) - 7)


def compare(name, got: torch.Tensor, ref: np.ndarray, dtype: str, rows=None):
    """max-abs and mean-abs error of GPU output vs the fp64 oracle.

    bf16 outputs: the stated bounds are 1e-2 max-abs and 1e-3 mean-abs.  A bf16 number
    with |o| >= 2 has spacing >= 2^-6 > 1e-2, so there the nearest representable value can
    already miss the exact one by up to 0.0078 (|o| < 4) or 0.0156 (|o| < 8); such elements
    (a handful: short contexts, where the output is close to a single large V entry) are
    held to one bf16 spacing of the exact value instead.  Their count is printed."""
    if rows is not None:   # select on the device first: full outputs can be gigabytes
        got = got[torch.as_tensor(np.asarray(rows), dtype=torch.long, device=got.device)]
    g = got.detach().double().cpu().numpy()
    assert g.shape == ref.shape, (g.shape, ref.shape)
    assert np.all(np.isfinite(g)), f"{name}: non-finite values in the GPU output"
    err = np.abs(g - ref)
    mx, mean = float(err.max()) if err.size else 0.0, float(err.mean()) if err.size else 0.0
    tmax, tmean = TOL[dtype]
    bound = np.full(ref.shape, tmax)
    coarse = 0
    if dtype == "bf16":
        bound = np.maximum(bound, bf16_ulp(ref))
        coarse = int((np.abs(ref) >= 2.0).sum())
    worst = float((err / bound).max()) if err.size else 0.0
    say(f"  {name}: max-abs {mx:.3e} (<= {tmax:g}; {coarse} of {ref.size} elements with |o| >= 2 held to one "
        f"bf16 spacing; worst err/bound {worst:.2f})  mean-abs {mean:.3e} (<= {tmean:g})")
    assert np.all(err <= bound) and mean <= tmean, f"{name}: max-abs {mx:.3e}, mean-abs {mean:.3e}, worst {worst:.2f}"
    return mx, mean


def compare_lse(name, got: torch.Tensor, ref: np.ndarray, dtype: str, rows=None):
    if rows is not None:
        got = got[torch.as_tensor(np.asarray(rows), dtype=torch.long, device=got.device)]
    g = got.detach().double().cpu().numpy()
    err = float(np.abs(g - ref).max()) if ref.size else 0.0
    say(f"  {name}: lse max-abs {err:.3e} (<= {LSE_TOL[dtype]:g})")
    assert err <= LSE_TOL[dtype], f"{name}: lse error {err:.3e}"
