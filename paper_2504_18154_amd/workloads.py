"""Seeded synthetic inputs for the paged-attention hot path.

This module only draws shapes, lengths, block tables and N(0,1) tensors.  It
holds none of the method's arithmetic and is the single piece of code that
both the GPU tests/benchmark and the CPU oracle's tests draw their inputs
from.  It imports neither the GPU binding nor the oracle.

The workloads stand in for the paper's Alpaca-gpt4 / ShareGPT / LongBench
traces (Section 4.1, Table 4; prompts truncated to 4096 tokens): attention
cost depends only on sequence lengths and head shapes, so lengths are drawn
from seeded distributions of matching range and skew, and Q/K/V are i.i.d.
N(0,1) rounded to the storage type.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np
import torch

BLOCK_SIZE = 16


@dataclass(frozen=True)
class ModelShape:
    name: str
    Hq: int
    Hkv: int
    D: int
    layers: int
    dtype: str  # "bf16" | "f32"
    bs: int = BLOCK_SIZE

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    @property
    def kv_bytes_per_token_layer(self) -> int:
        return 2 * self.Hkv * self.D * self.elem_bytes


TINY = ModelShape("tiny-fp32", Hq=4, Hkv=2, D=64, layers=1, dtype="f32")
M30B = ModelShape("30B-scale", Hq=40, Hkv=8, D=128, layers=64, dtype="bf16")
M70B = ModelShape("70B-scale", Hq=64, Hkv=8, D=128, layers=80, dtype="bf16")
# multi-head attention, no K/V sharing: the head shape of the third model of the paper's evaluation (Section 4.1)
M30B_MHA = ModelShape("30B-scale-MHA", Hq=52, Hkv=52, D=128, layers=60, dtype="bf16")


def config_seed(config_id: int) -> int:
    return 1234 + int(config_id)


def rng_for(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(int(seed)))


def lengths_uniform(rng, n: int, lo: int, hi: int) -> np.ndarray:
    """n integers uniform in [lo, hi] inclusive."""
    return rng.integers(lo, hi + 1, size=n, dtype=np.int64).astype(np.int32)


def lengths_lognormal(rng, n: int, mean: float, sigma: float, lo: int, hi: int) -> np.ndarray:
    """Round(exp(N(mu, sigma^2))) clipped to [lo, hi], with mu chosen so that the
    unclipped distribution mean is `mean` (right-skewed like Table 4's avg/median pairs)."""
    mu = math.log(mean) - 0.5 * sigma * sigma
    x = np.exp(rng.normal(mu, sigma, size=n))
    return np.clip(np.rint(x), lo, hi).astype(np.int32)


# Table 4 of the paper: (input average, input median, output average, output median) of the three datasets.
TABLE4 = {"alpaca": (20.63, 17.0, 163.80, 119.0), "sharegpt": (343.76, 148.0, 237.20, 152.0),
          "longbench": (2686.89, 2736.5, 101.78, 19.0)}


def table4_lengths(name: str, rng, n: int, max_len: int = 4096):
    """(input, output) token counts shaped like one dataset of Table 4: lognormal with the table's average
    and median where the average exceeds the median (sigma^2 = 2 ln(avg / median)), else (LongBench inputs)
    normal around the average with a third of it as deviation; inputs are cut at `max_len` as in Section 4.1."""
    in_avg, in_med, out_avg, out_med = TABLE4[name]

    def draw(avg, med, lo, hi):
        if avg > med:
            sigma = math.sqrt(2.0 * math.log(avg / med))
            return lengths_lognormal(rng, n, avg, sigma, lo, hi)
        return np.clip(np.rint(rng.normal(avg, avg / 3.0, size=n)), lo, hi).astype(np.int32)

    return draw(in_avg, in_med, 1, max_len), draw(out_avg, out_med, 1, max_len)


def table4_decode_batch(model: ModelShape, name: str, B: int, seed: int) -> "DecodeBatch":
    """A decode-only batch in steady state on one dataset's shape: every sequence holds its prompt and a
    uniformly drawn part of its output."""
    rng = rng_for(seed)
    n_in, n_out = table4_lengths(name, rng, B)
    ctx = (n_in + np.floor(rng.random(B) * n_out).astype(np.int32) + 1).astype(np.int32)
    table, nb = make_block_table(rng, ctx.astype(np.int64), model.bs)
    return DecodeBatch(model, ctx, table, nb, seed)


def make_block_table(rng, capacity_tokens, bs: int = BLOCK_SIZE, pool_factor: float = 1.1,
                     min_spare: int = 2, stride: int | None = None):
    """Block table for sequences that may grow to capacity_tokens[b] tokens.

    Physical blocks are a random sample (without replacement) of a pool that is
    pool_factor times larger than needed, so the pool has holes and consecutive
    logical blocks are scattered.  Unused entries are -1.
    Returns (table int32 [B, stride], num_blocks)."""
    cap = np.asarray(capacity_tokens, dtype=np.int64)
    nblk = (cap + bs - 1) // bs
    need = int(nblk.sum())
    num_blocks = max(int(math.ceil(need * pool_factor)), need + min_spare)
    phys = rng.permutation(num_blocks)[:need].astype(np.int32)
    width = int(nblk.max()) if len(nblk) else 0
    stride = max(width, 1) if stride is None else int(stride)
    assert stride >= width
    table = np.full((len(cap), stride), -1, dtype=np.int32)
    o = 0
    for b, n in enumerate(nblk):
        table[b, : int(n)] = phys[o : o + int(n)]
        o += int(n)
    return table, num_blocks


def cu_from_lengths(lengths) -> np.ndarray:
    cu = np.zeros(len(lengths) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(np.asarray(lengths, dtype=np.int64))
    return cu


def randn(shape, dtype: str, seed: int, device="cpu", scale: float = 1.0) -> torch.Tensor:
    """N(0,1)*scale drawn in fp32 from a seeded generator on `device`, rounded
    (nearest-even) to the storage type.  The stream depends on the device kind, so
    a tensor is drawn once and the same bits are handed to both sides."""
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    t = torch.randn(tuple(shape), generator=g, device=device, dtype=torch.float32)
    if scale != 1.0:
        t = t * scale
    return t.to(torch.bfloat16 if dtype == "bf16" else torch.float32)


def to_bits(t: torch.Tensor) -> np.ndarray:
    """Host NumPy view of a tensor in the form the oracle takes: uint16 bit patterns
    for bf16, float32 otherwise."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


@dataclass
class DecodeBatch:
    model: ModelShape
    ctx_len: np.ndarray          # [B] tokens in cache INCLUDING the new token
    block_table: np.ndarray      # [B, stride]
    num_blocks: int
    seed: int

    @property
    def B(self) -> int:
        return len(self.ctx_len)

    @property
    def max_ctx_len(self) -> int:
        return int(self.ctx_len.max())


@dataclass
class PrefillBatch:
    model: ModelShape
    q_len: np.ndarray            # [B] new tokens per sequence
    ctx_before: np.ndarray       # [B]
    block_table: np.ndarray
    num_blocks: int
    seed: int
    cu_q: np.ndarray = field(init=False)

    def __post_init__(self):
        self.cu_q = cu_from_lengths(self.q_len)

    @property
    def B(self) -> int:
        return len(self.q_len)

    @property
    def T(self) -> int:
        return int(self.cu_q[-1])

    @property
    def max_q_len(self) -> int:
        return int(self.q_len.max()) if len(self.q_len) else 0


def decode_batch(model: ModelShape, B: int, lo: int, hi: int, seed: int, grow: int = 0) -> DecodeBatch:
    """B resident sequences with context lengths uniform in [lo, hi]; tables have room
    for `grow` more tokens per sequence."""
    rng = rng_for(seed)
    ctx = lengths_uniform(rng, B, lo, hi)
    table, nb = make_block_table(rng, ctx.astype(np.int64) + grow, model.bs)
    return DecodeBatch(model, ctx, table, nb, seed)


def prefill_batch(model: ModelShape, q_len, seed: int, ctx_before=None, grow: int = 0) -> PrefillBatch:
    rng = rng_for(seed)
    q_len = np.asarray(q_len, dtype=np.int32)
    cb = np.zeros_like(q_len) if ctx_before is None else np.asarray(ctx_before, dtype=np.int32)
    table, nb = make_block_table(rng, q_len.astype(np.int64) + cb + grow, model.bs)
    return PrefillBatch(model, q_len, cb, table, nb, seed)


# ---- the five workloads (sizes per the benchmark spec `configs`) ----------------------------

def config1_tiny():
    """Tiny PaDG cycle, fp32: prompts of 37 and 100 tokens, then 8 decode steps."""
    return prefill_batch(TINY, [37, 100], config_seed(1), grow=8)


def config2_decode_30b() -> DecodeBatch:
    return decode_batch(M30B, 128, 512, 4096, config_seed(2))


def config3_prefill_30b() -> PrefillBatch:
    rng = rng_for(config_seed(3))
    q_len = lengths_lognormal(rng, 16, mean=1024.0, sigma=1.0, lo=128, hi=4096)
    return prefill_batch(M30B, q_len, config_seed(3) + 1000)


def config4_decode_70b() -> DecodeBatch:
    return decode_batch(M70B, 256, 1024, 4096, config_seed(4))


def config5_switch_70b(n_resident: int = 192, n_new: int = 8, prompt: int = 8192, steps: int = 64):
    """Temporal-disaggregation switch: resident decode sequences, a prefill burst into the
    same pool, then decode steps with the union.  Returns (resident_ctx [n_resident],
    q_len [n_new], block_table [n_resident+n_new, stride], num_blocks).  Rows
    0..n_resident-1 are the resident sequences, the rest the new prompts."""
    rng = rng_for(config_seed(5))
    resident = lengths_uniform(rng, n_resident, 1024, 4096)
    q_len = np.full(n_new, prompt, dtype=np.int32)
    cap = np.concatenate([resident.astype(np.int64) + steps, q_len.astype(np.int64) + steps])
    table, nb = make_block_table(rng, cap, M70B.bs)
    return resident, q_len, table, nb
