"""Algorithmic work of the hot path: the bytes and FLOPs the method must move or
compute, used as the numerator of every roofline figure the benchmark prints.

Conventions
  * KV bytes per token (Section 2.1, "memory-compute trade-off" paragraph; Table 3):
    2 (K and V) x layers x Hkv x D x sizeof(element).
  * Table 2 counts only the two attention matmuls (softmax is left out, Section 2.1
    "distinct arithmetic intensity"): decode QK^T and PV are 2*B*S*H FLOPs each with
    H = Hq*D; prefill 2*B*S^2*H each over the full square.  Causal prefill touches
    S(S+1)/2 of the S^2 score entries, and only those are credited here.
"""
from __future__ import annotations

import numpy as np


def kv_bytes_per_token(layers: int, Hkv: int, D: int, elem_bytes: int = 2) -> int:
    return 2 * layers * Hkv * D * elem_bytes


def table2_attention_flops(phase: str, B: int, S: int, Hq: int, D: int) -> int:
    """FLOPs of ONE of the two attention matmuls of Table 2 (QK^T or PV), uniform length S."""
    H = Hq * D
    if phase == "prefill":
        return 2 * B * S * S * H
    if phase == "decode":
        return 2 * B * S * H
    raise ValueError(phase)


def decode_flops(ctx_len, Hq: int, D: int) -> int:
    """Both matmuls, one layer: 4 * Hq * D * sum(L_b)."""
    return int(4 * Hq * D * np.asarray(ctx_len, dtype=np.int64).sum())


def decode_bytes(ctx_len, Hq: int, Hkv: int, D: int, bs: int, elem_bytes: int = 2) -> int:
    """One layer: K and V of every cached token read once, Q read, O written, block table read."""
    L = np.asarray(ctx_len, dtype=np.int64)
    kv = int(L.sum()) * 2 * Hkv * D * elem_bytes
    qo = len(L) * 2 * Hq * D * elem_bytes
    table = int(((L + bs - 1) // bs).sum()) * 4
    return kv + qo + table


def prefill_flops_causal(q_len, Hq: int, D: int, ctx_before=None) -> int:
    """Both matmuls, one layer, causal: query i of a sequence with c cached tokens sees c+i+1 keys."""
    S = np.asarray(q_len, dtype=np.int64)
    c = np.zeros_like(S) if ctx_before is None else np.asarray(ctx_before, dtype=np.int64)
    pairs = S * c + S * (S + 1) // 2
    return int(4 * Hq * D * pairs.sum())


def append_bytes(T: int, Hkv: int, D: int, elem_bytes: int = 2) -> int:
    """One layer: new K and V rows read once and written once."""
    return 2 * (T * 2 * Hkv * D * elem_bytes)


# Published MI355X peaks used as roofline denominators.
PEAK_HBM_GBPS = 8000.0
PEAK_BF16_TFLOPS = 2500.0
