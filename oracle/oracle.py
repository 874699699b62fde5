"""ctypes front end of the fp64 CPU oracle (oracle/ecoserve_oracle.c).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only tests/, the smoke check and the
benchmark's cpu_baseline leg may import this module.  It never imports the
GPU package and the GPU package never imports it.

Arrays are NumPy.  bf16 data travels as uint16 bit patterns, fp32 as float32;
the C side widens exactly to double.  Outputs are float64.

The logical cache view is [num_blocks, Hkv, bs, D] (one array for K, one for V).
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ecoserve_oracle.c")
_LIB = os.path.join(_HERE, "libecoserve_oracle.so")

BF16, F32 = 0, 1
_ERR = {1: "invalid argument", 2: "block table entry or position out of range", 3: "out of memory"}


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, OpenMP, no fast-math)."""
    if force or (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


@dataclass(frozen=True)
class Shape:
    """Head layout and paging of one layer's cache (Table 1 notation: M heads, D per head)."""
    Hq: int
    Hkv: int
    D: int
    bs: int
    num_blocks: int
    dtype: int  # BF16 | F32

    @property
    def np_dtype(self):
        return np.uint16 if self.dtype == BF16 else np.float32

    @property
    def scale(self) -> float:
        # Eq. 2: 1 / sqrt(d_k), d_k = D
        return 1.0 / math.sqrt(self.D)


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a


def _check(rc: int):
    if rc != 0:
        raise ValueError(f"oracle: {_ERR.get(rc, rc)}")


def new_cache(shape: Shape, fill_bits=None):
    """Oracle-owned K and V pools; every slot pre-filled with a sentinel bit pattern
    (default: a NaN) so that a read of an unwritten slot poisons the result."""
    if fill_bits is None:
        fill_bits = 0x7FC1 if shape.dtype == BF16 else 0x7FC00001
    dims = (shape.num_blocks, shape.Hkv, shape.bs, shape.D)
    if shape.dtype == BF16:
        k = np.full(dims, fill_bits, dtype=np.uint16)
    else:
        k = np.full(dims, fill_bits, dtype=np.uint32).view(np.float32)
    return k, k.copy()


def kv_append(shape: Shape, k_cache, v_cache, k_new, v_new, cu_q, ctx_before, block_table):
    """In-place append of k_new/v_new [T,Hkv,D] into the logical caches."""
    lib = _load()
    cu_q, ctx_before, block_table = _i32(cu_q), _i32(ctx_before), _i32(block_table)
    B = len(ctx_before)
    assert k_cache.flags.c_contiguous and v_cache.flags.c_contiguous
    k_new = np.ascontiguousarray(k_new)
    v_new = np.ascontiguousarray(v_new)
    assert k_new.dtype == shape.np_dtype and k_cache.dtype == shape.np_dtype
    assert k_new.shape == (int(cu_q[B]), shape.Hkv, shape.D) if B > 0 else True
    rc = lib.oracle_kv_append(_p(k_cache), _p(v_cache), _p(k_new), _p(v_new), _p(cu_q), _p(ctx_before),
                              _p(block_table), ctypes.c_int32(block_table.shape[1]), ctypes.c_int32(B),
                              ctypes.c_int32(shape.Hkv), ctypes.c_int32(shape.D), ctypes.c_int32(shape.bs),
                              ctypes.c_int32(shape.num_blocks), ctypes.c_int32(shape.dtype))
    _check(rc)


def attn_rows(shape: Shape, q, k_cache, v_cache, block_table, seq_row_start, row_tok, row_pos,
              scale=None, want_probs=False):
    """Attention for selected query rows (grouped by sequence).  Returns (out, lse[, probs])."""
    lib = _load()
    block_table = _i32(block_table)
    seq_row_start, row_tok, row_pos = _i32(seq_row_start), _i32(row_tok), _i32(row_pos)
    B = len(seq_row_start) - 1
    R = len(row_tok)
    q = np.ascontiguousarray(q)
    assert q.dtype == shape.np_dtype and k_cache.dtype == shape.np_dtype
    assert k_cache.flags.c_contiguous and v_cache.flags.c_contiguous
    out = np.empty((R, shape.Hq, shape.D), dtype=np.float64)
    lse = np.empty((R, shape.Hq), dtype=np.float64)
    probs = None
    stride = 0
    if want_probs:
        stride = int(row_pos.max()) + 1 if R else 1
        probs = np.zeros((R, shape.Hq, stride), dtype=np.float64)
    sc = shape.scale if scale is None else float(scale)
    rc = lib.oracle_attn_rows(_p(q), _p(k_cache), _p(v_cache), _p(block_table),
                              ctypes.c_int32(block_table.shape[1]), _p(seq_row_start), _p(row_tok), _p(row_pos),
                              ctypes.c_int32(B), ctypes.c_int32(shape.Hq), ctypes.c_int32(shape.Hkv),
                              ctypes.c_int32(shape.D), ctypes.c_int32(shape.bs), ctypes.c_int32(shape.num_blocks),
                              ctypes.c_int32(shape.dtype), ctypes.c_double(sc), _p(out), _p(lse), _p(probs),
                              ctypes.c_int32(stride))
    _check(rc)
    return (out, lse, probs) if want_probs else (out, lse)


def attn_prefill(shape: Shape, q, k_cache, v_cache, cu_q, ctx_before, block_table, scale=None):
    """Causal prefill attention over the (already appended) cache.  Returns (out [T,Hq,D], lse [T,Hq])."""
    lib = _load()
    cu_q, ctx_before, block_table = _i32(cu_q), _i32(ctx_before), _i32(block_table)
    B = len(ctx_before)
    T = int(cu_q[B]) if B > 0 else 0
    q = np.ascontiguousarray(q)
    assert q.dtype == shape.np_dtype and q.shape == (T, shape.Hq, shape.D)
    out = np.empty((T, shape.Hq, shape.D), dtype=np.float64)
    lse = np.empty((T, shape.Hq), dtype=np.float64)
    sc = shape.scale if scale is None else float(scale)
    rc = lib.oracle_attn_prefill(_p(q), _p(k_cache), _p(v_cache), _p(cu_q), _p(ctx_before), _p(block_table),
                                 ctypes.c_int32(block_table.shape[1]), ctypes.c_int32(B),
                                 ctypes.c_int32(shape.Hq), ctypes.c_int32(shape.Hkv), ctypes.c_int32(shape.D),
                                 ctypes.c_int32(shape.bs), ctypes.c_int32(shape.num_blocks),
                                 ctypes.c_int32(shape.dtype), ctypes.c_double(sc), _p(out), _p(lse))
    _check(rc)
    return out, lse


def attn_decode(shape: Shape, q, k_cache, v_cache, block_table, ctx_len, scale=None):
    """Decode attention: one query per sequence at position ctx_len-1.  Returns (out [B,Hq,D], lse [B,Hq])."""
    lib = _load()
    ctx_len, block_table = _i32(ctx_len), _i32(block_table)
    B = len(ctx_len)
    q = np.ascontiguousarray(q)
    assert q.dtype == shape.np_dtype and q.shape == (B, shape.Hq, shape.D)
    out = np.empty((B, shape.Hq, shape.D), dtype=np.float64)
    lse = np.empty((B, shape.Hq), dtype=np.float64)
    sc = shape.scale if scale is None else float(scale)
    rc = lib.oracle_attn_decode(_p(q), _p(k_cache), _p(v_cache), _p(block_table),
                                ctypes.c_int32(block_table.shape[1]), _p(ctx_len), ctypes.c_int32(B),
                                ctypes.c_int32(shape.Hq), ctypes.c_int32(shape.Hkv), ctypes.c_int32(shape.D),
                                ctypes.c_int32(shape.bs), ctypes.c_int32(shape.num_blocks),
                                ctypes.c_int32(shape.dtype), ctypes.c_double(sc), _p(out), _p(lse))
    _check(rc)
    return out, lse
