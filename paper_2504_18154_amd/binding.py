"""Thin ctypes binding of the C ABI in include/ecoserve.h.

Argument marshalling only: every step of the hot path runs in the HIP kernels of
libecoserve.so.  PyTorch tensors provide device memory and the current HIP stream.
Importing this module without a built library raises: there is no fallback.
"""
from __future__ import annotations

import ctypes
import math
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# ECOSERVE_LIB overrides the library to load (to compare builds); the default is the one built in-tree
LIB_PATH = os.environ.get("ECOSERVE_LIB") or os.path.join(_HERE, "libecoserve.so")

OK, EINVAL, EUNSUPPORTED, ENOMEM, EHIP, ECONTENT = range(6)
BF16, F32 = 0, 1
OPT_DECODE_SPLIT_TOKENS, OPT_FORCE_PLAIN, OPT_PROFILE, OPT_DECODE_ADAPTIVE, OPT_PREFILL_REUSE_PLAN = 1, 2, 3, 4, 5
KERNEL_APPEND, KERNEL_PREFILL, KERNEL_DECODE = 0, 1, 2

EXPORTS = [
    "ecoserve_create", "ecoserve_destroy", "ecoserve_set_option", "ecoserve_strerror", "ecoserve_cache_bytes",
    "ecoserve_k_cache_index", "ecoserve_v_cache_index", "ecoserve_workspace_bytes", "ecoserve_kv_append",
    "ecoserve_attn_prefill", "ecoserve_attn_decode", "ecoserve_debug_validate", "ecoserve_profile_read",
    "ecoserve_profile_reset", "ecoserve_probe_hbm_read", "ecoserve_probe_mfma_bf16",
    "ecoserve_kv_append_strided", "ecoserve_attn_prefill_strided", "ecoserve_attn_decode_strided",
    "ecoserve_attn_decode_append", "ecoserve_attn_decode_noalloc", "ecoserve_probe_mfma_valu",
    "ecoserve_debug_prefill_queue_shares",
]


class Layout(ctypes.Structure):
    _fields_ = [("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("block_size", ctypes.c_int32), ("num_blocks", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("softmax_scale", ctypes.c_float)]


class EcoserveError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: {strerror(status)} (status {status})")
        self.status = status


def _load(path: str = LIB_PATH) -> ctypes.CDLL:
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2504_18154_amd.build` "
                          "(there is no fallback path)")
    lib = ctypes.CDLL(path)
    vp, i32, i32p = ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p
    lib.ecoserve_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int, ctypes.POINTER(Layout), i32, i32]
    lib.ecoserve_destroy.argtypes = [vp]
    lib.ecoserve_set_option.argtypes = [vp, i32, i32]
    lib.ecoserve_strerror.argtypes = [ctypes.c_int]
    lib.ecoserve_strerror.restype = ctypes.c_char_p
    lib.ecoserve_cache_bytes.argtypes = [ctypes.POINTER(Layout)]
    lib.ecoserve_cache_bytes.restype = ctypes.c_size_t
    for f in (lib.ecoserve_k_cache_index, lib.ecoserve_v_cache_index):
        f.argtypes = [ctypes.POINTER(Layout), i32, i32, i32, i32]
        f.restype = ctypes.c_size_t
    lib.ecoserve_workspace_bytes.argtypes = [vp]
    lib.ecoserve_workspace_bytes.restype = ctypes.c_size_t
    lib.ecoserve_kv_append.argtypes = [vp, vp, vp, vp, vp, i32p, i32p, i32p, i32, i32, i32, i32, vp]
    lib.ecoserve_attn_prefill.argtypes = [vp, vp, vp, vp, i32p, i32p, i32p, i32, vp, vp, i32, i32, i32, vp]
    lib.ecoserve_attn_decode.argtypes = [vp, vp, vp, vp, i32p, i32, i32p, vp, vp, i32, i32, vp]
    i64 = ctypes.c_int64
    lib.ecoserve_kv_append_strided.argtypes = [vp, vp, vp, vp, vp, i64, i32p, i32p, i32p, i32, i32, i32, i32, vp]
    lib.ecoserve_attn_prefill_strided.argtypes = [vp, vp, i64, vp, vp, i32p, i32p, i32p, i32, vp, vp, i32, i32, i32, vp]
    lib.ecoserve_attn_decode_strided.argtypes = [vp, vp, i64, vp, vp, i32p, i32, i32p, vp, vp, i32, i32, vp]
    lib.ecoserve_attn_decode_append.argtypes = [vp, vp, i64, vp, vp, i64, vp, vp, i32p, i32, i32p, vp, vp, i32, i32, vp]
    lib.ecoserve_attn_decode_noalloc.argtypes = [ctypes.c_int, ctypes.POINTER(Layout), vp, vp, vp, i32p, i32, i32p, vp, vp,
                                                 i32, i32, vp]
    lib.ecoserve_debug_validate.argtypes = [vp, i32p, i32p, i32p, i32, i32]
    lib.ecoserve_debug_prefill_queue_shares.argtypes = [vp, ctypes.POINTER(ctypes.c_float)]
    lib.ecoserve_profile_read.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    lib.ecoserve_profile_reset.argtypes = [vp]
    lib.ecoserve_probe_hbm_read.argtypes = [ctypes.c_int, ctypes.c_size_t, i32, ctypes.POINTER(ctypes.c_double)]
    lib.ecoserve_probe_mfma_bf16.argtypes = [ctypes.c_int, i32, i32, ctypes.POINTER(ctypes.c_double)]
    lib.ecoserve_probe_mfma_valu.argtypes = [ctypes.c_int, i32, i32, i32, i32, ctypes.POINTER(ctypes.c_double),
                                             ctypes.POINTER(ctypes.c_double)]
    return lib


_lib = _load()


def strerror(status: int) -> str:
    return _lib.ecoserve_strerror(int(status)).decode()


def _check(status: int, what: str):
    if status != OK:
        raise EcoserveError(status, what)


def make_layout(Hq, Hkv, D, num_blocks, dtype, bs=16, softmax_scale=0.0) -> Layout:
    code = {"bf16": BF16, "f32": F32, torch.bfloat16: BF16, torch.float32: F32, BF16: BF16, F32: F32}[dtype]
    return Layout(int(Hq), int(Hkv), int(D), int(bs), int(num_blocks), code, float(softmax_scale))


def cache_bytes(layout: Layout) -> int:
    return int(_lib.ecoserve_cache_bytes(ctypes.byref(layout)))


def k_cache_index(layout: Layout, blk, g, slot, d) -> int:
    return int(_lib.ecoserve_k_cache_index(ctypes.byref(layout), blk, g, slot, d))


def v_cache_index(layout: Layout, blk, g, slot, d) -> int:
    return int(_lib.ecoserve_v_cache_index(ctypes.byref(layout), blk, g, slot, d))


def probe_hbm_read(nbytes: int = 4 << 30, reps: int = 5, device: int = 0) -> float:
    """Sustained device-memory read rate of `device` in GB/s (1e9 bytes per second)."""
    rate = ctypes.c_double()
    _check(_lib.ecoserve_probe_hbm_read(int(device), int(nbytes), int(reps), ctypes.byref(rate)),
           "ecoserve_probe_hbm_read")
    return rate.value


def probe_mfma_bf16(random_operands: bool, reps: int = 5, device: int = 0) -> float:
    """Sustained bf16 matrix-core rate of `device` in TFLOP/s."""
    rate = ctypes.c_double()
    _check(_lib.ecoserve_probe_mfma_bf16(int(device), int(bool(random_operands)), int(reps), ctypes.byref(rate)),
           "ecoserve_probe_mfma_bf16")
    return rate.value


def probe_mfma_valu(with_mfma: bool, fma_per_slot: int, exp_per_slot: int, waves_per_simd: int = 2, device: int = 0):
    """(shader clocks a SIMD spends per slot of one matrix instruction + the given vector work, shader clock in GHz)."""
    clocks, ghz = ctypes.c_double(), ctypes.c_double()
    _check(_lib.ecoserve_probe_mfma_valu(int(device), int(bool(with_mfma)), int(fma_per_slot), int(exp_per_slot),
                                         int(waves_per_simd), ctypes.byref(clocks), ctypes.byref(ghz)),
           "ecoserve_probe_mfma_valu")
    return clocks.value, ghz.value


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def attn_decode_noalloc(layout: Layout, q, k_cache, v_cache, block_table, ctx_len, out, max_ctx_len, lse=None,
                        device: int = 0) -> int:
    """ecoserve_attn_decode without a context and without any allocation; returns the status code."""
    return int(_lib.ecoserve_attn_decode_noalloc(int(device), ctypes.byref(layout), _ptr(q), _ptr(k_cache),
                                                 _ptr(v_cache), _ptr(block_table), int(block_table.shape[1]),
                                                 _ptr(ctx_len), _ptr(out), _ptr(lse), int(ctx_len.numel()),
                                                 int(max_ctx_len), _stream()))


def _row_stride(t) -> int:
    """Elements between consecutive tokens of a [tokens, heads, D] tensor or view whose heads are contiguous."""
    if t.dim() != 3 or t.stride(2) != 1 or t.stride(1) != t.shape[2]:
        raise ValueError("expected a [tokens, heads, D] tensor with contiguous heads")
    return int(t.stride(0)) if t.shape[0] > 1 else int(t.shape[1] * t.shape[2])


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


class Context:
    """Owns an ecoserve_ctx.  Tensors handed to the hot calls must live on the context's GPU."""

    def __init__(self, Hq, Hkv, D, num_blocks, dtype, max_batch, max_blocks_per_seq, device=0, bs=16,
                 softmax_scale=0.0):
        self.layout = make_layout(Hq, Hkv, D, num_blocks, dtype, bs, softmax_scale)
        self.torch_dtype = torch.bfloat16 if self.layout.dtype == BF16 else torch.float32
        self.device = torch.device("cuda", device)
        self._h = ctypes.c_void_p()
        _check(_lib.ecoserve_create(ctypes.byref(self._h), int(device), ctypes.byref(self.layout), int(max_batch),
                                    int(max_blocks_per_seq)), "ecoserve_create")

    def close(self):
        if getattr(self, "_h", None):
            _lib.ecoserve_destroy(self._h)
            self._h = None

    __del__ = close

    def set_option(self, option: int, value: int):
        _check(_lib.ecoserve_set_option(self._h, int(option), int(value)), "ecoserve_set_option")

    def workspace_bytes(self) -> int:
        return int(_lib.ecoserve_workspace_bytes(self._h))

    # ---- cache helpers (layout plumbing only) ------------------------------------------
    def new_cache(self, fill_bits=None):
        """One layer's K and V pools as flat tensors, every element set to a sentinel bit
        pattern (default a NaN)."""
        L = self.layout
        n = L.num_blocks * L.num_kv_heads * L.block_size * L.head_dim
        if L.dtype == BF16:
            bits = 0x7FC1 if fill_bits is None else fill_bits
            k = torch.full((n,), bits - 65536 if bits >= 32768 else bits, dtype=torch.int16,
                           device=self.device).view(torch.bfloat16)
        else:
            bits = 0x7FC00001 if fill_bits is None else fill_bits
            k = torch.full((n,), bits, dtype=torch.int32, device=self.device).view(torch.float32)
        return k, k.clone()

    def k_logical(self, k_cache: torch.Tensor) -> torch.Tensor:
        """View of a K pool as [num_blocks, Hkv, bs, D] (a permutation of the physical
        [num_blocks, Hkv, D/x, bs, x])."""
        L = self.layout
        x = 8 if L.dtype == BF16 else 4
        return k_cache.view(L.num_blocks, L.num_kv_heads, L.head_dim // x, L.block_size, x).permute(0, 1, 3, 2, 4) \
            .reshape(L.num_blocks, L.num_kv_heads, L.block_size, L.head_dim)

    def v_logical(self, v_cache: torch.Tensor) -> torch.Tensor:
        """View of a V pool as [num_blocks, Hkv, bs, D] (physical [num_blocks, Hkv, D, bs])."""
        L = self.layout
        return v_cache.view(L.num_blocks, L.num_kv_heads, L.head_dim, L.block_size).permute(0, 1, 3, 2)

    # ---- the three hot calls -------------------------------------------------------------
    def kv_append(self, k_cache, v_cache, k_new, v_new, cu_q, ctx_before, block_table, max_new_len=None):
        B = ctx_before.numel()
        T = k_new.shape[0]
        if max_new_len is None:
            max_new_len = T
        _check(_lib.ecoserve_kv_append(self._h, _ptr(k_cache), _ptr(v_cache), _ptr(k_new), _ptr(v_new), _ptr(cu_q),
                                       _ptr(ctx_before), _ptr(block_table), int(block_table.shape[1]), int(B),
                                       int(T), int(max_new_len), _stream()), "ecoserve_kv_append")

    def attn_prefill(self, q, k_cache, v_cache, cu_q, ctx_before, block_table, out, lse=None, max_q_len=None):
        B = ctx_before.numel()
        T = q.shape[0]
        if max_q_len is None:
            max_q_len = T
        _check(_lib.ecoserve_attn_prefill(self._h, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(cu_q),
                                          _ptr(ctx_before), _ptr(block_table), int(block_table.shape[1]), _ptr(out),
                                          _ptr(lse), int(B), int(T), int(max_q_len), _stream()),
               "ecoserve_attn_prefill")

    # the same on views into wider rows (e.g. slices of a fused projection output [T, Hq + 2 Hkv, D])
    def kv_append_strided(self, k_cache, v_cache, k_new, v_new, cu_q, ctx_before, block_table, max_new_len=None):
        B = ctx_before.numel()
        T = k_new.shape[0]
        if max_new_len is None:
            max_new_len = T
        if _row_stride(k_new) != _row_stride(v_new):
            raise ValueError("k_new and v_new must have the same row stride")
        _check(_lib.ecoserve_kv_append_strided(self._h, _ptr(k_cache), _ptr(v_cache), _ptr(k_new), _ptr(v_new),
                                               _row_stride(k_new), _ptr(cu_q), _ptr(ctx_before), _ptr(block_table),
                                               int(block_table.shape[1]), int(B), int(T), int(max_new_len),
                                               _stream()), "ecoserve_kv_append_strided")

    def attn_prefill_strided(self, q, k_cache, v_cache, cu_q, ctx_before, block_table, out, lse=None,
                             max_q_len=None):
        B = ctx_before.numel()
        T = q.shape[0]
        if max_q_len is None:
            max_q_len = T
        _check(_lib.ecoserve_attn_prefill_strided(self._h, _ptr(q), _row_stride(q), _ptr(k_cache), _ptr(v_cache),
                                                  _ptr(cu_q), _ptr(ctx_before), _ptr(block_table),
                                                  int(block_table.shape[1]), _ptr(out), _ptr(lse), int(B), int(T),
                                                  int(max_q_len), _stream()), "ecoserve_attn_prefill_strided")

    def attn_decode_strided(self, q, k_cache, v_cache, block_table, ctx_len, out, max_ctx_len, lse=None):
        B = ctx_len.numel()
        _check(_lib.ecoserve_attn_decode_strided(self._h, _ptr(q), _row_stride(q), _ptr(k_cache), _ptr(v_cache),
                                                 _ptr(block_table), int(block_table.shape[1]), _ptr(ctx_len),
                                                 _ptr(out), _ptr(lse), int(B), int(max_ctx_len), _stream()),
               "ecoserve_attn_decode_strided")

    def attn_decode_append(self, q, k_new, v_new, k_cache, v_cache, block_table, ctx_len, out, max_ctx_len, lse=None):
        """Decode with the append of the step's one new token per sequence fused in (ctx_len counts it)."""
        B = ctx_len.numel()
        if _row_stride(k_new) != _row_stride(v_new):
            raise ValueError("k_new and v_new must have the same row stride")
        _check(_lib.ecoserve_attn_decode_append(self._h, _ptr(q), _row_stride(q), _ptr(k_new), _ptr(v_new),
                                                _row_stride(k_new), _ptr(k_cache), _ptr(v_cache), _ptr(block_table),
                                                int(block_table.shape[1]), _ptr(ctx_len), _ptr(out), _ptr(lse), int(B),
                                                int(max_ctx_len), _stream()), "ecoserve_attn_decode_append")

    def attn_decode(self, q, k_cache, v_cache, block_table, ctx_len, out, max_ctx_len, lse=None):
        B = ctx_len.numel()
        _check(_lib.ecoserve_attn_decode(self._h, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_table),
                                         int(block_table.shape[1]), _ptr(ctx_len), _ptr(out), _ptr(lse), int(B),
                                         int(max_ctx_len), _stream()), "ecoserve_attn_decode")

    # ---- debugging / profiling -----------------------------------------------------------
    def debug_validate(self, cu_q, ctx_total, block_table):
        return int(_lib.ecoserve_debug_validate(self._h, _ptr(cu_q), _ptr(ctx_total), _ptr(block_table),
                                                int(block_table.shape[1]), int(ctx_total.numel())))

    def debug_prefill_queue_shares(self):
        shares = (ctypes.c_float * 8)()
        _check(_lib.ecoserve_debug_prefill_queue_shares(self._h, shares), "ecoserve_debug_prefill_queue_shares")
        return [float(x) for x in shares]

    def profile_reset(self):
        _check(_lib.ecoserve_profile_reset(self._h), "ecoserve_profile_reset")

    def profile_read(self, kernel: int):
        ms, n = ctypes.c_double(), ctypes.c_int64()
        _check(_lib.ecoserve_profile_read(self._h, int(kernel), ctypes.byref(ms), ctypes.byref(n)),
               "ecoserve_profile_read")
        return ms.value, n.value


def default_scale(D: int) -> float:
    return 1.0 / math.sqrt(D)
