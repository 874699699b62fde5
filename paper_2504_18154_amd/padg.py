"""ctypes marshalling for include/ecoserve_padg.h (the host-side macro-instance model): same names,
plain Python containers in, plain Python containers out.  All of the model runs in the library."""
from __future__ import annotations

import ctypes
from typing import List, NamedTuple, Sequence, Tuple

from . import binding

i32, i64 = ctypes.c_int32, ctypes.c_int64


class _Request(ctypes.Structure):
    _fields_ = [("arrival_us", i64), ("input_len", i32), ("output_len", i32)]


class _Config(ctypes.Structure):
    _fields_ = [("n_instances", i32), ("search_all", i32), ("slo_ttft_us", i64), ("slo_tpot_us", i64),
                ("kv_capacity_tokens", i64), ("n_prefill_points", i32), ("prefill_len", ctypes.POINTER(i32)),
                ("prefill_us", ctypes.POINTER(i64)), ("decode_base_us", i64), ("decode_per_seq_ns", i64),
                ("decode_per_token_ns", i64)]


class _Result(ctypes.Structure):
    _fields_ = [("instance", i32), ("check", i32), ("first_token_us", i64), ("finish_us", i64)]


class Result(NamedTuple):
    instance: int
    check: int
    first_token_us: int
    finish_us: int


_lib = binding._lib
_lib.ecoserve_padg_prefill_us.argtypes = [ctypes.POINTER(_Config), i32]
_lib.ecoserve_padg_prefill_us.restype = i64
_lib.ecoserve_padg_check_constraints.argtypes = [ctypes.POINTER(_Config), i64, ctypes.POINTER(i32), i32,
                                                 ctypes.POINTER(i32), ctypes.POINTER(i64), i32, i64, i32]
_lib.ecoserve_padg_simulate.argtypes = [ctypes.POINTER(_Config), ctypes.POINTER(_Request), i64,
                                        ctypes.POINTER(_Result)]


class Config:
    """Owns the C config and the arrays it points to."""

    def __init__(self, n_instances: int, slo_ttft_us: int, slo_tpot_us: int, kv_capacity_tokens: int,
                 prefill_len: Sequence[int], prefill_us: Sequence[int], decode_base_us: int, decode_per_seq_ns: int,
                 decode_per_token_ns: int, search_all: bool = False):
        assert len(prefill_len) == len(prefill_us)
        self._len = (i32 * len(prefill_len))(*[int(x) for x in prefill_len])
        self._us = (i64 * len(prefill_us))(*[int(x) for x in prefill_us])
        self.c = _Config(int(n_instances), int(bool(search_all)), int(slo_ttft_us), int(slo_tpot_us),
                         int(kv_capacity_tokens), len(prefill_len), self._len, self._us, int(decode_base_us),
                         int(decode_per_seq_ns), int(decode_per_token_ns))


def prefill_us(cfg: Config, input_len: int) -> int:
    t = int(_lib.ecoserve_padg_prefill_us(ctypes.byref(cfg.c), int(input_len)))
    if t < 0:
        raise binding.EcoserveError(binding.EINVAL, "ecoserve_padg_prefill_us")
    return t


def check_constraints(cfg: Config, now_us: int, phase_input_len: Sequence[int], decode_generated: Sequence[int],
                      decode_first_token_us: Sequence[int], kv_used_tokens: int, req_input_len: int) -> int:
    ph = (i32 * max(len(phase_input_len), 1))(*[int(x) for x in phase_input_len])
    gen = (i32 * max(len(decode_generated), 1))(*[int(x) for x in decode_generated])
    first = (i64 * max(len(decode_first_token_us), 1))(*[int(x) for x in decode_first_token_us])
    st = int(_lib.ecoserve_padg_check_constraints(ctypes.byref(cfg.c), int(now_us), ph, len(phase_input_len), gen,
                                                  first, len(decode_generated), int(kv_used_tokens),
                                                  int(req_input_len)))
    if st < 0:
        raise binding.EcoserveError(-st, "ecoserve_padg_check_constraints")
    return st


def simulate(cfg: Config, requests: Sequence[Tuple[int, int, int]]) -> List[Result]:
    """requests: (arrival_us, input_len, output_len), sorted by arrival."""
    n = len(requests)
    reqs = (_Request * max(n, 1))(*[_Request(int(a), int(i), int(o)) for a, i, o in requests])
    out = (_Result * max(n, 1))()
    binding._check(int(_lib.ecoserve_padg_simulate(ctypes.byref(cfg.c), reqs, n, out)), "ecoserve_padg_simulate")
    return [Result(out[k].instance, out[k].check, out[k].first_token_us, out[k].finish_us) for k in range(n)]
