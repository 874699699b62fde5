"""Plain Python model of one EcoServe macro instance (test infrastructure only).

Written from the paper, step by step and in its notation, with no attempt at speed:
Section 3.2.1 (temporal disaggregation: an instance runs one phase at a time and puts
prefills first), Section 3.4 (Algorithm 1, InterSchedule; Algorithm 2, CheckConstraints;
the prefill-duration predictor profiled over sequence lengths) and the metrics of Sections
3.3 / 4.1 (TTFT including the phase-switching wait, TPOT measured from the first token,
SLO attainment).  Integer microseconds and token counts throughout, so results are exact.

Only tests/ may import this module; the product is the C++ implementation behind
include/ecoserve_padg.h, with which it shares no code.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

SATISFIED, TTFT, TPOT, MEMORY = 0, 1, 2, 3


@dataclass
class Config:
    n_instances: int
    slo_ttft_us: int
    slo_tpot_us: int
    kv_capacity_tokens: int
    prefill_len: Sequence[int]      # profile points: input lengths, increasing
    prefill_us: Sequence[int]       # and the prefill duration measured at each
    decode_base_us: int
    decode_per_seq_ns: int
    decode_per_token_ns: int
    search_all: bool = False        # Algorithm 1 as printed (False) or as the text reads (True)


@dataclass
class Request:
    arrival_us: int
    input_len: int
    output_len: int
    # filled in by the run
    instance: int = -1
    check: int = -1
    generated: int = 0
    first_token_us: int = -1
    finish_us: int = -1


def prefill_us(cfg: Config, n: int) -> int:
    """Section 3.4: the prefill duration of a request is predicted from a profile over sequence lengths.
    Linear interpolation between neighbouring profile points, the outer segments extended outwards."""
    L, U = cfg.prefill_len, cfg.prefill_us
    k = 0
    while k + 2 < len(L) and n >= L[k + 1]:
        k += 1
    t = U[k] + ((U[k + 1] - U[k]) * (n - L[k])) // (L[k + 1] - L[k])   # Python's // rounds towards -infinity
    return max(t, 1)


def decode_step_us(cfg: Config, batch: int, tokens: int) -> int:
    return cfg.decode_base_us + (cfg.decode_per_seq_ns * batch + cfg.decode_per_token_ns * tokens) // 1000


def check_constraints(cfg: Config, now_us: int, phase_input_len: Sequence[int], decode_generated: Sequence[int],
                      decode_first_token_us: Sequence[int], kv_used_tokens: int, req_input_len: int) -> int:
    """Algorithm 2 on a snapshot of an instance."""
    # Constraint 1: the prefill phase, with the new request added, must fit into the TTFT SLO
    t_total = sum(prefill_us(cfg, n) for n in phase_input_len) + prefill_us(cfg, req_input_len)
    if t_total > cfg.slo_ttft_us:
        return TTFT
    # Constraint 2: the decodes that the phase interrupts must have saved that much TPOT, on average
    saved = [L * cfg.slo_tpot_us - (now_us - first) for L, first in zip(decode_generated, decode_first_token_us)]
    if saved and sum(saved) < t_total * len(saved):      # mean(saved) < t_total, without a division
        return TPOT
    # Constraint 3: the request's KV cache must fit into what is left
    if req_input_len > cfg.kv_capacity_tokens - kv_used_tokens:
        return MEMORY
    return SATISFIED


@dataclass
class Instance:
    pending: List[Request] = field(default_factory=list)         # routed here, prefill not yet run
    decoding: List[Request] = field(default_factory=list)        # have their first token, not finished
    done_in_phase: List[Request] = field(default_factory=list)   # prefilled in the current prefill phase
    running: Optional[str] = None                                # "prefill" | "decode" | None (idle)
    running_end: int = 0
    running_req: Optional[Request] = None

    def kv_used(self) -> int:
        return sum(r.input_len + r.generated for r in self.pending + self.decoding)


class MacroInstance:
    def __init__(self, cfg: Config):
        self.cfg = cfg
        self.inst = [Instance() for _ in range(cfg.n_instances)]
        self.prev_idx = 0

    # ---- one instance: Section 3.2.1 -------------------------------------------------------------
    def _start_next(self, I: Instance, now: int):
        if I.pending:                       # prefills first
            r = I.pending.pop(0)
            I.running, I.running_req = "prefill", r
            I.running_end = now + prefill_us(self.cfg, r.input_len)
        elif I.decoding:
            I.done_in_phase = []            # a decode step starts: the prefill phase is over
            tokens = sum(r.input_len + r.generated for r in I.decoding)
            I.running, I.running_req = "decode", None
            I.running_end = now + decode_step_us(self.cfg, len(I.decoding), tokens)
        else:
            I.done_in_phase = []            # idle: no phase at all
            I.running, I.running_req = None, None

    def _complete(self, I: Instance):
        end = I.running_end
        if I.running == "prefill":
            r = I.running_req
            r.first_token_us, r.generated = end, 1
            I.done_in_phase.append(r)
            if r.output_len == 1:
                r.finish_us = end
            else:
                I.decoding.append(r)
        else:
            for r in I.decoding:
                r.generated += 1
                if r.generated == r.output_len:
                    r.finish_us = end
            I.decoding = [r for r in I.decoding if r.finish_us < 0]
        self._start_next(I, end)

    def _advance(self, I: Instance, now: Optional[int]):
        while I.running is not None and (now is None or I.running_end <= now):
            self._complete(I)

    # ---- Algorithm 2 on the live state ---------------------------------------------------------------
    def _check(self, I: Instance, req: Request, now: int) -> int:
        phase = [r.input_len for r in I.done_in_phase]
        if I.running == "prefill":
            phase.append(I.running_req.input_len)
        phase += [r.input_len for r in I.pending]
        existed = [r for r in I.decoding if not any(r is d for d in I.done_in_phase)]
        used = I.kv_used() + (I.running_req.input_len if I.running == "prefill" else 0)
        return check_constraints(self.cfg, now, phase, [r.generated for r in existed],
                                 [r.first_token_us for r in existed], used, req.input_len)

    # ---- Algorithm 1 -------------------------------------------------------------------------------------
    def _inter_schedule(self, req: Request, now: int) -> int:
        n = self.cfg.n_instances
        req.check = self._check(self.inst[self.prev_idx], req, now)
        if req.check == SATISFIED:
            return self.prev_idx
        if self.cfg.search_all:
            for k in range(1, n):
                idx = (self.prev_idx + k) % n
                if self._check(self.inst[idx], req, now) == SATISFIED:
                    return idx
        return (self.prev_idx + 1) % n

    def run(self, reqs: List[Request]) -> List[Request]:
        for req in reqs:
            now = req.arrival_us
            for I in self.inst:
                self._advance(I, now)
            idx = self._inter_schedule(req, now)
            req.instance = idx
            self.prev_idx = idx
            I = self.inst[idx]
            I.pending.append(req)
            if I.running is None:
                self._start_next(I, now)
        for I in self.inst:
            self._advance(I, None)
        return reqs


def simulate(cfg: Config, reqs: List[Request]) -> List[Request]:
    return MacroInstance(cfg).run(reqs)


def slo_attainment(cfg: Config, reqs: Sequence[Request]) -> float:
    """Share of requests that meet both SLOs (Section 4.1): TTFT = first token - arrival (phase-switching
    wait included, Section 3.3), TPOT = (finish - first token) / (output tokens after the first)."""
    ok = 0
    for r in reqs:
        ttft = r.first_token_us - r.arrival_us
        tpot_ok = r.output_len == 1 or (r.finish_us - r.first_token_us) <= cfg.slo_tpot_us * (r.output_len - 1)
        ok += ttft <= cfg.slo_ttft_us and tpot_ok
    return ok / max(len(reqs), 1)
