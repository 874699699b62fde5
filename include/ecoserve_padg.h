/*
 * ecoserve_padg.h -- host-side model of one EcoServe macro instance: the
 * inter-instance scheduling of Section 3.4 (Algorithm 1, InterSchedule, and
 * Algorithm 2, CheckConstraints) over instances that each follow the
 * temporal disaggregation of Section 3.2.1 (one phase at a time, prefills
 * first), driven by measured step durations.  It turns kernel timings into
 * the paper's currency: TTFT, TPOT and SLO attainment of a request stream
 * (Section 3.3, Section 4.1).  No GPU is involved; everything is host
 * memory and every pointer is a host pointer owned by the caller.
 *
 * All times are integer microseconds, all sizes are tokens, so that the
 * result is exactly reproducible.  Status codes are those of ecoserve.h.
 *
 * The model, step by step (the readings of the paper are listed in the
 * repository's design notes):
 *
 *  Requests arrive in order of `arrival_us`.  At an arrival, every instance
 *  is first advanced to that time (batches that end at or before it are
 *  completed), then Algorithm 1 picks the instance and the request joins that
 *  instance's pending prefills.
 *
 *  An instance runs one batch at a time, back to back:
 *    - if it has pending prefills when a batch ends (or when work arrives at
 *      an idle instance), it is in its prefill phase and runs the prefill of
 *      the oldest pending request alone; at the end of that batch the request
 *      has its first token (counted as output token 1) and joins the decodes,
 *      or is finished if output_len == 1;
 *    - otherwise, if it has decoding requests, it runs one decode step over
 *      all of them; at its end each has one more token and those that reached
 *      output_len are finished and release their cache;
 *    - otherwise it is idle.
 *    A prefill phase begins when a pending prefill is started after a decode
 *    step or from idle, and lasts until a decode step starts or the instance
 *    falls idle.
 *
 *  Durations: prefill of a request with n input tokens = piecewise-linear
 *  interpolation through the profile points (extrapolating the first / last
 *  segment outside them, never below 1), the predictor Algorithm 2 asks for
 *  (Section 3.4: profiled in advance for sequences of various lengths);
 *  decode step over b sequences holding t cached tokens in total =
 *  decode_base_us + (decode_per_seq_ns * b + decode_per_token_ns * t) / 1000.
 *
 *  Algorithm 2, for instance I and request r at time `now`:
 *    1. t_total = sum of the predicted prefill durations of the requests of
 *       I's current prefill phase (already prefilled in it, being prefilled,
 *       or still pending -- the pending ones also while I is still finishing
 *       a decode step) and of r.
 *       t_total > slo_ttft_us: not satisfied (reason 1).
 *    2. for every request that was decoding on I before this prefill phase
 *       (all decoding requests if I is decoding):
 *         saved = generated_tokens * slo_tpot_us - (now - first_token_us);
 *       mean(saved) < t_total: not satisfied (reason 2).  No such request:
 *       the constraint holds.
 *    3. r's input tokens > kv_capacity_tokens - tokens cached on I
 *       (input + generated of its unfinished requests, pending ones
 *       included): not satisfied (reason 3).
 *
 *  Algorithm 1: try the instance the previous request was routed to (instance
 *  0 for the first request); if Algorithm 2 is not satisfied, take the next
 *  instance cyclically -- as printed, without checking it (search_all == 0),
 *  or, as the text of Section 3.4 reads, checking each following instance in
 *  turn and falling back to the next one only if none satisfies
 *  (search_all == 1).
 */
#ifndef ECOSERVE_PADG_H
#define ECOSERVE_PADG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int64_t arrival_us;
  int32_t input_len;  /* >= 1 */
  int32_t output_len; /* >= 1, the first token included */
} ecoserve_padg_request;

typedef struct {
  int32_t n_instances; /* >= 1 */
  int32_t search_all;  /* Algorithm 1: 0 as printed, 1 cyclic search */
  int64_t slo_ttft_us;
  int64_t slo_tpot_us;
  int64_t kv_capacity_tokens; /* per instance */
  int32_t n_prefill_points;   /* >= 2 */
  const int32_t* prefill_len; /* host [n_prefill_points], strictly increasing, >= 1 */
  const int64_t* prefill_us;  /* host [n_prefill_points], >= 1 */
  int64_t decode_base_us;
  int64_t decode_per_seq_ns;
  int64_t decode_per_token_ns;
} ecoserve_padg_config;

typedef struct {
  int32_t instance;       /* where Algorithm 1 sent the request */
  int32_t check;          /* Algorithm 2 on the instance tried first: 0 satisfied, else the reason 1..3 */
  int64_t first_token_us; /* end of its prefill batch */
  int64_t finish_us;      /* end of the batch that produced its last token */
} ecoserve_padg_result;

/* Predicted prefill duration of a request with `input_len` tokens.  Returns -1 on a bad config. */
int64_t ecoserve_padg_prefill_us(const ecoserve_padg_config* cfg, int32_t input_len);

/*
 * Algorithm 2 on an explicit snapshot of an instance: the input lengths of
 * the requests of its current prefill phase, the (generated tokens, first
 * token time) of the requests that were decoding before it, the tokens it has
 * cached, and the candidate.  Returns 0 (satisfied) or the reason 1..3;
 * negative status (-ECOSERVE_EINVAL) on bad arguments.
 */
int ecoserve_padg_check_constraints(const ecoserve_padg_config* cfg, int64_t now_us, const int32_t* phase_input_len,
                                    int32_t n_phase, const int32_t* decode_generated,
                                    const int64_t* decode_first_token_us, int32_t n_decode, int64_t kv_used_tokens,
                                    int32_t req_input_len);

/*
 * Runs the whole stream.  `reqs` must be sorted by arrival_us (ties keep their
 * order); `out[i]` describes request i.  ECOSERVE_EINVAL on a bad config or an
 * unsorted or malformed stream.  Deterministic; no state is kept.
 */
int ecoserve_padg_simulate(const ecoserve_padg_config* cfg, const ecoserve_padg_request* reqs, int64_t n_reqs,
                           ecoserve_padg_result* out);

#ifdef __cplusplus
}
#endif
#endif /* ECOSERVE_PADG_H */
