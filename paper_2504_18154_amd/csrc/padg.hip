// Host-side model of one EcoServe macro instance (no device code in this file).
//
// Section 3.2.1 of the paper: every instance runs one phase at a time for an extended duration
// and puts prefills first.  Section 3.4: Algorithm 1 (InterSchedule) routes each request to the
// instance that took the previous one while Algorithm 2 (CheckConstraints: the prefill phase must
// fit the TTFT SLO, the interrupted decodes must have saved enough TPOT on average, the KV cache
// must fit) allows it, else moves on cyclically -- which staggers the instances' prefill phases
// (rolling activation, Section 3.2.2).  The exact rules of the model are stated in
// include/ecoserve_padg.h; this file is their only implementation on the product side.
//
// Requests are kept in flat arrays and referred to by index; an instance is three index lists
// and a running batch.  Time is integer microseconds.
#include <stdint.h>

#include <algorithm>
#include <limits>
#include <vector>

#include "../../include/ecoserve.h"
#include "../../include/ecoserve_padg.h"

namespace {

constexpr int64_t kNever = std::numeric_limits<int64_t>::max();

// floor(a / b) for b > 0
int64_t floor_div(int64_t a, int64_t b) {
  int64_t q = a / b;
  if ((a % b != 0) && (a < 0)) --q;
  return q;
}

bool config_ok(const ecoserve_padg_config* c) {
  if (!c || c->n_instances < 1 || c->n_prefill_points < 2 || !c->prefill_len || !c->prefill_us) return false;
  if (c->slo_ttft_us < 0 || c->slo_tpot_us < 0 || c->kv_capacity_tokens < 0) return false;
  if (c->decode_base_us < 0 || c->decode_per_seq_ns < 0 || c->decode_per_token_ns < 0) return false;
  for (int32_t k = 0; k < c->n_prefill_points; ++k) {
    if (c->prefill_len[k] < 1 || c->prefill_us[k] < 1) return false;
    if (k > 0 && c->prefill_len[k] <= c->prefill_len[k - 1]) return false;
  }
  return true;
}

// Section 3.4: the predictor profiled over sequence lengths
int64_t predict_prefill(const ecoserve_padg_config& c, int32_t n) {
  const int32_t* L = c.prefill_len;
  const int64_t* U = c.prefill_us;
  // the segment [L[k], L[k+1]) that holds n; the first and the last one also serve what lies outside
  int32_t k = (int32_t)(std::upper_bound(L + 1, L + c.n_prefill_points - 1, n) - (L + 1));
  const int64_t t = U[k] + floor_div((U[k + 1] - U[k]) * (int64_t)(n - L[k]), (int64_t)(L[k + 1] - L[k]));
  return t < 1 ? 1 : t;
}

int64_t decode_step(const ecoserve_padg_config& c, int64_t batch, int64_t tokens) {
  return c.decode_base_us + (c.decode_per_seq_ns * batch + c.decode_per_token_ns * tokens) / 1000;
}

// Algorithm 2 with the sums already taken: t_phase = predicted durations of the phase's requests,
// saved_sum / n_saved = the interrupted decodes' saved TPOT, free_tokens = what the cache has left.
int check(const ecoserve_padg_config& c, int64_t t_phase, int64_t saved_sum, int64_t n_saved, int64_t free_tokens,
          int32_t req_input_len) {
  const int64_t t_total = t_phase + predict_prefill(c, req_input_len);
  if (t_total > c.slo_ttft_us) return 1;
  if (n_saved > 0 && saved_sum < t_total * n_saved) return 2;  // mean(saved) < t_total
  if ((int64_t)req_input_len > free_tokens) return 3;
  return 0;
}

enum Batch { kIdle, kPrefill, kDecode };

struct Sim {
  const ecoserve_padg_config& c;
  const ecoserve_padg_request* req;
  ecoserve_padg_result* res;
  std::vector<int32_t> generated;  // per request
  std::vector<char> in_phase;      // per request: prefilled in its instance's current prefill phase

  struct Instance {
    std::vector<int64_t> pending;   // request indices, oldest first
    std::vector<int64_t> decoding;  // in the order they got their first token
    std::vector<int64_t> phase;     // prefilled in the current prefill phase
    Batch running = kIdle;
    int64_t end = kNever;
    int64_t prefilling = -1;
  };
  std::vector<Instance> inst;

  Sim(const ecoserve_padg_config& cfg, const ecoserve_padg_request* r, int64_t n, ecoserve_padg_result* out)
      : c(cfg), req(r), res(out), generated((size_t)n, 0), in_phase((size_t)n, 0), inst((size_t)cfg.n_instances) {}

  void end_phase(Instance& I) {
    for (int64_t r : I.phase) in_phase[(size_t)r] = 0;
    I.phase.clear();
  }

  // the instance has just become free at `now`: prefills first, then a decode step, else idle
  void start_next(Instance& I, int64_t now) {
    if (!I.pending.empty()) {
      I.prefilling = I.pending.front();
      I.pending.erase(I.pending.begin());
      I.running = kPrefill;
      I.end = now + predict_prefill(c, req[I.prefilling].input_len);
    } else if (!I.decoding.empty()) {
      end_phase(I);
      int64_t tokens = 0;
      for (int64_t r : I.decoding) tokens += (int64_t)req[r].input_len + generated[(size_t)r];
      I.running = kDecode;
      I.end = now + decode_step(c, (int64_t)I.decoding.size(), tokens);
    } else {
      end_phase(I);
      I.running = kIdle;
      I.end = kNever;
    }
  }

  void complete(Instance& I) {
    const int64_t now = I.end;
    if (I.running == kPrefill) {
      const int64_t r = I.prefilling;
      I.prefilling = -1;
      res[r].first_token_us = now;
      generated[(size_t)r] = 1;
      I.phase.push_back(r);
      in_phase[(size_t)r] = 1;
      if (req[r].output_len == 1)
        res[r].finish_us = now;
      else
        I.decoding.push_back(r);
    } else {
      size_t keep = 0;
      for (size_t i = 0; i < I.decoding.size(); ++i) {
        const int64_t r = I.decoding[i];
        if (++generated[(size_t)r] == req[r].output_len)
          res[r].finish_us = now;
        else
          I.decoding[keep++] = r;
      }
      I.decoding.resize(keep);
    }
    start_next(I, now);
  }

  void advance(Instance& I, int64_t now) {
    while (I.running != kIdle && I.end <= now) complete(I);
  }

  int check_live(const Instance& I, int64_t r_new, int64_t now) const {
    int64_t t_phase = 0, used = 0;
    for (int64_t r : I.phase) t_phase += predict_prefill(c, req[r].input_len);
    if (I.running == kPrefill) {
      t_phase += predict_prefill(c, req[I.prefilling].input_len);
      used += req[I.prefilling].input_len;
    }
    for (int64_t r : I.pending) {
      t_phase += predict_prefill(c, req[r].input_len);
      used += req[r].input_len;
    }
    int64_t saved = 0, n_saved = 0;
    for (int64_t r : I.decoding) {
      used += (int64_t)req[r].input_len + generated[(size_t)r];
      if (in_phase[(size_t)r]) continue;  // it joined the decodes in this very phase: nothing of it was interrupted
      saved += (int64_t)generated[(size_t)r] * c.slo_tpot_us - (now - res[r].first_token_us);
      ++n_saved;
    }
    return check(c, t_phase, saved, n_saved, c.kv_capacity_tokens - used, req[r_new].input_len);
  }
};

}  // namespace

extern "C" {

int64_t ecoserve_padg_prefill_us(const ecoserve_padg_config* cfg, int32_t input_len) {
  if (!config_ok(cfg) || input_len < 1) return -1;
  return predict_prefill(*cfg, input_len);
}

int ecoserve_padg_check_constraints(const ecoserve_padg_config* cfg, int64_t now_us, const int32_t* phase_input_len,
                                    int32_t n_phase, const int32_t* decode_generated,
                                    const int64_t* decode_first_token_us, int32_t n_decode, int64_t kv_used_tokens,
                                    int32_t req_input_len) {
  if (!config_ok(cfg) || n_phase < 0 || n_decode < 0 || req_input_len < 1 || kv_used_tokens < 0) return -ECOSERVE_EINVAL;
  if ((n_phase > 0 && !phase_input_len) || (n_decode > 0 && (!decode_generated || !decode_first_token_us)))
    return -ECOSERVE_EINVAL;
  int64_t t_phase = 0, saved = 0;
  for (int32_t i = 0; i < n_phase; ++i) {
    if (phase_input_len[i] < 1) return -ECOSERVE_EINVAL;
    t_phase += predict_prefill(*cfg, phase_input_len[i]);
  }
  for (int32_t i = 0; i < n_decode; ++i)
    saved += (int64_t)decode_generated[i] * cfg->slo_tpot_us - (now_us - decode_first_token_us[i]);
  return check(*cfg, t_phase, saved, n_decode, cfg->kv_capacity_tokens - kv_used_tokens, req_input_len);
}

int ecoserve_padg_simulate(const ecoserve_padg_config* cfg, const ecoserve_padg_request* reqs, int64_t n_reqs,
                           ecoserve_padg_result* out) {
  if (!config_ok(cfg) || n_reqs < 0 || (n_reqs > 0 && (!reqs || !out))) return ECOSERVE_EINVAL;
  for (int64_t i = 0; i < n_reqs; ++i) {
    if (reqs[i].input_len < 1 || reqs[i].output_len < 1 || reqs[i].arrival_us < 0) return ECOSERVE_EINVAL;
    if (i > 0 && reqs[i].arrival_us < reqs[i - 1].arrival_us) return ECOSERVE_EINVAL;
  }
  Sim sim(*cfg, reqs, n_reqs, out);
  const int32_t n = cfg->n_instances;
  int32_t prev = 0;
  for (int64_t r = 0; r < n_reqs; ++r) {
    const int64_t now = reqs[r].arrival_us;
    out[r].first_token_us = out[r].finish_us = -1;
    for (auto& I : sim.inst) sim.advance(I, now);
    // Algorithm 1
    int32_t target = prev;
    out[r].check = sim.check_live(sim.inst[(size_t)prev], r, now);
    if (out[r].check != 0) {
      target = (prev + 1) % n;
      if (cfg->search_all) {
        for (int32_t k = 1; k < n; ++k) {
          const int32_t idx = (prev + k) % n;
          if (sim.check_live(sim.inst[(size_t)idx], r, now) == 0) {
            target = idx;
            break;
          }
        }
      }
    }
    out[r].instance = target;
    prev = target;
    auto& I = sim.inst[(size_t)target];
    I.pending.push_back(r);
    if (I.running == kIdle) sim.start_next(I, now);
  }
  for (auto& I : sim.inst) sim.advance(I, kNever);
  return ECOSERVE_OK;
}

}  // extern "C"
