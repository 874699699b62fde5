// Host-side paths of libecoserve under ASan/UBSan (api.hip and padg.hip compiled with the sanitizers on the
// host pass, see tests/test_host_sanitizers.py): everything a process without a GPU can reach.  The helper
// calls with valid and invalid layouts, every status string, the hot calls' argument checks that return
// before any HIP call, context creation where no device answers, and the macro-instance model (Algorithms 1
// and 2) on a seeded stream of requests with both routing variants.  The program checks return codes only;
// the sanitizers check the memory accesses and the arithmetic.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "ecoserve.h"
#include "ecoserve_padg.h"

static int fails = 0;
#define EXPECT(cond)                                                  \
  do {                                                                \
    if (!(cond)) {                                                    \
      std::printf("%s:%d: %s is false\n", __FILE__, __LINE__, #cond); \
      ++fails;                                                        \
    }                                                                 \
  } while (0)

static uint32_t rng_state = 2024u;
static uint32_t rnd() {
  rng_state = rng_state * 1664525u + 1013904223u;
  return rng_state >> 8;
}

int main() {
  // ---- helpers ------------------------------------------------------------------------------------------
  for (int st = -1; st <= 7; ++st) EXPECT(std::strlen(ecoserve_strerror(st)) > 0);
  ecoserve_layout lay = {40, 8, 128, 16, 1000, ECOSERVE_BF16, 0.0f};
  EXPECT(ecoserve_cache_bytes(&lay) == (size_t)1000 * 8 * 16 * 128 * 2);
  EXPECT(ecoserve_cache_bytes(nullptr) == 0);
  ecoserve_layout bad = lay;
  bad.num_q_heads = 41;
  EXPECT(ecoserve_cache_bytes(&bad) == 0);
  bad = lay;
  bad.block_size = 32;
  EXPECT(ecoserve_cache_bytes(&bad) == 0);
  // the two index maps are bijections onto one (block, head) piece
  std::vector<uint8_t> seen_k(16 * 128, 0), seen_v(16 * 128, 0);
  const size_t base_k = ecoserve_k_cache_index(&lay, 7, 3, 0, 0), base_v = ecoserve_v_cache_index(&lay, 7, 3, 0, 0);
  for (int slot = 0; slot < 16; ++slot)
    for (int d = 0; d < 128; ++d) {
      const size_t ik = ecoserve_k_cache_index(&lay, 7, 3, slot, d) - base_k + (base_k % 2048);
      const size_t iv = ecoserve_v_cache_index(&lay, 7, 3, slot, d) - base_v + (base_v % 2048);
      EXPECT(ik < 2048 && iv < 2048);
      if (ik < 2048) seen_k[ik]++;
      if (iv < 2048) seen_v[iv]++;
    }
  for (int i = 0; i < 2048; ++i) EXPECT(seen_k[i] == 1 && seen_v[i] == 1);
  EXPECT(ecoserve_workspace_bytes(nullptr) == 0);

  // ---- calls that must fail before they touch a device ----------------------------------------------------
  ecoserve_ctx* ctx = nullptr;
  EXPECT(ecoserve_create(nullptr, 0, &lay, 1, 1) == ECOSERVE_EINVAL);
  EXPECT(ecoserve_create(&ctx, 0, &bad, 1, 1) == ECOSERVE_EUNSUPPORTED && ctx == nullptr);
  EXPECT(ecoserve_create(&ctx, 0, &lay, 0, 1) == ECOSERVE_EINVAL && ctx == nullptr);
  EXPECT(ecoserve_create(&ctx, -1, &lay, 1, 1) == ECOSERVE_EINVAL && ctx == nullptr);
  // a valid request: with no GPU in the machine it reports the runtime's refusal (and leaks nothing)
  const int st = ecoserve_create(&ctx, 0, &lay, 16, 256);
  EXPECT(st == ECOSERVE_OK || st == ECOSERVE_EHIP || st == ECOSERVE_EINVAL || st == ECOSERVE_ENOMEM);
  if (st == ECOSERVE_OK) EXPECT(ecoserve_destroy(ctx) == ECOSERVE_OK);
  EXPECT(ecoserve_destroy(nullptr) == ECOSERVE_OK);
  EXPECT(ecoserve_set_option(nullptr, ECOSERVE_OPT_PROFILE, 1) == ECOSERVE_EINVAL);
  EXPECT(ecoserve_kv_append(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 1, 1, 1, 1, nullptr) ==
         ECOSERVE_EINVAL);
  EXPECT(ecoserve_attn_prefill(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 1, nullptr, nullptr, 1, 1, 1,
                               nullptr) == ECOSERVE_EINVAL);
  EXPECT(ecoserve_attn_decode(nullptr, nullptr, nullptr, nullptr, nullptr, 1, nullptr, nullptr, nullptr, 1, 1, nullptr) ==
         ECOSERVE_EINVAL);
  EXPECT(ecoserve_attn_decode_append(nullptr, nullptr, 0, nullptr, nullptr, 0, nullptr, nullptr, nullptr, 1, nullptr, nullptr,
                                     nullptr, 1, 1, nullptr) == ECOSERVE_EINVAL);
  EXPECT(ecoserve_debug_validate(nullptr, nullptr, nullptr, nullptr, 1, 1) == ECOSERVE_EINVAL);
  float sh[8];
  EXPECT(ecoserve_debug_prefill_queue_shares(nullptr, sh) == ECOSERVE_EINVAL);
  double x = 0.0;
  int64_t n = 0;
  EXPECT(ecoserve_profile_read(nullptr, 0, &x, &n) == ECOSERVE_EINVAL);
  EXPECT(ecoserve_profile_reset(nullptr) == ECOSERVE_EINVAL);
  EXPECT(ecoserve_probe_hbm_read(0, 100, 1, &x) == ECOSERVE_EINVAL);
  EXPECT(ecoserve_probe_mfma_bf16(0, 0, 0, &x) == ECOSERVE_EINVAL);
  EXPECT(ecoserve_probe_mfma_valu(0, 1, 3, 0, 2, &x, &x) == ECOSERVE_EINVAL);
  EXPECT(ecoserve_attn_decode_noalloc(0, &bad, nullptr, nullptr, nullptr, nullptr, 1, nullptr, nullptr, nullptr, 1, 1, nullptr) ==
         ECOSERVE_EUNSUPPORTED);
  EXPECT(ecoserve_attn_decode_noalloc(0, &lay, nullptr, nullptr, nullptr, nullptr, 1, nullptr, nullptr, nullptr, 0, 1, nullptr) ==
         ECOSERVE_OK);
  EXPECT(ecoserve_attn_decode_noalloc(0, &lay, nullptr, nullptr, nullptr, nullptr, 1, nullptr, nullptr, nullptr, 1, 1, nullptr) ==
         ECOSERVE_EINVAL);

  // ---- the macro-instance model -----------------------------------------------------------------------------
  const int32_t plen[] = {16, 64, 256, 1024, 2048, 4096};
  const int64_t pus[] = {21000, 24000, 38000, 72000, 131000, 255000};
  for (int variant = 0; variant < 4; ++variant) {
    ecoserve_padg_config cfg;
    cfg.n_instances = 1 + 3 * (variant & 1);
    cfg.search_all = variant >> 1;
    cfg.slo_ttft_us = 1000000;
    cfg.slo_tpot_us = 100000;
    cfg.kv_capacity_tokens = variant == 3 ? 20000 : 750000;
    cfg.n_prefill_points = 6;
    cfg.prefill_len = plen;
    cfg.prefill_us = pus;
    cfg.decode_base_us = 21200;
    cfg.decode_per_seq_ns = 53000;
    cfg.decode_per_token_ns = 41;
    EXPECT(ecoserve_padg_prefill_us(&cfg, 1) > 0 && ecoserve_padg_prefill_us(&cfg, 100000) > 0);
    EXPECT(ecoserve_padg_prefill_us(&cfg, 300) >= ecoserve_padg_prefill_us(&cfg, 256));
    std::vector<ecoserve_padg_request> reqs(3000);
    int64_t t = 0;
    for (auto& r : reqs) {
      t += rnd() % 60000;
      r.arrival_us = t;
      r.input_len = 1 + (int32_t)(rnd() % 4096);
      r.output_len = 1 + (int32_t)(rnd() % 300);
    }
    std::vector<ecoserve_padg_result> out(reqs.size());
    EXPECT(ecoserve_padg_simulate(&cfg, reqs.data(), (int64_t)reqs.size(), out.data()) == ECOSERVE_OK);
    for (size_t i = 0; i < reqs.size(); ++i) {
      EXPECT(out[i].instance >= 0 && out[i].instance < cfg.n_instances);
      EXPECT(out[i].first_token_us > reqs[i].arrival_us && out[i].finish_us >= out[i].first_token_us);
    }
    EXPECT(ecoserve_padg_simulate(&cfg, reqs.data(), 0, out.data()) == ECOSERVE_OK);
    std::swap(reqs[10], reqs[2000]);  // unsorted
    EXPECT(ecoserve_padg_simulate(&cfg, reqs.data(), (int64_t)reqs.size(), out.data()) == ECOSERVE_EINVAL);
    const int32_t phase[] = {100, 2000, 37};
    const int32_t gen[] = {5, 1, 200};
    const int64_t first[] = {1000, 90000, 5000};
    const int c = ecoserve_padg_check_constraints(&cfg, 100000, phase, 3, gen, first, 3, 10000, 512);
    EXPECT(c >= 0 && c <= 3);
    EXPECT(ecoserve_padg_check_constraints(&cfg, 100000, nullptr, 0, nullptr, nullptr, 0, 0, 512) == 0);
    EXPECT(ecoserve_padg_check_constraints(nullptr, 0, nullptr, 0, nullptr, nullptr, 0, 0, 1) < 0);
    cfg.n_prefill_points = 1;
    EXPECT(ecoserve_padg_prefill_us(&cfg, 10) == -1);
  }
  std::printf(fails ? "host driver FAILED (%d checks)\n" : "host driver ok\n", fails);
  return fails ? 1 : 0;
}
