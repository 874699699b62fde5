// C ABI of the library (see include/ecoserve.h): context management, host-side
// validation, launch planning and dispatch to the kernels.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <vector>

#include "common.h"

using namespace eco;

namespace eco {

bool layout_ok(const ecoserve_layout* L, int* status) {
  *status = ECOSERVE_EINVAL;
  if (!L) return false;
  if (L->num_q_heads <= 0 || L->num_kv_heads <= 0 || L->head_dim <= 0 || L->block_size <= 0 || L->num_blocks < 0)
    return false;
  if (L->num_q_heads % L->num_kv_heads != 0) return false;
  if (L->dtype != ECOSERVE_BF16 && L->dtype != ECOSERVE_F32) return false;
  if (!(L->softmax_scale >= 0.f) || isinf(L->softmax_scale)) return false;
  *status = ECOSERVE_EUNSUPPORTED;
  if (L->block_size != kBlockSize) return false;
  if (L->num_q_heads / L->num_kv_heads > kMaxGroup) return false;
  const int X = L->dtype == ECOSERVE_BF16 ? 8 : 4;
  if (L->head_dim % X != 0 || L->head_dim > 256) return false;
  *status = ECOSERVE_OK;
  return true;
}

}  // namespace eco

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool use_mfma(const ecoserve_ctx* c) {
  return !c->opt_force_plain && c->lay.dtype == ECOSERVE_BF16 && c->lay.head_dim == 128;
}

int32_t ceil_div(int32_t a, int32_t b) { return (a + b - 1) / b; }

// Tokens per decode split.  Smaller splits balance ragged contexts across the 256 CUs
// and shorten the tail; larger ones write fewer partial states.
int32_t plan_split_tokens(const ecoserve_ctx* c, int32_t B, int32_t max_ctx_len) {
  if (c->opt_split_tokens > 0) return c->opt_split_tokens;
  const int64_t heads = c->lay.num_q_heads;
  const int64_t want = 8LL * c->num_cu;  // workgroups needed to fill the chip a few times over
  int32_t st = 512;
  while (st > kMinSplitTokens && (int64_t)B * heads * ceil_div(max_ctx_len, st) < want) st >>= 1;
  return st;
}

// Partial-state slots (128 floats of ws_acc and 2 of ws_ml each) the context's current options can ask for.
// Matrix-core decode: two groups of G per wavefront of the launch - the persistent grid, or the larger grid
// of a forced split at the context's limits.  Plain decode: one per (sequence, query head, split).
int64_t slots_needed(const ecoserve_ctx* c, int32_t* plain_splits) {
  *plain_splits = 0;
  if (use_mfma(c)) {
    const int64_t waves = decode_mfma_waves(c->max_batch, c->lay.num_kv_heads, c->max_blocks_per_seq * kBlockSize,
                                            c->opt_split_tokens, c->num_cu * kDecodeWgsPerCu);
    return 2 * waves * (c->lay.num_q_heads / c->lay.num_kv_heads);
  }
  // a sequence of n blocks cut into chunks of >= c blocks at arbitrary offsets has at most n/c + 2 pieces
  *plain_splits = ceil_div(c->max_blocks_per_seq * kBlockSize, kMinSplitTokens) + 2;
  return (int64_t)c->max_batch * c->lay.num_q_heads * *plain_splits;
}

// Makes the partial-state arrays large enough for the current options (they only ever grow).  Called where
// allocation is allowed: ecoserve_create and ecoserve_set_option.
int ensure_partial_states(ecoserve_ctx* c) {
  int32_t plain_splits;
  const int64_t need = slots_needed(c, &plain_splits);
  if (plain_splits) c->ws_splits = plain_splits;
  if (need <= c->ws_slots) return ECOSERVE_OK;
  if (c->ws_acc || c->ws_ml) {
    if (hipDeviceSynchronize() != hipSuccess) return ECOSERVE_EHIP;  // launches in flight may still use them
    if (c->ws_acc) (void)hipFree(c->ws_acc);
    if (c->ws_ml) (void)hipFree(c->ws_ml);
    c->ws_bytes -= (size_t)c->ws_slots * (c->lay.head_dim + 2) * sizeof(float);
  }
  c->ws_acc = nullptr;
  c->ws_ml = nullptr;
  c->ws_slots = 0;
  const size_t acc_bytes = (size_t)need * c->lay.head_dim * sizeof(float);
  const size_t ml_bytes = (size_t)need * 2 * sizeof(float);
  if (hipMalloc(&c->ws_acc, acc_bytes) != hipSuccess || hipMalloc(&c->ws_ml, ml_bytes) != hipSuccess) {
    (void)hipGetLastError();
    if (c->ws_acc) (void)hipFree(c->ws_acc);
    c->ws_acc = nullptr;
    c->ws_ml = nullptr;
    return ECOSERVE_ENOMEM;
  }
  c->ws_slots = need;
  c->ws_bytes += acc_bytes + ml_bytes;
  return ECOSERVE_OK;
}

// The parts of the workspace whose size the options do not change: the decode launch's numbering and the
// prefill plan.
int alloc_fixed_workspace(ecoserve_ctx* c) {
  const size_t meta_bytes = ((size_t)c->max_batch + 19) * sizeof(int32_t);
  // a prefill batch cannot bring more new tokens than the pool holds
  c->plan_tiles = prefill_plan_tiles(c->max_batch, (int32_t)std::min<int64_t>(
                                                        (int64_t)c->lay.num_blocks * kBlockSize, 0x7fffffffLL));
  const size_t plan_bytes = ((size_t)kPlanHeaderInts + (size_t)c->plan_tiles * kRecInts) * sizeof(int32_t);
  if (hipMalloc(&c->ws_meta, meta_bytes) != hipSuccess || hipMalloc(&c->ws_plan, plan_bytes) != hipSuccess) {
    (void)hipGetLastError();
    return ECOSERVE_ENOMEM;
  }
  // the plan's header carries state from one prefill launch to the next (queue shares, busy times): none yet
  if (hipMemset(c->ws_plan, 0, (size_t)kPlanHeaderInts * sizeof(int32_t)) != hipSuccess) {
    (void)hipGetLastError();
    return ECOSERVE_EHIP;
  }
  c->ws_bytes += meta_bytes + plan_bytes;
  return ECOSERVE_OK;
}

// Profiling: a pair of events around the dominant kernel of a hot call (of every n-th call of a kind).
struct ProfileScope {
  ecoserve_ctx* c;
  int which;
  hipStream_t s;
  EventPair* ep;
  ProfileScope(ecoserve_ctx* ctx, int w, hipStream_t st) : c(ctx), which(w), s(st), ep(nullptr) {
    if (!c->opt_profile || c->prof_seq[which]++ % (uint32_t)c->opt_profile != 0) return;
    if (c->ev_used[which] == c->ev[which].size()) {
      EventPair e;
      if (hipEventCreate(&e.start) != hipSuccess) return;
      if (hipEventCreate(&e.stop) != hipSuccess) { (void)hipEventDestroy(e.start); return; }
      c->ev[which].push_back(e);
    }
    ep = &c->ev[which][c->ev_used[which]++];
    (void)hipEventRecord(ep->start, s);
  }
  ~ProfileScope() {
    if (ep) (void)hipEventRecord(ep->stop, s);
  }
};

}  // namespace

extern "C" {

const char* ecoserve_strerror(int status) {
  switch (status) {
    case ECOSERVE_OK: return "ok";
    case ECOSERVE_EINVAL: return "invalid argument";
    case ECOSERVE_EUNSUPPORTED: return "unsupported layout (block size, head size, group size or dtype)";
    case ECOSERVE_ENOMEM: return "out of memory";
    case ECOSERVE_EHIP: return "HIP runtime error";
    case ECOSERVE_ECONTENT: return "device-resident argument contents out of range";
    default: return "unknown status";
  }
}

size_t ecoserve_cache_bytes(const ecoserve_layout* L) {
  int st;
  if (!layout_ok(L, &st)) return 0;
  const size_t es = L->dtype == ECOSERVE_BF16 ? 2 : 4;
  return (size_t)L->num_blocks * L->num_kv_heads * L->block_size * L->head_dim * es;
}

size_t ecoserve_k_cache_index(const ecoserve_layout* L, int32_t blk, int32_t g, int32_t slot, int32_t d) {
  const size_t X = L->dtype == ECOSERVE_BF16 ? 8 : 4;
  const size_t D = L->head_dim, bs = L->block_size;
  return ((((size_t)blk * L->num_kv_heads + g) * (D / X) + d / X) * bs + slot) * X + d % X;
}

size_t ecoserve_v_cache_index(const ecoserve_layout* L, int32_t blk, int32_t g, int32_t slot, int32_t d) {
  const size_t D = L->head_dim, bs = L->block_size;
  return (((size_t)blk * L->num_kv_heads + g) * D + d) * bs + slot;
}

size_t ecoserve_workspace_bytes(const ecoserve_ctx* ctx) { return ctx ? ctx->ws_bytes : 0; }

int ecoserve_create(ecoserve_ctx** out, int device, const ecoserve_layout* layout, int32_t max_batch,
                    int32_t max_blocks_per_seq) {
  if (!out) return ECOSERVE_EINVAL;
  *out = nullptr;
  int st;
  if (!layout_ok(layout, &st)) return st;
  if (max_batch <= 0 || max_batch > kMaxBatch || max_blocks_per_seq <= 0 || device < 0) return ECOSERVE_EINVAL;
  if ((int64_t)max_blocks_per_seq * kBlockSize > 0x7fffffffLL) return ECOSERVE_EINVAL;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess) { (void)hipGetLastError(); return ECOSERVE_EHIP; }
  if (device >= ndev) return ECOSERVE_EINVAL;
  DeviceGuard guard(device);
  if (!guard.ok) return ECOSERVE_EHIP;
  ecoserve_ctx* c = new (std::nothrow) ecoserve_ctx();
  if (!c) return ECOSERVE_ENOMEM;
  c->device = device;
  c->lay = *layout;
  c->scale = layout->softmax_scale > 0.f ? layout->softmax_scale : 1.0f / sqrtf((float)layout->head_dim);
  c->max_batch = max_batch;
  c->max_blocks_per_seq = max_blocks_per_seq;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device) != hipSuccess) { delete c; return ECOSERVE_EHIP; }
  c->num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  c->opt_split_tokens = 0;
  c->opt_force_plain = 0;
  c->opt_profile = 0;
  c->opt_adaptive = 0;
  c->opt_reuse_plan = 0;
  c->plan_parity = 0;
  c->plan_key.valid = false;
  c->share_parity = 0;
  c->ws_share = nullptr;
  c->ws_acc = nullptr;
  c->ws_ml = nullptr;
  c->ws_meta = nullptr;
  c->ws_plan = nullptr;
  c->plan_tiles = 0;
  c->ws_splits = 0;
  c->ws_slots = 0;
  c->ws_bytes = 0;
  for (int i = 0; i < 3; ++i) c->ev_used[i] = 0, c->prof_seq[i] = 0;
  st = alloc_fixed_workspace(c);
  if (st == ECOSERVE_OK) st = ensure_partial_states(c);
  if (st == ECOSERVE_OK && prepare_kv_append(c) != hipSuccess) st = ECOSERVE_EHIP;
  if (st != ECOSERVE_OK) { (void)ecoserve_destroy(c); return st; }
  {
    // per-XCD shares start equal; samples of 4 wavefronts per CU follow, then each chunk's report to the merge
    const size_t share_bytes = (24 + 6 * (size_t)c->num_cu * kDecodeWgsPerCu * 4) * sizeof(int32_t);
    const float ones[16] = {1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f};
    if (hipMalloc(&c->ws_share, share_bytes) != hipSuccess || hipMemset(c->ws_share, 0, share_bytes) != hipSuccess ||
        hipMemcpy(c->ws_share, ones, sizeof(ones), hipMemcpyHostToDevice) != hipSuccess) {
      (void)hipGetLastError();
      (void)ecoserve_destroy(c);
      return ECOSERVE_ENOMEM;
    }
    c->ws_bytes += share_bytes;
  }
  *out = c;
  return ECOSERVE_OK;
}

int ecoserve_destroy(ecoserve_ctx* c) {
  if (!c) return ECOSERVE_OK;
  DeviceGuard guard(c->device);
  int rc = ECOSERVE_OK;
  if (!guard.ok || hipDeviceSynchronize() != hipSuccess) rc = ECOSERVE_EHIP;
  if (c->ws_acc) (void)hipFree(c->ws_acc);
  if (c->ws_ml) (void)hipFree(c->ws_ml);
  if (c->ws_meta) (void)hipFree(c->ws_meta);
  if (c->ws_plan) (void)hipFree(c->ws_plan);
  if (c->ws_share) (void)hipFree(c->ws_share);
  for (int i = 0; i < 3; ++i)
    for (EventPair& e : c->ev[i]) { (void)hipEventDestroy(e.start); (void)hipEventDestroy(e.stop); }
  delete c;
  return rc;
}

int ecoserve_set_option(ecoserve_ctx* c, int32_t option, int32_t value) {
  if (!c) return ECOSERVE_EINVAL;
  switch (option) {
    case ECOSERVE_OPT_DECODE_SPLIT_TOKENS: {
      if (value != 0 && (value < kMinSplitTokens || value > kMaxSplitTokens || value % 64 != 0)) return ECOSERVE_EINVAL;
      // a forced split launches a grid that grows with the batch, and so do its partial states
      const int32_t before = c->opt_split_tokens;
      c->opt_split_tokens = value;
      DeviceGuard guard(c->device);
      const int st = guard.ok ? ensure_partial_states(c) : ECOSERVE_EHIP;
      if (st != ECOSERVE_OK) c->opt_split_tokens = before;
      return st;
    }
    case ECOSERVE_OPT_FORCE_PLAIN: {
      const int32_t before = c->opt_force_plain;
      c->opt_force_plain = value ? 1 : 0;
      DeviceGuard guard(c->device);
      const int st = guard.ok ? ensure_partial_states(c) : ECOSERVE_EHIP;
      if (st != ECOSERVE_OK) c->opt_force_plain = before;
      return st;
    }
    case ECOSERVE_OPT_PROFILE:
      if (value < 0) return ECOSERVE_EINVAL;
      c->opt_profile = value;
      return ECOSERVE_OK;
    case ECOSERVE_OPT_DECODE_ADAPTIVE:
      c->opt_adaptive = value ? 1 : 0;
      return ECOSERVE_OK;
    case ECOSERVE_OPT_PREFILL_REUSE_PLAN:
      c->opt_reuse_plan = value ? 1 : 0;
      c->plan_key.valid = false;
      return ECOSERVE_OK;
    default:
      return ECOSERVE_EINVAL;
  }
}

// A row stride in elements: at least the packed row, 16-byte multiples, 32-bit.
static bool stride_ok(const ecoserve_ctx* c, int64_t stride, int32_t heads) {
  const int64_t esize = c->lay.dtype == ECOSERVE_BF16 ? 2 : 4;
  return stride >= (int64_t)heads * c->lay.head_dim && stride < (int64_t)1 << 31 && (stride * esize) % 16 == 0;
}

int ecoserve_kv_append(ecoserve_ctx* c, void* k_cache, void* v_cache, const void* k_new, const void* v_new,
                       const int32_t* cu_q, const int32_t* ctx_before, const int32_t* block_table,
                       int32_t bt_stride, int32_t B, int32_t T, int32_t max_new_len, void* stream) {
  if (!c) return ECOSERVE_EINVAL;
  return ecoserve_kv_append_strided(c, k_cache, v_cache, k_new, v_new,
                                    (int64_t)c->lay.num_kv_heads * c->lay.head_dim, cu_q, ctx_before, block_table,
                                    bt_stride, B, T, max_new_len, stream);
}

int ecoserve_kv_append_strided(ecoserve_ctx* c, void* k_cache, void* v_cache, const void* k_new, const void* v_new,
                               int64_t new_row_stride, const int32_t* cu_q, const int32_t* ctx_before,
                               const int32_t* block_table, int32_t bt_stride, int32_t B, int32_t T,
                               int32_t max_new_len, void* stream) {
  if (!c || B < 0 || T < 0 || max_new_len < 0) return ECOSERVE_EINVAL;
  if (!stride_ok(c, new_row_stride, c->lay.num_kv_heads)) return ECOSERVE_EINVAL;
  if (B == 0 || T == 0) return ECOSERVE_OK;
  if (!k_cache || !v_cache || !k_new || !v_new || !cu_q || !ctx_before || !block_table) return ECOSERVE_EINVAL;
  if (B > c->max_batch || bt_stride <= 0 || max_new_len > T || max_new_len == 0) return ECOSERVE_EINVAL;
  if (!aligned16(k_cache) || !aligned16(v_cache) || !aligned16(k_new) || !aligned16(v_new)) return ECOSERVE_EINVAL;
  DeviceGuard guard(c->device);
  if (!guard.ok) return ECOSERVE_EHIP;
  hipStream_t s = (hipStream_t)stream;
  ProfileScope prof(c, ECOSERVE_KERNEL_APPEND, s);
  const hipError_t e = launch_kv_append(c, k_cache, v_cache, k_new, v_new, (int32_t)new_row_stride, cu_q, ctx_before,
                                        block_table, bt_stride, B, T, max_new_len, 0, s);
  return e == hipSuccess ? ECOSERVE_OK : ECOSERVE_EHIP;
}

static AttnArgs make_args(const ecoserve_ctx* c, const void* q, int64_t q_row_stride, const void* k_cache, const void* v_cache,
                          const int32_t* block_table, int32_t bt_stride, void* out, float* lse, int32_t B) {
  AttnArgs a;
  a.q = q;
  a.q_row_stride = (int32_t)q_row_stride;
  a.k_new = nullptr;
  a.v_new = nullptr;
  a.new_row_stride = 0;
  a.k_cache = k_cache;
  a.v_cache = v_cache;
  a.block_table = block_table;
  a.bt_stride = bt_stride;
  a.out = out;
  a.lse = lse;
  a.B = B;
  a.Hq = c->lay.num_q_heads;
  a.Hkv = c->lay.num_kv_heads;
  a.D = c->lay.head_dim;
  a.dtype = c->lay.dtype;
  a.scale_log2e = c->scale * kLog2e;
  return a;
}

int ecoserve_attn_prefill(ecoserve_ctx* c, const void* q, const void* k_cache, const void* v_cache,
                          const int32_t* cu_q, const int32_t* ctx_before, const int32_t* block_table,
                          int32_t bt_stride, void* out, float* lse, int32_t B, int32_t T, int32_t max_q_len,
                          void* stream) {
  if (!c) return ECOSERVE_EINVAL;
  return ecoserve_attn_prefill_strided(c, q, (int64_t)c->lay.num_q_heads * c->lay.head_dim, k_cache, v_cache, cu_q,
                                       ctx_before, block_table, bt_stride, out, lse, B, T, max_q_len, stream);
}

int ecoserve_attn_prefill_strided(ecoserve_ctx* c, const void* q, int64_t q_row_stride, const void* k_cache,
                                  const void* v_cache, const int32_t* cu_q, const int32_t* ctx_before,
                                  const int32_t* block_table, int32_t bt_stride, void* out, float* lse, int32_t B,
                                  int32_t T, int32_t max_q_len, void* stream) {
  if (!c || B < 0 || T < 0 || max_q_len < 0) return ECOSERVE_EINVAL;
  if (!stride_ok(c, q_row_stride, c->lay.num_q_heads)) return ECOSERVE_EINVAL;
  if (B == 0 || T == 0) return ECOSERVE_OK;
  if (!q || !k_cache || !v_cache || !cu_q || !ctx_before || !block_table || !out) return ECOSERVE_EINVAL;
  if (B > c->max_batch || bt_stride <= 0 || max_q_len > T || max_q_len == 0) return ECOSERVE_EINVAL;
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out)) return ECOSERVE_EINVAL;
  if (lse && (reinterpret_cast<uintptr_t>(lse) & 3u)) return ECOSERVE_EINVAL;
  if (prefill_plan_tiles(B, T) > c->plan_tiles) return ECOSERVE_EINVAL;  // more new tokens than the pool holds
  DeviceGuard guard(c->device);
  if (!guard.ok) return ECOSERVE_EHIP;
  hipStream_t s = (hipStream_t)stream;
  const AttnArgs a = make_args(c, q, q_row_stride, k_cache, v_cache, block_table, bt_stride, out, lse, B);
  ProfileScope prof(c, ECOSERVE_KERNEL_PREFILL, s);
  hipError_t e;
  if (use_mfma(c)) {
    // The tile list depends only on the batch arrays.  With ECOSERVE_OPT_PREFILL_REUSE_PLAN the caller
    // vouches that calls naming the same arrays, B and T see the same contents (the layers of one step),
    // and the list of the first such call serves the following ones.
    const int32_t n_wgs = c->num_cu * kPrefillWgsPerCu;
    const int32_t grid = prefill_mfma_grid(a, T, n_wgs);
    auto& key = c->plan_key;
    if (c->opt_reuse_plan) {
      // whether a recorded launch builds the list or relies on an earlier one would be frozen into the graph
      hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
      if (hipStreamIsCapturing(s, &cap) != hipSuccess) { (void)hipGetLastError(); return ECOSERVE_EHIP; }
      if (cap != hipStreamCaptureStatusNone) return ECOSERVE_EINVAL;
    }
    const bool same = c->opt_reuse_plan && key.valid && key.cu_q == cu_q && key.ctx_before == ctx_before &&
                      key.block_table == block_table && key.bt_stride == bt_stride && key.B == B && key.T == T &&
                      key.n_wg == grid;
    e = launch_prefill_mfma(a, cu_q, ctx_before, T, max_q_len, c->ws_plan, n_wgs, !same, c->plan_parity, s);
    c->plan_parity ^= 1;
    key.valid = e == hipSuccess;
    key.cu_q = cu_q;
    key.ctx_before = ctx_before;
    key.block_table = block_table;
    key.bt_stride = bt_stride;
    key.B = B;
    key.T = T;
    key.n_wg = grid;
  } else
    e = launch_prefill_plain(a, cu_q, ctx_before, T, s);
  return e == hipSuccess ? ECOSERVE_OK : ECOSERVE_EHIP;
}

static int decode_impl(ecoserve_ctx* c, const void* q, int64_t q_row_stride, const void* k_new, const void* v_new,
                       int64_t new_row_stride, void* k_cache, void* v_cache,
                       const int32_t* block_table, int32_t bt_stride, const int32_t* ctx_len, void* out, float* lse,
                       int32_t B, int32_t max_ctx_len, void* stream);

int ecoserve_attn_decode(ecoserve_ctx* c, const void* q, const void* k_cache, const void* v_cache,
                         const int32_t* block_table, int32_t bt_stride, const int32_t* ctx_len, void* out,
                         float* lse, int32_t B, int32_t max_ctx_len, void* stream) {
  if (!c) return ECOSERVE_EINVAL;
  return ecoserve_attn_decode_strided(c, q, (int64_t)c->lay.num_q_heads * c->lay.head_dim, k_cache, v_cache,
                                      block_table, bt_stride, ctx_len, out, lse, B, max_ctx_len, stream);
}

int ecoserve_attn_decode_strided(ecoserve_ctx* c, const void* q, int64_t q_row_stride, const void* k_cache,
                                 const void* v_cache, const int32_t* block_table, int32_t bt_stride,
                                 const int32_t* ctx_len, void* out, float* lse, int32_t B, int32_t max_ctx_len,
                                 void* stream) {
  return decode_impl(c, q, q_row_stride, nullptr, nullptr, 0, const_cast<void*>(k_cache),
                     const_cast<void*>(v_cache), block_table, bt_stride, ctx_len, out, lse, B, max_ctx_len, stream);
}

int ecoserve_attn_decode_append(ecoserve_ctx* c, const void* q, int64_t q_row_stride, const void* k_new,
                                const void* v_new, int64_t new_row_stride, void* k_cache,
                                void* v_cache, const int32_t* block_table, int32_t bt_stride, const int32_t* ctx_len,
                                void* out, float* lse, int32_t B, int32_t max_ctx_len, void* stream) {
  if (!c || !stride_ok(c, new_row_stride, c->lay.num_kv_heads)) return ECOSERVE_EINVAL;
  if (B > 0 && (!k_new || !v_new || !aligned16(k_new) || !aligned16(v_new))) return ECOSERVE_EINVAL;
  return decode_impl(c, q, q_row_stride, k_new, v_new, new_row_stride, k_cache, v_cache, block_table,
                     bt_stride, ctx_len, out, lse, B, max_ctx_len, stream);
}

// Decode, with the step's append fused in if k_new is given.
static int decode_impl(ecoserve_ctx* c, const void* q, int64_t q_row_stride, const void* k_new, const void* v_new,
                       int64_t new_row_stride, void* k_cache, void* v_cache,
                       const int32_t* block_table, int32_t bt_stride, const int32_t* ctx_len, void* out, float* lse,
                       int32_t B, int32_t max_ctx_len, void* stream) {
  if (!c || B < 0 || max_ctx_len < 0) return ECOSERVE_EINVAL;
  if (!stride_ok(c, q_row_stride, c->lay.num_q_heads)) return ECOSERVE_EINVAL;
  if (B == 0) return ECOSERVE_OK;
  if (!q || !k_cache || !v_cache || !block_table || !ctx_len || !out) return ECOSERVE_EINVAL;
  if (B > c->max_batch || bt_stride <= 0 || max_ctx_len < 1) return ECOSERVE_EINVAL;
  if ((int64_t)max_ctx_len > (int64_t)c->max_blocks_per_seq * kBlockSize) return ECOSERVE_EINVAL;
  if ((int64_t)max_ctx_len > (int64_t)bt_stride * kBlockSize) return ECOSERVE_EINVAL;
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out)) return ECOSERVE_EINVAL;
  if (lse && (reinterpret_cast<uintptr_t>(lse) & 3u)) return ECOSERVE_EINVAL;
  if (B > 65535) return ECOSERVE_EINVAL;  // grid.z limit
  DeviceGuard guard(c->device);
  if (!guard.ok) return ECOSERVE_EHIP;
  hipStream_t s = (hipStream_t)stream;
  AttnArgs a = make_args(c, q, q_row_stride, k_cache, v_cache, block_table, bt_stride, out, lse, B);
  hipError_t e;
  if (k_new && !use_mfma(c)) {
    // the plain kernels do not fuse: the one-token append runs as its own kernel first (position = ctx_len - 1)
    ProfileScope prof(c, ECOSERVE_KERNEL_APPEND, s);
    e = launch_kv_append(c, k_cache, v_cache, k_new, v_new, (int32_t)new_row_stride, nullptr, ctx_len, block_table,
                         bt_stride, B, B, 1, -1, s);
    if (e != hipSuccess) return ECOSERVE_EHIP;
  }
  if (use_mfma(c)) {
    a.k_new = k_new;
    a.v_new = v_new;
    a.new_row_stride = (int32_t)new_row_stride;
    const int n_wgs = c->num_cu * kDecodeWgsPerCu;
    const bool adaptive = c->opt_adaptive && c->opt_split_tokens == 0 && n_wgs % 8 == 0;
    const float* const share_in = adaptive ? c->ws_share + 8 * c->share_parity : nullptr;
    float* const share_out = adaptive ? c->ws_share + 8 * (1 - c->share_parity) : nullptr;
    float* const speed = adaptive ? c->ws_share + 16 : nullptr;
    int32_t* const wave_samples = adaptive ? reinterpret_cast<int32_t*>(c->ws_share + 24) : nullptr;
    // the persistent grid lists its cut (sequence, head)s for the merge; a forced split has its own, larger grid
    int32_t* const cuts = c->opt_split_tokens == 0 ? reinterpret_cast<int32_t*>(c->ws_share + 24) + 2 * c->num_cu * kDecodeWgsPerCu * 4 : nullptr;
    if (adaptive) c->share_parity ^= 1;
    {
      ProfileScope prof(c, ECOSERVE_KERNEL_DECODE, s);
      e = launch_decode_mfma(a, ctx_len, c->opt_split_tokens, max_ctx_len, n_wgs, c->ws_acc, c->ws_ml, c->ws_meta,
                             c->ws_slots / (2 * (a.Hq / a.Hkv)), share_in, share_out, speed, wave_samples, cuts, s);
    }
    if (e != hipSuccess) return ECOSERVE_EHIP;
    e = launch_decode_mfma_merge(a, ctx_len, c->ws_acc, c->ws_ml, c->ws_meta, speed, wave_samples, cuts,
                                 n_wgs * 4, s);
    return e == hipSuccess ? ECOSERVE_OK : ECOSERVE_EHIP;
  }
  const int32_t split_tokens = plan_split_tokens(c, B, max_ctx_len);
  const int32_t n_split_max = ceil_div(max_ctx_len, split_tokens);
  if (n_split_max > c->ws_splits) return ECOSERVE_EINVAL;  // cannot happen for split_tokens >= kMinSplitTokens
  {
    ProfileScope prof(c, ECOSERVE_KERNEL_DECODE, s);
    e = launch_decode_plain(a, ctx_len, split_tokens, n_split_max, c->ws_acc, c->ws_ml, c->ws_splits, s);
  }
  if (e != hipSuccess) return ECOSERVE_EHIP;
  if (n_split_max > 1) {
    e = launch_decode_merge(a, ctx_len, split_tokens, c->ws_acc, c->ws_ml, c->ws_splits, s);
    if (e != hipSuccess) return ECOSERVE_EHIP;
  }
  return ECOSERVE_OK;
}

int ecoserve_debug_prefill_queue_shares(ecoserve_ctx* c, float* shares) {
  if (!c || !shares) return ECOSERVE_EINVAL;
  DeviceGuard guard(c->device);
  if (!guard.ok) return ECOSERVE_EHIP;
  if (hipDeviceSynchronize() != hipSuccess) return ECOSERVE_EHIP;
  // the last launch wrote the set of the parity it ran with; the context's parity has moved on since
  const int32_t* src = c->ws_plan + kPlanShare0 + kPlanMaxQueues * (c->plan_parity ^ 1);
  if (hipMemcpy(shares, src, kPlanMaxQueues * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess) return ECOSERVE_EHIP;
  for (int q = 0; q < kPlanMaxQueues; ++q)
    if (!(shares[q] > 0.f)) shares[q] = 1.f;  // nothing launched yet
  return ECOSERVE_OK;
}

int ecoserve_debug_validate(ecoserve_ctx* c, const int32_t* cu_q, const int32_t* ctx_total,
                            const int32_t* block_table, int32_t bt_stride, int32_t B) {
  if (!c || !ctx_total || !block_table || B < 0 || bt_stride <= 0) return ECOSERVE_EINVAL;
  if (B == 0) return ECOSERVE_OK;
  DeviceGuard guard(c->device);
  if (!guard.ok) return ECOSERVE_EHIP;
  std::vector<int32_t> cu, len((size_t)B), bt((size_t)B * bt_stride);
  if (hipDeviceSynchronize() != hipSuccess) return ECOSERVE_EHIP;
  if (cu_q) {
    cu.resize((size_t)B + 1);
    if (hipMemcpy(cu.data(), cu_q, cu.size() * 4, hipMemcpyDeviceToHost) != hipSuccess) return ECOSERVE_EHIP;
  }
  if (hipMemcpy(len.data(), ctx_total, len.size() * 4, hipMemcpyDeviceToHost) != hipSuccess) return ECOSERVE_EHIP;
  if (hipMemcpy(bt.data(), block_table, bt.size() * 4, hipMemcpyDeviceToHost) != hipSuccess) return ECOSERVE_EHIP;
  if (cu_q) {
    if (cu[0] != 0) return ECOSERVE_ECONTENT;
    for (int b = 0; b < B; ++b)
      if (cu[b + 1] < cu[b]) return ECOSERVE_ECONTENT;
  }
  std::vector<uint8_t> seen((size_t)c->lay.num_blocks, 0);
  for (int b = 0; b < B; ++b) {
    const int32_t L = len[b];
    if (L < (cu_q ? 0 : 1)) return ECOSERVE_ECONTENT;
    const int64_t nblk = ((int64_t)L + kBlockSize - 1) / kBlockSize;
    if (nblk > bt_stride) return ECOSERVE_ECONTENT;
    for (int64_t j = 0; j < nblk; ++j) {
      const int32_t p = bt[(size_t)b * bt_stride + j];
      if (p < 0 || p >= c->lay.num_blocks) return ECOSERVE_ECONTENT;
      if (seen[p]) return ECOSERVE_ECONTENT;
      seen[p] = 1;
    }
  }
  return ECOSERVE_OK;
}

int ecoserve_profile_reset(ecoserve_ctx* c) {
  if (!c) return ECOSERVE_EINVAL;
  DeviceGuard guard(c->device);
  if (!guard.ok || hipDeviceSynchronize() != hipSuccess) return ECOSERVE_EHIP;
  for (int i = 0; i < 3; ++i) c->ev_used[i] = 0, c->prof_seq[i] = 0;
  return ECOSERVE_OK;
}

int ecoserve_profile_read(ecoserve_ctx* c, int32_t kernel, double* ms_total, int64_t* launches) {
  if (!c || kernel < 0 || kernel > 2 || !ms_total || !launches) return ECOSERVE_EINVAL;
  DeviceGuard guard(c->device);
  if (!guard.ok || hipDeviceSynchronize() != hipSuccess) return ECOSERVE_EHIP;
  double sum = 0.0;
  for (size_t i = 0; i < c->ev_used[kernel]; ++i) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, c->ev[kernel][i].start, c->ev[kernel][i].stop) != hipSuccess) return ECOSERVE_EHIP;
    sum += ms;
  }
  *ms_total = sum;
  *launches = (int64_t)c->ev_used[kernel];
  return ECOSERVE_OK;
}

}  // extern "C"
