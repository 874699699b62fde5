// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "../../include/ecoserve.h"

namespace eco {

constexpr int kBlockSize = 16;        // tokens per cache block (the only supported value)
constexpr int kMaxGroup = 16;         // largest supported Hq / Hkv
constexpr int kMinSplitTokens = 64;   // smallest decode split
constexpr int kMaxSplitTokens = 4096; // largest forced decode split
constexpr int kDecodeWgsPerCu = 1;    // persistent decode grid: workgroups per CU (one wavefront per SIMD)
constexpr int kMaxBatch = 4096;       // largest max_batch a context accepts (batch prefix sums live in LDS)
constexpr int kPrefillTileRows = 128; // query rows of one prefill work item
constexpr int kPrefillWgsPerCu = 2;   // persistent prefill grid: workgroups per CU
constexpr int kPlanMaxQueues = 8;     // prefill plan: most work queues
constexpr int kPlanCounter0 = 32;     // prefill plan: first queue counter; each counter has a cache line of its own
constexpr int kPlanCounterStride = 32;
constexpr int kPlanShare0 = 8;        // prefill plan: two sets of 8 floats, the queues' shares of the items (0: none yet)
constexpr int kPlanMeta0 = 24;        // prefill plan: per set, the item count [24 + p] and the grid [26 + p] of the launch that wrote it
constexpr int kPlanMaxWgs = 1024;     // prefill plan: most workgroups whose busy times a launch records
constexpr int kPlanBusy0 = kPlanCounter0 + kPlanCounterStride * 2 * kPlanMaxQueues;  // two sets of kPlanMaxWgs busy times (10 ns units)
constexpr int kPlanHeaderInts = kPlanBusy0 + 2 * kPlanMaxWgs;  // two counter sets, the busy times, then the records
constexpr int kRecInts = 20;          // prefill plan: int32 fields per query-tile record
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct EventPair {
  hipEvent_t start, stop;
};

// Division of n < 2^31 by a fixed d >= 1 without a divide: q = (mulhi(n, magic) + n) >> shift with
// shift = ceil(log2 d), magic = floor(2^(32 + shift) / d) + 1 - 2^32 (round-up method; the sum
// cannot overflow because n < 2^31 and mulhi(n, magic) <= n).
struct Divisor {
  uint32_t magic, shift, d;
};
inline Divisor make_divisor(uint32_t d) {
  Divisor v;
  v.d = d;
  v.shift = 0;
  while ((1u << v.shift) < d) ++v.shift;
  v.magic = (uint32_t)((((uint64_t)1 << (32 + v.shift)) / d) + 1 - ((uint64_t)1 << 32));
  return v;
}

// Upper bound, computable on the host, on the number of query tiles of a prefill batch:
// sum over sequences of ceil(S_b / 128) <= T / 128 + (number of non-empty sequences).
inline int64_t prefill_plan_tiles(int32_t B, int32_t T) {
  return (int64_t)T / kPrefillTileRows + (B < T ? B : T);
}

// Makes `dev` the calling thread's current device for a scope, and puts the previous one back.
struct DeviceGuard {
  int prev;
  bool ok;
  explicit DeviceGuard(int dev) : prev(-1), ok(false) {
    if (hipGetDevice(&prev) != hipSuccess) return;
    ok = (prev == dev) || hipSetDevice(dev) == hipSuccess;
  }
  ~DeviceGuard() {
    int cur = -1;
    if (ok && hipGetDevice(&cur) == hipSuccess && cur != prev) (void)hipSetDevice(prev);
  }
};

}  // namespace eco

struct ecoserve_ctx {
  int device;
  ecoserve_layout lay;
  float scale;                 // resolved softmax scale
  int32_t max_batch;
  int32_t max_blocks_per_seq;
  int num_cu;
  // knobs
  int32_t opt_split_tokens;    // 0 = automatic
  int32_t opt_force_plain;
  int32_t opt_profile;         // 0 off, n: time every n-th hot call of each kind
  int32_t opt_adaptive;        // decode: per-XCD shares of the stream follow measured speeds
  int32_t opt_reuse_plan;      // prefill: calls that name the same batch arrays share one tile list
  // split-context workspace: unnormalised partial outputs and (max, sum) pairs, ws_slots slots of D floats
  // and of 2.  Matrix-core decode: two groups of G slots per wavefront of the launch; plain decode:
  // [max_batch][Hq][ws_splits].
  float* ws_acc;
  float* ws_ml;
  int64_t ws_slots;
  int32_t* ws_meta;            // [max_batch + 19]: chunk sizes and batch prefix sums of the last decode launch
  float* ws_share;             // per-XCD shares (mean 1) [2][8], speeds [8], then as int32 [2 * wavefronts]: units, ticks,
                               // then [4 * wavefronts]: the cut (sequence, K/V head) each chunk reports to the merge
  int share_parity;            // which of the two share vectors the next adaptive decode launch reads
  int32_t ws_splits;
  int32_t* ws_plan;            // prefill plan: header and one record per query tile of the last prefill launch
  int64_t plan_tiles;          // records ws_plan has room for
  int plan_parity;             // which of the plan's two sets of queue counters the next prefill launch takes
  struct {                     // the batch the tile list in ws_plan was made for (valid = false: none)
    bool valid;
    const int32_t *cu_q, *ctx_before, *block_table;
    int32_t bt_stride, B, T, n_wg;
  } plan_key;
  size_t ws_bytes;
  // profiling
  std::vector<eco::EventPair> ev[3];
  size_t ev_used[3];
  uint32_t prof_seq[3];        // hot calls of each kind since the last profile reset (every opt_profile-th is timed)
};

namespace eco {

// Arguments common to the attention launchers.
struct AttnArgs {
  const void* q;
  int32_t q_row_stride;  // elements between the query rows of consecutive tokens (>= Hq * D)
  const void* k_new;     // decode with the append fused in: the step's new K and V rows, else NULL
  const void* v_new;
  int32_t new_row_stride;
  const void* k_cache;
  const void* v_cache;
  const int32_t* block_table;
  int32_t bt_stride;
  void* out;
  float* lse;
  int32_t B;
  int32_t Hq, Hkv, D;
  int32_t dtype;
  float scale_log2e;  // softmax scale times log2(e): scores live in the exp2 domain
};

// api.hip: *status = ECOSERVE_OK and true, or the status that names what is wrong with the layout
bool layout_ok(const ecoserve_layout* L, int* status);

// kv_append.hip
// (at context creation: a batch of thousands needs more dynamic LDS than a kernel may use by default, and the
// limit is raised here, once, rather than by a hot call)
hipError_t prepare_kv_append(const ecoserve_ctx* ctx);
// (new_row_stride: elements between the K rows, and between the V rows, of consecutive tokens.  With
// max_new_len <= 1, cu_q may be NULL: one token per sequence, token b for sequence b, stored at position
// ctx_before[b] + pos_bias; otherwise pos_bias must be 0.)
hipError_t launch_kv_append(const ecoserve_ctx* ctx, void* k_cache, void* v_cache, const void* k_new,
                            const void* v_new, int32_t new_row_stride, const int32_t* cu_q, const int32_t* ctx_before,
                            const int32_t* block_table, int32_t bt_stride, int32_t B, int32_t T,
                            int32_t max_new_len, int32_t pos_bias, hipStream_t s);

// attn_plain.hip: any head size / dtype, no matrix cores
hipError_t launch_prefill_plain(const AttnArgs& a, const int32_t* cu_q, const int32_t* ctx_before, int32_t T,
                                hipStream_t s);
hipError_t launch_decode_plain(const AttnArgs& a, const int32_t* ctx_len, int32_t split_tokens, int32_t n_split_max,
                               float* ws_acc, float* ws_ml, int32_t ws_splits, hipStream_t s);
// merges split partials into out/lse (shared by the plain and matrix-core decode paths)
hipError_t launch_decode_merge(const AttnArgs& a, const int32_t* ctx_len, int32_t split_tokens, const float* ws_acc,
                               const float* ws_ml, int32_t ws_splits, hipStream_t s);

// attn_decode_mfma.hip: bf16, D = 128
// (split_tokens 0 = equal share per wavefront of the persistent grid; > 0 forces the chunk size)
// (share_in / share_out: per-XCD shares [8] read and left for the next launch; xcd_speed [8]: speeds the merge
// kernel measured from the per-wavefront samples ws_wave [2 * wavefronts]; share_in NULL: equal chunks)
// (partial states: two groups of G slots per wavefront of the launch, so ws_acc holds 2 * ws_waves * G * 128
// floats and ws_ml 2 * ws_waves * G * 2; decode_mfma_waves() says how many wavefronts a launch has; a launch
// that needs more than ws_waves is refused with hipErrorInvalidValue)
int64_t decode_mfma_waves(int32_t B, int32_t Hkv, int32_t max_ctx_len, int32_t split_tokens, int32_t n_persistent_wgs);
hipError_t launch_decode_mfma(const AttnArgs& a, const int32_t* ctx_len, int32_t split_tokens, int32_t max_ctx_len,
                              int32_t n_persistent_wgs, float* ws_acc, float* ws_ml, int32_t* ws_meta, int64_t ws_waves,
                              const float* share_in, float* share_out, const float* xcd_speed, int32_t* ws_wave,
                              int32_t* ws_cut, hipStream_t s);
// (with a.k_new given, the merge launch also stores every sequence's new token into the cache, position
// ctx_len[b] - 1: the decode kernel has taken it from the new rows and left the cache alone)
hipError_t launch_decode_mfma_merge(const AttnArgs& a, const int32_t* ctx_len, const float* ws_acc, const float* ws_ml,
                                    const int32_t* ws_meta, float* xcd_speed,
                                    const int32_t* ws_wave, const int32_t* ws_cut, int32_t n_waves, hipStream_t s);

// attn_prefill_mfma.hip: bf16, D = 128
// (ws_plan must hold kPlanHeaderInts + prefill_plan_tiles(B, T) * kRecInts int32; make_plan false: the tile list
// of an earlier launch for the same batch and grid is still in ws_plan; parity alternates from launch to launch)
int32_t prefill_mfma_grid(const AttnArgs& a, int32_t T, int32_t n_persistent_wgs);
hipError_t launch_prefill_mfma(const AttnArgs& a, const int32_t* cu_q, const int32_t* ctx_before, int32_t T,
                               int32_t max_q_len, int32_t* ws_plan, int32_t n_persistent_wgs, bool make_plan,
                               int parity, hipStream_t s);

}  // namespace eco

#if defined(__HIPCC__)
namespace eco {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ int fast_div(int n, const Divisor& v) {
  return (int)((__umulhi((uint32_t)n, v.magic) + (uint32_t)n) >> v.shift);
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even fp32 -> bf16 bit pattern (NaN kept quiet)
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Two fp32 values rounded to nearest even and packed as bf16 (low half first) with the hardware conversion
// of gfx950; the same bits as float_to_bf16_bits for every finite value.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const bf16x2_t v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, v);
}

template <typename E>
struct Elem;
template <>
struct Elem<uint16_t> {  // bf16 storage
  static constexpr int X = 8;  // elements per 16-byte unit
  static __device__ __forceinline__ float load(const uint16_t* p) { return bf16_bits_to_float(*p); }
  static __device__ __forceinline__ void store(uint16_t* p, float v) { *p = float_to_bf16_bits(v); }
};
template <>
struct Elem<float> {
  static constexpr int X = 4;
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};

// Element offsets inside the paged pools (see include/ecoserve.h, "Cache layout").
template <int X>
__device__ __forceinline__ size_t k_index(int64_t blk, int g, int slot, int d, int Hkv, int D) {
  return (((size_t)blk * Hkv + g) * (D / X) + (d / X)) * (kBlockSize * X) + (size_t)slot * X + (d % X);
}
__device__ __forceinline__ size_t v_index(int64_t blk, int g, int slot, int d, int Hkv, int D) {
  return (((size_t)blk * Hkv + g) * D + d) * kBlockSize + slot;
}

// One wavefront stores one new token of one (sequence, K/V head) into its cache slot: the K row as
// 16-byte units, the V row scattered into the slot's column.  `lane` 0..63.
template <typename E>
__device__ __forceinline__ void append_one_row(E* __restrict__ k_cache, E* __restrict__ v_cache,
                                               const E* __restrict__ ksrc, const E* __restrict__ vsrc, int64_t blk,
                                               int g, int slot, int Hkv, int D, int lane) {
  constexpr int X = Elem<E>::X;
  typedef uint32_t u4 __attribute__((ext_vector_type(4)));
  E* kdst = k_cache + ((size_t)blk * Hkv + g) * 16 * D + (size_t)slot * X;
  for (int c = lane; c < D / X; c += 64)
    *reinterpret_cast<u4*>(kdst + (size_t)c * 16 * X) = *reinterpret_cast<const u4*>(ksrc + c * X);
  E* vdst = v_cache + ((size_t)blk * Hkv + g) * D * 16 + slot;
  for (int d = lane; d < D; d += 64) vdst[(size_t)d * 16] = vsrc[d];
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

}  // namespace eco
#endif
