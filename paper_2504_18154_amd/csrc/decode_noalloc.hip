// Decode attention for callers that cannot allocate: ecoserve_attn_decode_noalloc.
//
// The same two launches as ecoserve_attn_decode on the matrix-core path (persistent split-context kernel,
// then the merge of the cut (sequence, head)s), without a context: the scratch memory those kernels need -
// the partial softmax states of cut pieces, the launch's numbering, each chunk's report to the merge - is a
// file-scope device array of fixed size instead of a workspace allocated by ecoserve_create.  The call makes
// no allocation of any kind (no hipMalloc / hipFree, no events, no library routine that allocates), so it can
// be used under graph capture, in serving loops and in harnesses that forbid allocation.
//
// Every GPU holds its own copy of the array at its own address; the address is looked up once per device
// (hipGetSymbolAddress with that device current) and kept.  All calls on one GPU share that GPU's array:
// calls that overlap on one GPU (two streams, two threads) race on it.  Nothing in the array has to start
// at zero: a launch writes every word it later reads (each wavefront writes its report, the merge reads only
// the states a report names).
#include <mutex>

#include "common.h"

namespace eco {
namespace {

constexpr int kNoallocMaxWgs = 256;                    // persistent grid: at most one workgroup per CU of an MI355X
constexpr int kNoallocMaxWaves = kNoallocMaxWgs * 4;
constexpr size_t kAccFloats = (size_t)2 * kNoallocMaxWaves * kMaxGroup * 128;  // two slot groups per wavefront
constexpr size_t kMlFloats = (size_t)2 * kNoallocMaxWaves * kMaxGroup * 2;
constexpr size_t kMetaInts = (kMaxBatch + 19 + 63) / 64 * 64;
constexpr size_t kCutInts = (size_t)4 * kNoallocMaxWaves;
constexpr size_t kScratchBytes = (kAccFloats + kMlFloats + kMetaInts + kCutInts) * 4;  // 16.3 MiB

// On the host this name is only a handle for hipGetSymbolAddress; device code and kernel arguments use the
// address looked up below.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
struct PerDevice {
  bool ready;
  void* scratch;  // device address of `scratch` on this GPU
  int num_cu;
};
PerDevice g_dev[kMaxDevices];
std::mutex g_mutex;

// First call on a device (that device current): the array's address there, and the CU count.
int setup_device(int device, PerDevice* out) {
  std::lock_guard<std::mutex> lock(g_mutex);
  PerDevice& d = g_dev[device];
  if (!d.ready) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
      (void)hipGetLastError();
      return ECOSERVE_EHIP;
    }
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus <= 0) {
      (void)hipGetLastError();
      return ECOSERVE_EHIP;
    }
    d.scratch = ptr;
    d.num_cu = cus;
    d.ready = true;
  }
  *out = d;
  return ECOSERVE_OK;
}

}  // namespace
}  // namespace eco

using namespace eco;

extern "C" int ecoserve_attn_decode_noalloc(int device, const ecoserve_layout* layout, const void* q,
                                            const void* k_cache, const void* v_cache, const int32_t* block_table,
                                            int32_t bt_stride, const int32_t* ctx_len, void* out, float* lse,
                                            int32_t B, int32_t max_ctx_len, void* stream) {
  int st;
  if (!layout_ok(layout, &st)) return st;
  if (layout->dtype != ECOSERVE_BF16 || layout->head_dim != 128) return ECOSERVE_EUNSUPPORTED;
  if (device < 0 || device >= kMaxDevices || B < 0 || max_ctx_len < 0) return ECOSERVE_EINVAL;
  if (B == 0) return ECOSERVE_OK;
  if (!q || !k_cache || !v_cache || !block_table || !ctx_len || !out) return ECOSERVE_EINVAL;
  // the limits the scratch array is sized for
  if (B > kMaxBatch) return ECOSERVE_EINVAL;
  if (bt_stride <= 0 || max_ctx_len < 1 || (int64_t)max_ctx_len > (int64_t)bt_stride * kBlockSize) return ECOSERVE_EINVAL;
  auto aligned16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out)) return ECOSERVE_EINVAL;
  if (lse && (reinterpret_cast<uintptr_t>(lse) & 3u)) return ECOSERVE_EINVAL;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess) { (void)hipGetLastError(); return ECOSERVE_EHIP; }
  if (device >= ndev) return ECOSERVE_EINVAL;
  DeviceGuard guard(device);
  if (!guard.ok) return ECOSERVE_EHIP;
  PerDevice dev;
  st = setup_device(device, &dev);
  if (st != ECOSERVE_OK) return st;

  float* const ws_acc = reinterpret_cast<float*>(dev.scratch);
  float* const ws_ml = ws_acc + kAccFloats;
  int32_t* const ws_meta = reinterpret_cast<int32_t*>(ws_ml + kMlFloats);
  int32_t* const ws_cut = ws_meta + kMetaInts;

  AttnArgs a;
  a.q = q;
  a.q_row_stride = layout->num_q_heads * layout->head_dim;
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
  a.Hq = layout->num_q_heads;
  a.Hkv = layout->num_kv_heads;
  a.D = layout->head_dim;
  a.dtype = layout->dtype;
  const float scale = layout->softmax_scale > 0.f ? layout->softmax_scale : 1.0f / sqrtf((float)layout->head_dim);
  a.scale_log2e = scale * kLog2e;

  const int n_wgs = dev.num_cu * kDecodeWgsPerCu < kNoallocMaxWgs ? dev.num_cu * kDecodeWgsPerCu : kNoallocMaxWgs;
  hipStream_t s = (hipStream_t)stream;
  // (a slot group holds G <= kMaxGroup states, so the array covers kNoallocMaxWaves wavefronts whatever G is)
  hipError_t e = launch_decode_mfma(a, ctx_len, 0, max_ctx_len, n_wgs, ws_acc, ws_ml, ws_meta, kNoallocMaxWaves,
                                    nullptr, nullptr, nullptr, nullptr, ws_cut, s);
  if (e != hipSuccess) return ECOSERVE_EHIP;
  e = launch_decode_mfma_merge(a, ctx_len, ws_acc, ws_ml, ws_meta, nullptr, nullptr, ws_cut, n_wgs * 4, s);
  return e == hipSuccess ? ECOSERVE_OK : ECOSERVE_EHIP;
}
