// Machine ceilings: what this GPU sustains on the two resources the paper's roofline
// argument (Section 2.1, Table 2) prices attention against -- bytes read from device memory
// (the decode phase) and bf16 matrix-core FLOPs (the prefill phase).  The published peaks are
// the denominators of every reported fraction; these two short measurements say how much of
// each peak any kernel could reach on the device at hand, so a reader can tell a kernel's
// loss from the machine's.  They allocate and synchronise: measurement helpers, not hot calls.
#include "common.h"

namespace eco {

typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kProbeThreads = 256;
constexpr int kProbePiece = 8192;  // bytes one wavefront reads at a time
constexpr int kMfmaChains = 4;     // independent accumulators per wavefront (hides the MFMA latency)
constexpr int kMfmaIters = 20000;  // per launch: 4 chains x 20000 MFMAs per wavefront, a few milliseconds

__device__ __forceinline__ uint32_t probe_hash(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

__global__ __launch_bounds__(kProbeThreads) void probe_fill_kernel(u4* __restrict__ dst, size_t n_vec) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += stride) {
    const uint32_t h = probe_hash((uint32_t)i);
    dst[i] = u4{h, h * 3u, h * 5u, h * 7u};
  }
}

// Every 8 KiB piece of the buffer is read once, by one wavefront, as eight coalesced 16-byte
// loads per lane with the non-temporal hint (the access shape of a paged K/V block as the decode
// kernel reads it; without the hint the same loop measures 10-12% lower on this device, and
// grid-stride streaming lower still).  Nothing is written unless the xor of all data hits one value.
__global__ __launch_bounds__(kProbeThreads) void probe_read_kernel(const u4* __restrict__ src, size_t n_pieces,
                                                                    u4* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  const size_t wave = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const size_t n_waves = ((size_t)gridDim.x * blockDim.x) >> 6;
  u4 acc = {0, 0, 0, 0};
  for (size_t c = wave; c < n_pieces; c += n_waves) {
    const u4* p = src + c * (kProbePiece / 16);
#pragma unroll
    for (int k = 0; k < kProbePiece / (64 * 16); ++k) acc ^= __builtin_nontemporal_load(&p[k * 64 + lane]);
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u && acc.x == 0x9e3779b9u) sink[lane] = acc;
}

// Register-only v_mfma_f32_32x32x16_bf16 loop.  With `random_operands` every chain multiplies
// its own pseudo-random fragments (values in [-2, 2)); otherwise all chains share one pair of
// smooth fragments.  The rates differ because the clock the chip holds under its power limit
// depends on how many operand bits toggle.
__global__ __launch_bounds__(kProbeThreads) void probe_mfma_kernel(float* __restrict__ sink, int iters,
                                                                    int random_operands) {
  bf16x8 a[kMfmaChains], b[kMfmaChains];
#pragma unroll
  for (int c = 0; c < kMfmaChains; ++c)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (random_operands) {
        const uint32_t h = probe_hash(threadIdx.x * 977u + blockIdx.x * 131u + c * 17u + i);
        a[c][i] = (__bf16)(((int)(h & 0xffff) - 32768) / 16384.0f);
        b[c][i] = (__bf16)(((int)(h >> 16) - 32768) / 16384.0f);
      } else {
        a[c][i] = (__bf16)(0.001f * (float)((threadIdx.x & 63) + i));
        b[c][i] = (__bf16)(0.002f * (float)(i + 1));
      }
    }
  f32x16 acc[kMfmaChains];
#pragma unroll
  for (int c = 0; c < kMfmaChains; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int c = 0; c < kMfmaChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c], b[c], acc[c], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kMfmaChains; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[c][i];
  if (s == 12345.678f) sink[threadIdx.x] = s;  // keeps the loop alive; practically never taken
}

// How much vector-ALU work the matrix cores hide: every wavefront runs `iters` rounds of four slots, a slot
// being one v_mfma_f32_32x32x16_bf16 (if kMfma; four accumulator chains in turn), kFma independent v_fma_f32
// and kExp independent v_exp_f32, in that order, with the compiler kept from regrouping them.  The online
// softmax of the prefill kernel is exactly such work beside its matrix instructions.  Each wavefront reports
// the shader clocks (s_memtime) and the 100 MHz ticks its loop took.
template <int kFma, int kExp, bool kMfma>
__global__ __launch_bounds__(kProbeThreads) void probe_slot_kernel(unsigned long long* __restrict__ clocks,
                                                                    float* __restrict__ sink, int iters) {
  bf16x8 a[kMfmaChains], b[kMfmaChains];
  f32x16 acc[kMfmaChains];
#pragma unroll
  for (int c = 0; c < kMfmaChains; ++c) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t h = probe_hash(threadIdx.x * 977u + blockIdx.x * 131u + c * 17u + i);
      a[c][i] = (__bf16)(((int)(h & 0xffff) - 32768) / 16384.0f);
      b[c][i] = (__bf16)(((int)(h >> 16) - 32768) / 16384.0f);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
  }
  float x[kFma > 0 ? kFma : 1] = {1.0f}, y[kExp > 0 ? kExp : 1] = {0.f};
  const float m1 = 0.999f + 1e-6f * (float)(threadIdx.x & 7), m2 = 1e-3f;
#pragma unroll
  for (int f = 0; f < kFma; ++f) x[f] = 1.0f + (float)f;
#pragma unroll
  for (int e = 0; e < kExp; ++e) y[e] = -0.5f - (float)e;
  const unsigned long long t0 = __builtin_readcyclecounter(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int c = 0; c < kMfmaChains; ++c) {
      if (kMfma) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c], b[c], acc[c], 0, 0, 0);
#pragma unroll
      for (int f = 0; f < kFma; ++f) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x[f]) : "v"(m1), "v"(m2));
#pragma unroll
      for (int e = 0; e < kExp; ++e) asm volatile("v_exp_f32 %0, %1" : "=v"(y[e]) : "v"(x[kFma > 0 ? e % kFma : 0]));
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  const unsigned long long t1 = __builtin_readcyclecounter(), w1 = wall_clock64();
  const size_t wave = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  if ((threadIdx.x & 63) == 0) {
    clocks[2 * wave] = t1 - t0;
    clocks[2 * wave + 1] = w1 - w0;
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kMfmaChains; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[c][i];
#pragma unroll
  for (int f = 0; f < kFma; ++f) s += x[f];
#pragma unroll
  for (int e = 0; e < kExp; ++e) s += y[e];
  if (s == 12345.678f) sink[threadIdx.x] = s;  // keeps the loop alive; practically never taken
}

struct ProbeTimer {
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipError_t init() {
    hipError_t e = hipEventCreate(&e0);
    return e != hipSuccess ? e : hipEventCreate(&e1);
  }
  ~ProbeTimer() {
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  }
};

// One untimed launch, then `reps` launches between two events on the null stream.
template <typename Launch>
static hipError_t time_launches(Launch launch, int reps, double* ms_per_launch) {
  ProbeTimer t;
  hipError_t e = t.init();
  if (e != hipSuccess) return e;
  launch();
  if ((e = hipDeviceSynchronize()) != hipSuccess) return e;
  if ((e = hipEventRecord(t.e0, nullptr)) != hipSuccess) return e;
  for (int r = 0; r < reps; ++r) launch();
  if ((e = hipEventRecord(t.e1, nullptr)) != hipSuccess) return e;
  if ((e = hipEventSynchronize(t.e1)) != hipSuccess) return e;
  if ((e = hipGetLastError()) != hipSuccess) return e;
  float ms = 0.f;
  if ((e = hipEventElapsedTime(&ms, t.e0, t.e1)) != hipSuccess) return e;
  *ms_per_launch = (double)ms / reps;
  return hipSuccess;
}

static int probe_num_cu(int device, int* num_cu) {
  int n = 0;
  if (hipGetDeviceCount(&n) != hipSuccess) {
    (void)hipGetLastError();
    return ECOSERVE_EHIP;
  }
  if (device < 0 || device >= n) return ECOSERVE_EINVAL;
  if (hipDeviceGetAttribute(num_cu, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || *num_cu <= 0)
    return ECOSERVE_EHIP;
  return ECOSERVE_OK;
}

}  // namespace eco

extern "C" {

int ecoserve_probe_hbm_read(int device, size_t bytes, int32_t reps, double* gb_per_s) {
  using namespace eco;
  if (!gb_per_s || reps <= 0 || reps > 1000 || bytes < (1u << 20) || bytes % kProbePiece != 0)
    return ECOSERVE_EINVAL;
  int num_cu = 0;
  if (int st = probe_num_cu(device, &num_cu)) return st;
  DeviceGuard guard(device);
  if (!guard.ok) return ECOSERVE_EHIP;
  u4 *buf = nullptr, *sink = nullptr;
  if (hipMalloc(&buf, bytes) != hipSuccess) {
    (void)hipGetLastError();
    return ECOSERVE_ENOMEM;
  }
  if (hipMalloc(&sink, 64 * sizeof(u4)) != hipSuccess) {
    (void)hipGetLastError();
    (void)hipFree(buf);
    return ECOSERVE_ENOMEM;
  }
  const size_t n_vec = bytes / 16;
  const dim3 grid((unsigned)(num_cu * 8)), block(kProbeThreads);
  hipLaunchKernelGGL(probe_fill_kernel, grid, block, 0, nullptr, buf, n_vec);
  // one wavefront per SIMD, as the decode kernel runs (more wavefronts read 3-6% slower with these loads)
  const dim3 read_grid((unsigned)num_cu);
  double ms = 0.0;
  const hipError_t e = time_launches(
      [&] { hipLaunchKernelGGL(probe_read_kernel, read_grid, block, 0, nullptr, buf, bytes / kProbePiece, sink); },
      reps, &ms);
  (void)hipFree(buf);
  (void)hipFree(sink);
  if (e != hipSuccess) return ECOSERVE_EHIP;
  *gb_per_s = (double)bytes / (ms * 1e-3) / 1e9;
  return ECOSERVE_OK;
}

int ecoserve_probe_mfma_bf16(int device, int32_t random_operands, int32_t reps, double* tflop_per_s) {
  using namespace eco;
  if (!tflop_per_s || reps <= 0 || reps > 1000) return ECOSERVE_EINVAL;
  int num_cu = 0;
  if (int st = probe_num_cu(device, &num_cu)) return st;
  DeviceGuard guard(device);
  if (!guard.ok) return ECOSERVE_EHIP;
  float* sink = nullptr;
  if (hipMalloc(&sink, kProbeThreads * sizeof(float)) != hipSuccess) {
    (void)hipGetLastError();
    return ECOSERVE_ENOMEM;
  }
  const int wgs = num_cu * 4;  // four workgroups of four wavefronts per CU: four wavefronts per SIMD
  double ms = 0.0;
  const hipError_t e = time_launches(
      [&] {
        hipLaunchKernelGGL(probe_mfma_kernel, dim3(wgs), dim3(kProbeThreads), 0, nullptr, sink, kMfmaIters,
                           random_operands ? 1 : 0);
      },
      reps, &ms);
  (void)hipFree(sink);
  if (e != hipSuccess) return ECOSERVE_EHIP;
  const double flops = 2.0 * 32 * 32 * 16 * (double)kMfmaChains * kMfmaIters * (kProbeThreads / 64) * wgs;
  *tflop_per_s = flops / (ms * 1e-3) / 1e12;
  return ECOSERVE_OK;
}

int ecoserve_probe_mfma_valu(int device, int32_t with_mfma, int32_t fma_per_slot, int32_t exp_per_slot,
                             int32_t waves_per_simd, double* clocks_per_slot, double* ghz) {
  using namespace eco;
  if (!clocks_per_slot || !ghz || waves_per_simd < 1 || waves_per_simd > 2) return ECOSERVE_EINVAL;
  typedef void (*Kernel)(unsigned long long*, float*, int);
  Kernel k = nullptr;
#define ECO_SLOT(F, E)                                                                              \
  if (fma_per_slot == F && exp_per_slot == E)                                                       \
    k = with_mfma ? (Kernel)probe_slot_kernel<F, E, true> : (Kernel)probe_slot_kernel<F, E, false>;
  ECO_SLOT(0, 0) ECO_SLOT(2, 0) ECO_SLOT(4, 0) ECO_SLOT(8, 0) ECO_SLOT(0, 2) ECO_SLOT(2, 2) ECO_SLOT(4, 2)
#undef ECO_SLOT
  if (!k || (!with_mfma && fma_per_slot == 0 && exp_per_slot == 0)) return ECOSERVE_EINVAL;
  int num_cu = 0;
  if (int st = probe_num_cu(device, &num_cu)) return st;
  DeviceGuard guard(device);
  if (!guard.ok) return ECOSERVE_EHIP;
  const int wgs = num_cu * waves_per_simd, n_waves = wgs * (kProbeThreads / 64), iters = 50000;  // several milliseconds: the clock settles
  unsigned long long* clocks = nullptr;
  float* sink = nullptr;
  if (hipMalloc(&clocks, (size_t)n_waves * 2 * sizeof(unsigned long long)) != hipSuccess ||
      hipMalloc(&sink, kProbeThreads * sizeof(float)) != hipSuccess) {
    (void)hipGetLastError();
    if (clocks) (void)hipFree(clocks);
    return ECOSERVE_ENOMEM;
  }
  std::vector<unsigned long long> host((size_t)n_waves * 2);
  hipError_t e = hipSuccess;
  for (int rep = 0; rep < 2 && e == hipSuccess; ++rep) {  // the second launch counts
    hipLaunchKernelGGL(k, dim3(wgs), dim3(kProbeThreads), 0, nullptr, clocks, sink, iters);
    e = hipDeviceSynchronize();
  }
  if (e == hipSuccess) e = hipMemcpy(host.data(), clocks, host.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost);
  (void)hipFree(clocks);
  (void)hipFree(sink);
  if (e != hipSuccess) { (void)hipGetLastError(); return ECOSERVE_EHIP; }
  double cyc = 0.0, ticks = 0.0;
  for (int w = 0; w < n_waves; ++w) cyc += (double)host[2 * w], ticks += (double)host[2 * w + 1];
  // clocks one SIMD spends per slot: a wavefront's clocks per slot, divided among the wavefronts that share it
  *clocks_per_slot = cyc / n_waves / ((double)iters * kMfmaChains) / waves_per_simd;
  *ghz = ticks > 0.0 ? cyc / ticks * 0.1 : 0.0;
  return ECOSERVE_OK;
}

}  // extern "C"
