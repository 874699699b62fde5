// KV-cache append: scatter new K/V rows into the paged pools through the block table.
//
// Section 2.1 of the paper (key/value embeddings of processed tokens are saved and
// reused) and Section 5 (fixed-size cache blocks).  New token i of sequence b goes to
// absolute position p = ctx_before[b] + i: block block_table[b][p / 16], slot p % 16.
// Pure integer indexing and byte copies, so the result is bit-exact.
//
// Source rows are [T][Hkv][D]; destination is the library's block layout
//   K: [blk][Hkv][D/x][16 slots][x]   (x = elements per 16 bytes)
//   V: [blk][Hkv][D][16 slots]
// One thread moves one 16-byte unit of K (a single 16-byte store) and the same x
// elements of V (x element stores, 16 slots apart).
#include "common.h"

namespace eco {

// Index of the sequence that owns packed token t: largest b with cu_q[b] <= t.
__device__ __forceinline__ int find_sequence(const int32_t* __restrict__ cu_q, int B, int t) {
  int lo = 0, hi = B;  // invariant: cu_q[lo] <= t < cu_q[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu_q[mid] <= t) lo = mid; else hi = mid;
  }
  return lo;
}

template <typename E>
__global__ __launch_bounds__(256) void kv_append_kernel(E* __restrict__ k_cache, E* __restrict__ v_cache,
                                                        const E* __restrict__ k_new, const E* __restrict__ v_new,
                                                        const int32_t* __restrict__ cu_q,
                                                        const int32_t* __restrict__ ctx_before,
                                                        const int32_t* __restrict__ block_table, int bt_stride,
                                                        int B, int T, int Hkv, int D) {
  constexpr int X = Elem<E>::X;
  const int units_per_row = D / X;
  const int64_t total = (int64_t)T * Hkv * units_per_row;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int c = (int)(idx % units_per_row);
  const int g = (int)((idx / units_per_row) % Hkv);
  const int t = (int)(idx / ((int64_t)units_per_row * Hkv));
  const int b = find_sequence(cu_q, B, t);
  const int p = ctx_before[b] + (t - cu_q[b]);
  const int64_t blk = block_table[(size_t)b * bt_stride + (p >> 4)];
  const int slot = p & 15;

  const size_t src = ((size_t)t * Hkv + g) * D + (size_t)c * X;
  typedef uint32_t u4 __attribute__((ext_vector_type(4)));
  const u4 kval = *reinterpret_cast<const u4*>(k_new + src);
  *reinterpret_cast<u4*>(k_cache + k_index<X>(blk, g, slot, c * X, Hkv, D)) = kval;

  const u4 vraw = *reinterpret_cast<const u4*>(v_new + src);
  const E* ve = reinterpret_cast<const E*>(&vraw);
  E* vdst = v_cache + v_index(blk, g, slot, c * X, Hkv, D);
#pragma unroll
  for (int e = 0; e < X; ++e) vdst[(size_t)e * kBlockSize] = ve[e];
}

hipError_t launch_kv_append(const ecoserve_ctx* ctx, void* k_cache, void* v_cache, const void* k_new,
                            const void* v_new, const int32_t* cu_q, const int32_t* ctx_before,
                            const int32_t* block_table, int32_t bt_stride, int32_t B, int32_t T,
                            int32_t /*max_new_len*/, hipStream_t s) {
  const ecoserve_layout& L = ctx->lay;
  const int X = L.dtype == ECOSERVE_BF16 ? 8 : 4;
  const int64_t total = (int64_t)T * L.num_kv_heads * (L.head_dim / X);
  const unsigned grid = (unsigned)((total + 255) / 256);
  if (L.dtype == ECOSERVE_BF16) {
    hipLaunchKernelGGL(kv_append_kernel<uint16_t>, dim3(grid), dim3(256), 0, s, (uint16_t*)k_cache,
                       (uint16_t*)v_cache, (const uint16_t*)k_new, (const uint16_t*)v_new, cu_q, ctx_before,
                       block_table, bt_stride, B, T, L.num_kv_heads, L.head_dim);
  } else {
    hipLaunchKernelGGL(kv_append_kernel<float>, dim3(grid), dim3(256), 0, s, (float*)k_cache, (float*)v_cache,
                       (const float*)k_new, (const float*)v_new, cu_q, ctx_before, block_table, bt_stride, B, T,
                       L.num_kv_heads, L.head_dim);
  }
  return hipGetLastError();
}

}  // namespace eco
