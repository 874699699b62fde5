// Plain (no matrix-core) attention kernels for any supported head size and element type,
// plus the split-context merge kernel that both decode paths share.
//
// They evaluate Eq. 2 of Section 2.1, softmax(Q K^T / sqrt(d_k)) V, over the paged cache
// with fp32 arithmetic and an online (running max / running sum) softmax in the exp2
// domain.  One wavefront handles one (query row, query head, context slice): lanes own
// tokens for the score pass and own head-vector elements for the value pass.  These
// kernels serve the fp32 configuration and odd head sizes; they are the correctness
// path, not the tuned one.
#include "common.h"

namespace eco {

constexpr int kMaxD = 256;

// Online-softmax attention of one query vector (already in LDS as fp32) over keys
// [t0, t1) of one sequence.  Result: running max m (exp2 domain), running sum l, and
// unnormalised output o[r] for d = lane + 64 r.
template <typename E>
__device__ __forceinline__ void plain_attend(const float* sq, float* sp, const E* __restrict__ k_cache,
                                             const E* __restrict__ v_cache, const int32_t* __restrict__ bt_row,
                                             int g, int Hkv, int D, int t0, int t1, float scale_log2e, float& m,
                                             float& l, float (&o)[kMaxD / 64]) {
  constexpr int X = Elem<E>::X;
  const int lane = threadIdx.x;
  m = -INFINITY;
  l = 0.f;
#pragma unroll
  for (int r = 0; r < kMaxD / 64; ++r) o[r] = 0.f;
  for (int base = t0; base < t1; base += 64) {
    const int tok = base + lane;
    const bool valid = tok < t1;
    float s = -INFINITY;
    if (valid) {
      const int64_t blk = bt_row[tok >> 4];
      const int slot = tok & 15;
      float acc = 0.f;
      for (int d = 0; d < D; ++d) acc += sq[d] * Elem<E>::load(k_cache + k_index<X>(blk, g, slot, d, Hkv, D));
      s = acc * scale_log2e;
    }
    const float m_new = fmaxf(m, wave_max(s));       // finite: the slice holds at least one valid token
    const float alpha = exp2f(m - m_new);            // 0 on the first tile (m = -inf)
    const float p = valid ? exp2f(s - m_new) : 0.f;
    l = l * alpha + wave_sum(p);
    m = m_new;
    sp[lane] = p;
    __syncthreads();
    const int n = min(64, t1 - base);
#pragma unroll
    for (int r = 0; r < kMaxD / 64; ++r) {
      const int d = lane + 64 * r;
      if (d < D) {
        float acc = o[r] * alpha;
        for (int j = 0; j < n; ++j) {
          const int tk = base + j;
          const int64_t blk = bt_row[tk >> 4];
          acc += sp[j] * Elem<E>::load(v_cache + v_index(blk, g, tk & 15, d, Hkv, D));
        }
        o[r] = acc;
      }
    }
    __syncthreads();
  }
}

template <typename E>
__device__ __forceinline__ void load_query(float* sq, const E* __restrict__ qrow, int D) {
  for (int d = threadIdx.x; d < D; d += 64) sq[d] = Elem<E>::load(qrow + d);
  __syncthreads();
}

__device__ __forceinline__ int find_seq(const int32_t* __restrict__ cu_q, int B, int t) {
  int lo = 0, hi = B;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu_q[mid] <= t) lo = mid; else hi = mid;
  }
  return lo;
}

// grid (T, Hq), 64 threads: query token t, head h; attends keys 0..ctx_before+i.
template <typename E>
__global__ __launch_bounds__(64) void prefill_plain_kernel(const E* __restrict__ q, int q_row_stride,
                                                           const E* __restrict__ k_cache,
                                                           const E* __restrict__ v_cache,
                                                           const int32_t* __restrict__ cu_q,
                                                           const int32_t* __restrict__ ctx_before,
                                                           const int32_t* __restrict__ block_table, int bt_stride,
                                                           E* __restrict__ out, float* __restrict__ lse, int B,
                                                           int Hq, int Hkv, int D, float scale_log2e) {
  __shared__ float sq[kMaxD];
  __shared__ float sp[64];
  const int t = blockIdx.x, h = blockIdx.y;
  const int b = find_seq(cu_q, B, t);
  const int p = ctx_before[b] + (t - cu_q[b]);
  const int g = h / (Hq / Hkv);
  load_query(sq, q + (size_t)t * q_row_stride + h * D, D);
  float m, l, o[kMaxD / 64];
  plain_attend<E>(sq, sp, k_cache, v_cache, block_table + (size_t)b * bt_stride, g, Hkv, D, 0, p + 1, scale_log2e,
                  m, l, o);
  const float inv = 1.f / l;
#pragma unroll
  for (int r = 0; r < kMaxD / 64; ++r) {
    const int d = threadIdx.x + 64 * r;
    if (d < D) Elem<E>::store(out + ((size_t)t * Hq + h) * D + d, o[r] * inv);
  }
  if (lse && threadIdx.x == 0) lse[(size_t)t * Hq + h] = (m + log2f(l)) * kLn2;
}

// grid (n_split_max, Hq, B), 64 threads: one context slice of one (sequence, head).
template <typename E>
__global__ __launch_bounds__(64) void decode_plain_kernel(const E* __restrict__ q, int q_row_stride,
                                                          const E* __restrict__ k_cache,
                                                          const E* __restrict__ v_cache,
                                                          const int32_t* __restrict__ block_table, int bt_stride,
                                                          const int32_t* __restrict__ ctx_len, E* __restrict__ out,
                                                          float* __restrict__ lse, float* __restrict__ ws_acc,
                                                          float* __restrict__ ws_ml, int ws_splits, int split_tokens,
                                                          int Hq, int Hkv, int D, float scale_log2e) {
  __shared__ float sq[kMaxD];
  __shared__ float sp[64];
  const int sp_idx = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int L = ctx_len[b];
  const int n_split = (L + split_tokens - 1) / split_tokens;
  if (sp_idx >= n_split) return;
  const int g = h / (Hq / Hkv);
  load_query(sq, q + (size_t)b * q_row_stride + h * D, D);
  const int t0 = sp_idx * split_tokens, t1 = min(L, t0 + split_tokens);
  float m, l, o[kMaxD / 64];
  plain_attend<E>(sq, sp, k_cache, v_cache, block_table + (size_t)b * bt_stride, g, Hkv, D, t0, t1, scale_log2e, m, l,
                  o);
  if (n_split == 1) {
    const float inv = 1.f / l;
#pragma unroll
    for (int r = 0; r < kMaxD / 64; ++r) {
      const int d = threadIdx.x + 64 * r;
      if (d < D) Elem<E>::store(out + ((size_t)b * Hq + h) * D + d, o[r] * inv);
    }
    if (lse && threadIdx.x == 0) lse[(size_t)b * Hq + h] = (m + log2f(l)) * kLn2;
  } else {
    const size_t slot = ((size_t)b * Hq + h) * ws_splits + sp_idx;
#pragma unroll
    for (int r = 0; r < kMaxD / 64; ++r) {
      const int d = threadIdx.x + 64 * r;
      if (d < D) ws_acc[slot * D + d] = o[r];
    }
    if (threadIdx.x == 0) {
      ws_ml[slot * 2 + 0] = m;
      ws_ml[slot * 2 + 1] = l;
    }
  }
}

// Merge of split-context partial softmax states (exact re-association of Eq. 2's
// normalisation): M = max_k m_k;  l = sum_k l_k 2^(m_k - M);  o = sum_k acc_k 2^(m_k - M) / l.
// grid (Hq, B), 64 threads; lanes own head-vector elements, the per-split weights are
// reduced across the wavefront with shuffles.
template <typename E>
__global__ __launch_bounds__(64) void decode_merge_kernel(const int32_t* __restrict__ ctx_len,
                                                          const float* __restrict__ ws_acc,
                                                          const float* __restrict__ ws_ml, int ws_splits,
                                                          int split_tokens, E* __restrict__ out,
                                                          float* __restrict__ lse, int Hq, int D) {
  const int h = blockIdx.x, b = blockIdx.y;
  const int L = ctx_len[b];
  const int n_split = (L + split_tokens - 1) / split_tokens;
  if (n_split <= 1) return;  // the partial kernel already wrote the final result
  const size_t base = ((size_t)b * Hq + h) * ws_splits;
  const int lane = threadIdx.x;
  // wavefront reduction of the running maxima and weighted sums (n_split may exceed 64)
  float mloc = -INFINITY;
  for (int k = lane; k < n_split; k += 64) mloc = fmaxf(mloc, ws_ml[(base + k) * 2]);
  const float M = wave_max(mloc);
  float lloc = 0.f;
  for (int k = lane; k < n_split; k += 64) lloc += ws_ml[(base + k) * 2 + 1] * exp2f(ws_ml[(base + k) * 2] - M);
  const float lsum = wave_sum(lloc);
  const float inv = 1.f / lsum;
  for (int d = lane; d < D; d += 64) {
    float acc = 0.f;
    for (int k = 0; k < n_split; ++k) acc += ws_acc[(base + k) * D + d] * exp2f(ws_ml[(base + k) * 2] - M);
    Elem<E>::store(out + ((size_t)b * Hq + h) * D + d, acc * inv);
  }
  if (lse && lane == 0) lse[(size_t)b * Hq + h] = (M + log2f(lsum)) * kLn2;
}

hipError_t launch_prefill_plain(const AttnArgs& a, const int32_t* cu_q, const int32_t* ctx_before, int32_t T,
                                hipStream_t s) {
  dim3 grid((unsigned)T, (unsigned)a.Hq);
  if (a.dtype == ECOSERVE_BF16) {
    hipLaunchKernelGGL(prefill_plain_kernel<uint16_t>, grid, dim3(64), 0, s, (const uint16_t*)a.q, a.q_row_stride,
                       (const uint16_t*)a.k_cache, (const uint16_t*)a.v_cache, cu_q, ctx_before, a.block_table,
                       a.bt_stride, (uint16_t*)a.out, a.lse, a.B, a.Hq, a.Hkv, a.D, a.scale_log2e);
  } else {
    hipLaunchKernelGGL(prefill_plain_kernel<float>, grid, dim3(64), 0, s, (const float*)a.q, a.q_row_stride,
                       (const float*)a.k_cache,
                       (const float*)a.v_cache, cu_q, ctx_before, a.block_table, a.bt_stride, (float*)a.out, a.lse,
                       a.B, a.Hq, a.Hkv, a.D, a.scale_log2e);
  }
  return hipGetLastError();
}

hipError_t launch_decode_plain(const AttnArgs& a, const int32_t* ctx_len, int32_t split_tokens, int32_t n_split_max,
                               float* ws_acc, float* ws_ml, int32_t ws_splits, hipStream_t s) {
  dim3 grid((unsigned)n_split_max, (unsigned)a.Hq, (unsigned)a.B);
  if (a.dtype == ECOSERVE_BF16) {
    hipLaunchKernelGGL(decode_plain_kernel<uint16_t>, grid, dim3(64), 0, s, (const uint16_t*)a.q, a.q_row_stride,
                       (const uint16_t*)a.k_cache, (const uint16_t*)a.v_cache, a.block_table, a.bt_stride, ctx_len,
                       (uint16_t*)a.out, a.lse, ws_acc, ws_ml, ws_splits, split_tokens, a.Hq, a.Hkv, a.D,
                       a.scale_log2e);
  } else {
    hipLaunchKernelGGL(decode_plain_kernel<float>, grid, dim3(64), 0, s, (const float*)a.q, a.q_row_stride,
                       (const float*)a.k_cache,
                       (const float*)a.v_cache, a.block_table, a.bt_stride, ctx_len, (float*)a.out, a.lse, ws_acc,
                       ws_ml, ws_splits, split_tokens, a.Hq, a.Hkv, a.D, a.scale_log2e);
  }
  return hipGetLastError();
}

hipError_t launch_decode_merge(const AttnArgs& a, const int32_t* ctx_len, int32_t split_tokens, const float* ws_acc,
                               const float* ws_ml, int32_t ws_splits, hipStream_t s) {
  dim3 grid((unsigned)a.Hq, (unsigned)a.B);
  if (a.dtype == ECOSERVE_BF16) {
    hipLaunchKernelGGL(decode_merge_kernel<uint16_t>, grid, dim3(64), 0, s, ctx_len, ws_acc, ws_ml, ws_splits,
                       split_tokens, (uint16_t*)a.out, a.lse, a.Hq, a.D);
  } else {
    hipLaunchKernelGGL(decode_merge_kernel<float>, grid, dim3(64), 0, s, ctx_len, ws_acc, ws_ml, ws_splits,
                       split_tokens, (float*)a.out, a.lse, a.Hq, a.D);
  }
  return hipGetLastError();
}

}  // namespace eco
