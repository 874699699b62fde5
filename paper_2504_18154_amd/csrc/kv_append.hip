// KV-cache append: scatter new K/V rows into the paged pools through the block table.
//
// Section 2.1 of the paper (key/value embeddings of processed tokens are saved and
// reused) and Section 5 (fixed-size cache blocks).  New token i of sequence b goes to
// absolute position p = ctx_before[b] + i: block block_table[b][p / 16], slot p % 16.
// Pure integer indexing and byte copies, so the result is bit-exact.
//
// Source rows are [Hkv][D] per token, consecutive tokens `new_row_stride` elements apart (Hkv * D for a
// packed [T][Hkv][D] array, more when K and V sit inside a wider row such as a fused projection output,
// Eq. 1); destination is the library's block layout
//   K: [blk][Hkv][D/x][16 slots][x]   (x = elements per 16 bytes)
//   V: [blk][Hkv][D][16 slots]
// One workgroup fills one destination block for up to four adjacent K/V heads: up to 16 token
// rows in, per head one contiguous K piece and one contiguous V piece out (4 KiB each for
// bf16, D = 128).  Several heads per workgroup keep more loads in flight per thread and
// spread the cost of finding the block over more bytes.
// K units keep their 16 bytes and only change place, so they are copied directly with the
// writes running along the destination.  V needs a transposition (16 slots of one element
// become contiguous): the token rows are staged in LDS with coalesced reads and written
// back as 16-byte units along the destination.  Blocks that are only partly addressed
// (the first block of an append that continues a sequence, the last block) write only the
// addressed slots, element by element where a 16-byte unit is not completely new.
//
// The destination blocks of the whole batch are numbered sequence after sequence; the grid
// covers an upper bound on their number that the host can compute (T/16 + 2 per sequence),
// and every workgroup finds its (sequence, block) from a prefix sum over the batch.
// A call that brings at most one token per sequence (the decode step) takes a leaner kernel:
// one wavefront per (sequence, K/V head), no numbering, no staging.
#include "common.h"

namespace eco {

constexpr int kAppendThreads = 256;

// Exclusive prefix sums over the batch of the number of cache blocks each sequence's new
// tokens touch: pre[b] = blocks of sequences 0..b-1, pre[B] = all.  The batch description is
// kept beside them (tok[b] = cu_q[b], tok[B] = T; cbs[b] = ctx_before[b]) so that the
// workgroup does not go back to global memory for it.  Called by all threads.
__device__ __forceinline__ void scan_touched_blocks(int* pre, int* tok, int* cbs, int* wsum,
                                                    const int32_t* __restrict__ cu_q,
                                                    const int32_t* __restrict__ ctx_before, int B) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int per = (B + kAppendThreads - 1) / kAppendThreads;
  const int b0 = tid * per;
  auto touched = [&](int b) {
    const int S = cu_q[b + 1] - cu_q[b], cb = ctx_before[b];
    return S > 0 ? ((cb + S - 1) >> 4) - (cb >> 4) + 1 : 0;
  };
  int local = 0;
  for (int i = 0; i < per; ++i)
    if (b0 + i < B) {
      local += touched(b0 + i);
      tok[b0 + i] = cu_q[b0 + i];
      cbs[b0 + i] = ctx_before[b0 + i];
    }
  if (tid == 0) tok[B] = cu_q[B];
  int x = local;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int y = __shfl_up(x, o);
    if (lane >= o) x += y;
  }
  if (lane == 63) wsum[wave] = x;
  __syncthreads();
  int run = x - local;
  for (int w = 0; w < wave; ++w) run += wsum[w];
  for (int i = 0; i < per; ++i)
    if (b0 + i < B) {
      pre[b0 + i] = run;
      run += touched(b0 + i);
    }
  if (tid == 0) pre[B] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
  __syncthreads();
}

template <typename E, int HPW>
__global__ __launch_bounds__(kAppendThreads) void kv_append_kernel(E* __restrict__ k_cache, E* __restrict__ v_cache,
                                                                    const E* __restrict__ k_new,
                                                                    const E* __restrict__ v_new, int new_row_stride,
                                                                    const int32_t* __restrict__ cu_q,
                                                                    const int32_t* __restrict__ ctx_before,
                                                                    const int32_t* __restrict__ block_table,
                                                                    int bt_stride, int B, int Hkv, int D) {
  constexpr int X = Elem<E>::X;
  typedef uint32_t u4 __attribute__((ext_vector_type(4)));
  // Sized by the launch (append_lds_bytes): three arrays of B + 1 ints, then HPW staged V tiles of
  // 16 rows of D + X elements (padded rows).  A small batch leaves room for more workgroups per CU.
  extern __shared__ __attribute__((aligned(16))) int pre[];
  int* tok = pre + (B + 1);
  int* cbs = tok + (B + 1);
  const int vrow = D + X;
  E* vt = reinterpret_cast<E*>(pre + ((3 * (B + 1) + 3) & ~3));
  __shared__ int wsum[kAppendThreads / 64];
  scan_touched_blocks(pre, tok, cbs, wsum, cu_q, ctx_before, B);
  if ((int)blockIdx.x >= pre[B]) return;
  int lo_b = 0, hi_b = B;
  while (hi_b - lo_b > 1) {
    const int mid = (lo_b + hi_b) >> 1;
    if (pre[mid] <= (int)blockIdx.x) lo_b = mid; else hi_b = mid;
  }
  const int b = lo_b, first_unit = pre[b];
  const int unit = blockIdx.x;  // destination block number within the batch
  const int g0 = blockIdx.y * HPW, tid = threadIdx.x;
  const int tok0 = tok[b], S = tok[b + 1] - tok0, cb = cbs[b];
  const int j = (cb >> 4) + (unit - first_unit);      // logical block of the sequence
  const int lo = max(0, cb - (j << 4));               // addressed slots [lo, hi) of this block
  const int hi = min(16, cb + S - (j << 4));
  const int t_slot0 = tok0 + (j << 4) - cb;           // packed token index of slot 0 (may be < tok0)
  const int64_t blk = block_table[(size_t)b * bt_stride + j];
  const int upr = D / X;                              // 16-byte units per head row

  // The HPW heads of one token are adjacent in the source, so each pass below issues HPW
  // independent 16-byte loads per thread before the first use.
  // K: unit (c, slot) -> destination [c][slot][X]; threads run along the destination
  E* kdst = k_cache + ((size_t)blk * Hkv + g0) * 16 * D;
  for (int u = tid; u < 16 * upr; u += kAppendThreads) {
    const int slot = u & 15, c = u >> 4;
    if (slot >= lo && slot < hi) {
      const E* src = k_new + (size_t)(t_slot0 + slot) * new_row_stride + g0 * D + c * X;
      u4 val[HPW];
#pragma unroll
      for (int h = 0; h < HPW; ++h) val[h] = *reinterpret_cast<const u4*>(src + (size_t)h * D);
#pragma unroll
      for (int h = 0; h < HPW; ++h) *reinterpret_cast<u4*>(kdst + ((size_t)h * 16 * D) + (size_t)u * X) = val[h];
    }
  }
  // V: stage rows (threads run along the source rows) ...
  for (int u = tid; u < 16 * upr; u += kAppendThreads) {
    const int slot = u / upr, c = u % upr;
    if (slot >= lo && slot < hi) {
      const E* src = v_new + (size_t)(t_slot0 + slot) * new_row_stride + g0 * D + c * X;
      u4 val[HPW];
#pragma unroll
      for (int h = 0; h < HPW; ++h) val[h] = *reinterpret_cast<const u4*>(src + (size_t)h * D);
#pragma unroll
      for (int h = 0; h < HPW; ++h) *reinterpret_cast<u4*>(vt + ((size_t)h * 16 + slot) * vrow + c * X) = val[h];
    }
  }
  __syncthreads();
  // ... and write [d][16 slots] in 16-byte units of X slots (threads run along the destination)
  E* vdst = v_cache + ((size_t)blk * Hkv + g0) * D * 16;
  constexpr int kGroups = 16 / X;  // 16-byte units per element row
  for (int u = tid; u < HPW * D * kGroups; u += kAppendThreads) {
    const int h = u / (D * kGroups), r = u % (D * kGroups);
    const int d = r / kGroups, s0 = (r % kGroups) * X;
    const E* col = vt + (size_t)h * 16 * vrow + d;
    E* dst = vdst + ((size_t)h * D + d) * 16;
    if (s0 >= lo && s0 + X <= hi) {
      E tmp[X];
#pragma unroll
      for (int e = 0; e < X; ++e) tmp[e] = col[(s0 + e) * vrow];
      *reinterpret_cast<u4*>(dst + s0) = *reinterpret_cast<const u4*>(tmp);
    } else {
#pragma unroll
      for (int e = 0; e < X; ++e)
        if (s0 + e >= lo && s0 + e < hi) dst[s0 + e] = col[(s0 + e) * vrow];
    }
  }
}

// At most one new token per sequence (the decode step): one wavefront per (sequence, K/V head)
// copies the token's K row as 16-byte units and scatters its V row into the slot's column.
template <typename E>
__global__ __launch_bounds__(kAppendThreads) void kv_append_one_kernel(E* __restrict__ k_cache, E* __restrict__ v_cache,
                                                                        const E* __restrict__ k_new,
                                                                        const E* __restrict__ v_new, int new_row_stride,
                                                                        const int32_t* __restrict__ cu_q,
                                                                        const int32_t* __restrict__ ctx_before,
                                                                        const int32_t* __restrict__ block_table,
                                                                        int bt_stride, int B, int Hkv, int D,
                                                                        int pos_bias) {
  const int pair = blockIdx.x * (kAppendThreads / 64) + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (pair >= B * Hkv) return;
  const int b = pair / Hkv, g = pair % Hkv;
  // cu_q == NULL: exactly one token per sequence, token b belongs to sequence b
  const int tok = cu_q ? cu_q[b] : b;
  if (cu_q && cu_q[b + 1] - tok <= 0) return;
  const int p = ctx_before[b] + pos_bias;
  if (p < 0) return;  // (pos_bias -1 on an empty sequence: nothing to store)
  const int64_t blk = block_table[(size_t)b * bt_stride + (p >> 4)];
  append_one_row<E>(k_cache, v_cache, k_new + (size_t)tok * new_row_stride + g * D,
                    v_new + (size_t)tok * new_row_stride + g * D, blk, g, p & 15, Hkv, D, lane);
}

// Dynamic LDS of the tiled kernel: the batch tables, then HPW staged V tiles.
template <typename E>
static size_t append_lds_bytes(int B, int D, int hpw) {
  const size_t tables = (size_t)((3 * (B + 1) + 3) & ~3) * sizeof(int);
  return tables + (size_t)hpw * 16 * (D + Elem<E>::X) * sizeof(E);
}

template <typename E, int HPW>
static void launch_tiled(const ecoserve_layout& L, void* k_cache, void* v_cache, const void* k_new, const void* v_new,
                         int32_t new_row_stride, const int32_t* cu_q, const int32_t* ctx_before, const int32_t* block_table,
                         int32_t bt_stride, int32_t B, int32_t T, hipStream_t s) {
  // a sequence with S new tokens touches at most S/16 + 2 blocks (ragged at both ends), and none if S == 0
  const int64_t max_units = (int64_t)T / 16 + 2 * (int64_t)(B < T ? B : T);
  const dim3 grid((unsigned)max_units, (unsigned)(L.num_kv_heads / HPW));
  // (above 64 KiB - a batch of thousands - the kernel's limit was raised when the context was created)
  const size_t lds = append_lds_bytes<E>(B, L.head_dim, HPW);
  hipLaunchKernelGGL((kv_append_kernel<E, HPW>), grid, dim3(kAppendThreads), lds, s, (E*)k_cache, (E*)v_cache,
                     (const E*)k_new, (const E*)v_new, new_row_stride, cu_q, ctx_before, block_table, bt_stride, B,
                     L.num_kv_heads, L.head_dim);
}

template <typename E>
static void launch_typed(const ecoserve_layout& L, void* k_cache, void* v_cache, const void* k_new, const void* v_new,
                         int32_t new_row_stride, const int32_t* cu_q, const int32_t* ctx_before, const int32_t* block_table,
                         int32_t bt_stride, int32_t B, int32_t T, int32_t max_new_len, int32_t pos_bias,
                         hipStream_t s) {
  if (max_new_len <= 1) {
    const int per_wg = kAppendThreads / 64;
    const dim3 grid((unsigned)(((int64_t)B * L.num_kv_heads + per_wg - 1) / per_wg));
    hipLaunchKernelGGL((kv_append_one_kernel<E>), grid, dim3(kAppendThreads), 0, s, (E*)k_cache, (E*)v_cache,
                       (const E*)k_new, (const E*)v_new, new_row_stride, cu_q, ctx_before, block_table, bt_stride, B,
                       L.num_kv_heads, L.head_dim, pos_bias);
  } else if (L.num_kv_heads % 4 == 0) {
    launch_tiled<E, 4>(L, k_cache, v_cache, k_new, v_new, new_row_stride, cu_q, ctx_before, block_table, bt_stride, B, T, s);
  } else if (L.num_kv_heads % 2 == 0) {
    launch_tiled<E, 2>(L, k_cache, v_cache, k_new, v_new, new_row_stride, cu_q, ctx_before, block_table, bt_stride, B, T, s);
  } else {
    launch_tiled<E, 1>(L, k_cache, v_cache, k_new, v_new, new_row_stride, cu_q, ctx_before, block_table, bt_stride, B, T, s);
  }
}

template <typename E, int HPW>
static hipError_t raise_lds_limit(const ecoserve_ctx* ctx) {
  const size_t lds = append_lds_bytes<E>(ctx->max_batch, ctx->lay.head_dim, HPW);
  if (lds <= 60 * 1024) return hipSuccess;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&kv_append_kernel<E, HPW>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
}

hipError_t prepare_kv_append(const ecoserve_ctx* ctx) {
  const int hkv = ctx->lay.num_kv_heads;
  if (ctx->lay.dtype == ECOSERVE_BF16)
    return hkv % 4 == 0 ? raise_lds_limit<uint16_t, 4>(ctx) : hkv % 2 == 0 ? raise_lds_limit<uint16_t, 2>(ctx)
                                                                          : raise_lds_limit<uint16_t, 1>(ctx);
  return hkv % 4 == 0 ? raise_lds_limit<float, 4>(ctx) : hkv % 2 == 0 ? raise_lds_limit<float, 2>(ctx)
                                                                      : raise_lds_limit<float, 1>(ctx);
}

hipError_t launch_kv_append(const ecoserve_ctx* ctx, void* k_cache, void* v_cache, const void* k_new,
                            const void* v_new, int32_t new_row_stride, const int32_t* cu_q,
                            const int32_t* ctx_before, const int32_t* block_table, int32_t bt_stride, int32_t B,
                            int32_t T, int32_t max_new_len, int32_t pos_bias, hipStream_t s) {
  const ecoserve_layout& L = ctx->lay;
  if (L.dtype == ECOSERVE_BF16)
    launch_typed<uint16_t>(L, k_cache, v_cache, k_new, v_new, new_row_stride, cu_q, ctx_before, block_table, bt_stride, B, T,
                           max_new_len, pos_bias, s);
  else
    launch_typed<float>(L, k_cache, v_cache, k_new, v_new, new_row_stride, cu_q, ctx_before, block_table, bt_stride, B, T,
                        max_new_len, pos_bias, s);
  return hipGetLastError();
}

}  // namespace eco
