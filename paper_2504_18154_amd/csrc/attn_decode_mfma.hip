// Split-context paged decode attention, bf16, head size 128, on gfx950 matrix cores.
//
// Eq. 2 of Section 2.1 for one new token per sequence against the whole cached context:
// the memory-bound phase of Table 2 (every cached K and V byte is read once per step,
// arithmetic intensity = the GQA group size).  The kernel is therefore organised around
// the HBM stream, and the matrix cores are used only so that arithmetic never gets in
// its way:
//
//   * grid (split, K/V head, sequence); a workgroup of 4 wavefronts owns one context
//     slice of one (sequence, K/V head) and serves all G query heads of the group from
//     one pass over the slice's K/V bytes;
//   * each wavefront streams whole 16-token cache blocks (4 KiB of K, 4 KiB of V) with
//     fully coalesced per-lane loads that land directly in MFMA operand layout - no LDS
//     staging, no barriers in the loop, next block prefetched into registers;
//   * scores S^T[token][head] = K . Q^T with v_mfma_f32_16x16x32_bf16 (heads padded to the
//     16 columns), online softmax per column in the exp2 domain, the 4x(16 lanes) partial
//     maxima combined with wavefront shuffles, and O^T[d][head] += V^T . P^T with
//     v_mfma_f32_16x16x16_bf16: the accumulator layout of the first product is already
//     the B-operand layout of the second, so P never leaves registers;
//   * the 4 wavefronts' states are merged through LDS; with one slice per sequence the
//     result is final, otherwise (m, l, unnormalised o) go to the workspace for the merge
//     kernel.
//
// Lane layouts relied upon (lane = 16*quad + col):
//   16x16x32:  A[row=col][k = 8*quad .. 8*quad+7],  B[k = 8*quad..+7][col],
//   16x16x16:  A[row=col][k = 4*quad .. 4*quad+3],  B[k = 4*quad..+3][col],
//   both:      C[row = 4*quad + i][col], i = 0..3.
#include "common.h"

namespace eco {

constexpr int kWaves = 4;

struct KVFrag {
  bf16x8 k[4];   // K block: unit (4*kk + quad, token = col)  ->  A operand of S^T step kk
  s16x4 v[8];    // V block: V^T[16*dt + col][tokens 4*quad..+3] ->  A operand of O^T tile dt
};

__device__ __forceinline__ void load_block(KVFrag& f, const char* __restrict__ kbase, const char* __restrict__ vbase,
                                           int lane, int col, int quad) {
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) f.k[kk] = *reinterpret_cast<const bf16x8*>(kbase + kk * 1024 + lane * 16);
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) f.v[dt] = *reinterpret_cast<const s16x4*>(vbase + dt * 512 + col * 32 + quad * 8);
}

__global__ __launch_bounds__(kWaves * 64) void decode_mfma_kernel(
    const uint16_t* __restrict__ q, const char* __restrict__ k_cache, const char* __restrict__ v_cache,
    const int32_t* __restrict__ block_table, int bt_stride, const int32_t* __restrict__ ctx_len,
    uint16_t* __restrict__ out, float* __restrict__ lse, float* __restrict__ ws_acc, float* __restrict__ ws_ml,
    int ws_splits, int blocks_per_split, int Hq, int Hkv, int G, float scale_log2e) {
  const int sp = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int L = ctx_len[b];
  const int nblk = (L + 15) >> 4;
  const int n_split = (nblk + blocks_per_split - 1) / blocks_per_split;
  if (sp >= n_split) return;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 15, quad = lane >> 4;

  // B operand of S^T: Q^T[d][head], heads beyond the group are zero columns
  bf16x8 qf[4];
  {
    const uint16_t* qrow = q + ((size_t)b * Hq + (size_t)g * G + col) * 128;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
      qf[kk] = col < G ? *reinterpret_cast<const bf16x8*>(qrow + kk * 32 + quad * 8) : z;
    }
  }

  const int blk_begin = sp * blocks_per_split;
  const int blk_end = min(nblk, blk_begin + blocks_per_split);
  const int32_t* bt_row = block_table + (size_t)b * bt_stride;
  const size_t head_off = (size_t)g * 4096;
  const size_t blk_stride = (size_t)Hkv * 4096;

  f32x4 acc[8];
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m = -INFINITY, l = 0.f;

  int j = blk_begin + wave;
  KVFrag cur;
  if (j < blk_end) {
    const size_t off = (size_t)__builtin_amdgcn_readfirstlane(bt_row[j]) * blk_stride + head_off;
    load_block(cur, k_cache + off, v_cache + off, lane, col, quad);
  }
  while (j < blk_end) {
    const int jn = j + kWaves;
    KVFrag nxt;
    if (jn < blk_end) {
      const size_t off = (size_t)__builtin_amdgcn_readfirstlane(bt_row[jn]) * blk_stride + head_off;
      load_block(nxt, k_cache + off, v_cache + off, lane, col, quad);
    }

    // S^T[token = 4*quad+i][head = col]
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur.k[kk], qf[kk], s, 0, 0, 0);
    s *= scale_log2e;
    if (j == nblk - 1) {
      // ragged tail of the sequence: slots >= L % 16 hold no token.  Their scores are
      // excluded, and their V entries zeroed so that stale bits (possibly NaN) times a
      // zero weight cannot reach the accumulator.
      const int tail = L - (j << 4);  // 1..16 valid slots
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (4 * quad + i >= tail) s[i] = -INFINITY;
#pragma unroll
      for (int dt = 0; dt < 8; ++dt)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (4 * quad + i >= tail) cur.v[dt][i] = 0;
    }
    float bm = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
    bm = fmaxf(bm, __shfl_xor(bm, 16));
    bm = fmaxf(bm, __shfl_xor(bm, 32));
    const float m_new = fmaxf(m, bm);  // finite: every block of the slice holds >= 1 token
    const float alpha = exp2f(m - m_new);
    f32x4 p;
#pragma unroll
    for (int i = 0; i < 4; ++i) p[i] = exp2f(s[i] - m_new);
    l = l * alpha + ((p[0] + p[1]) + (p[2] + p[3]));  // per-lane partial; quads are summed at the end
    if (__any(m_new != m)) {
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) acc[dt] *= alpha;
    }
    m = m_new;
    const bf16x4 pb = __builtin_convertvector(p, bf16x4);
    const s16x4 pbits = __builtin_bit_cast(s16x4, pb);
#pragma unroll
    for (int dt = 0; dt < 8; ++dt)
      acc[dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(cur.v[dt], pbits, acc[dt], 0, 0, 0);

    cur = nxt;
    j = jn;
  }

  // ---- merge the workgroup's wavefronts through LDS -------------------------------------
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  constexpr int kRow = 132;  // padded row of 128 floats
  __shared__ float sm_acc[kWaves][kMaxGroup][kRow];
  __shared__ float sm_m[kWaves][kMaxGroup];
  __shared__ float sm_l[kWaves][kMaxGroup];
  if (col < G) {
#pragma unroll
    for (int dt = 0; dt < 8; ++dt)
      *reinterpret_cast<f32x4*>(&sm_acc[wave][col][dt * 16 + 4 * quad]) = acc[dt];
    if (quad == 0) {
      sm_m[wave][col] = m;
      sm_l[wave][col] = l;
    }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < G * 128; idx += kWaves * 64) {
    const int hh = idx >> 7, d = idx & 127;
    float M = sm_m[0][hh];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) M = fmaxf(M, sm_m[w][hh]);
    float lsum = 0.f, o = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float wgt = exp2f(sm_m[w][hh] - M);  // a wavefront without blocks has m = -inf -> weight 0
      lsum += sm_l[w][hh] * wgt;
      o += sm_acc[w][hh][d] * wgt;
    }
    const int h = g * G + hh;
    if (n_split == 1) {
      out[((size_t)b * Hq + h) * 128 + d] = float_to_bf16_bits(o / lsum);
      if (lse && d == 0) lse[(size_t)b * Hq + h] = (M + log2f(lsum)) * kLn2;
    } else {
      const size_t slot = ((size_t)b * Hq + h) * ws_splits + sp;
      ws_acc[slot * 128 + d] = o;
      if (d == 0) {
        ws_ml[slot * 2 + 0] = M;
        ws_ml[slot * 2 + 1] = lsum;
      }
    }
  }
}

hipError_t launch_decode_mfma(const AttnArgs& a, const int32_t* ctx_len, int32_t split_tokens, int32_t n_split_max,
                              float* ws_acc, float* ws_ml, int32_t ws_splits, hipStream_t s) {
  dim3 grid((unsigned)n_split_max, (unsigned)a.Hkv, (unsigned)a.B);
  hipLaunchKernelGGL(decode_mfma_kernel, grid, dim3(kWaves * 64), 0, s, (const uint16_t*)a.q,
                     (const char*)a.k_cache, (const char*)a.v_cache, a.block_table, a.bt_stride, ctx_len,
                     (uint16_t*)a.out, a.lse, ws_acc, ws_ml, ws_splits, split_tokens / kBlockSize, a.Hq, a.Hkv,
                     a.Hq / a.Hkv, a.scale_log2e);
  return hipGetLastError();
}

}  // namespace eco
