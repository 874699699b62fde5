// Causal variable-length prefill attention over the paged cache, bf16, head size 128,
// on gfx950 matrix cores.
//
// Eq. 2 of Section 2.1 for all new tokens of a prefill-only batch: the compute-bound
// phase of Table 2 (both attention products grow with S^2).  The new tokens' K/V are
// already in the paged cache; query i of sequence b sits at absolute position
// ctx_before[b] + i and sees keys 0..that position (a cached prefix is handled by the
// same loop).
//
// Work decomposition: one workgroup (4 wavefronts) = 128 query rows of one query head;
// each wavefront owns 32 rows.  Workgroup ids are laid out so that consecutive ids differ
// first in the K/V head (ids are dealt round-robin to the 8 XCDs, so with 8 K/V heads
// each XCD's L2 holds one head's K/V), then in the query head of the group, then in the
// query tile (heaviest, i.e. last, tile first), then in the sequence.
//
// Per 64-key step: the four 16-token cache blocks of K and of V are copied (global ->
// registers -> LDS, double buffered, one barrier per step) in 16-byte units.  The cache
// layouts were chosen so that no transposition is needed anywhere:
//   K block  [16 units][16 tokens][8 elems]  ->  LDS [unit][64 keys][16 B]:  A operand of
//            S^T = K Q^T   (v_mfma_f32_32x32x16_bf16, rows = keys, cols = query rows)
//   V block  [128 d][16 tokens]              ->  LDS [8-key octet][128 d][16 B]:  A operand
//            of O^T = V^T P^T (rows = d, cols = query rows)
// The rows of each S^T tile are assigned to keys with bits 2 and 3 swapped so that the
// accumulator registers a lane holds (rows 8*(i/4) + 4*half + i%4) are 8 consecutive keys,
// which is exactly the B-operand fragment of the second product: P stays in registers.
// Softmax is the online form per query row (= per accumulator column: in-lane over 32
// values, one cross-half shuffle), in the exp2 domain with the scale folded into one FMA.
//
// Lane layout relied upon for 32x32x16 (lane = 32*half + col):
//   A[row = col][k = 8*half .. +7],  B[k = 8*half .. +7][col],
//   C[row = 8*(i/4) + 4*half + i%4][col], i = 0..15.
#include "common.h"

namespace eco {

constexpr int kTQ = 128;                       // query rows per workgroup
constexpr int kTK = 64;                        // keys per step
constexpr int kKTileBytes = 16 * kTK * 16;     // [16 units][64 keys][16 B]
constexpr int kVOctStride = 128 * 16 + 64;     // one 8-key octet: [128 d][16 B] + bank-spreading pad
constexpr int kVTileBytes = 8 * kVOctStride;
constexpr int kBufBytes = kKTileBytes + kVTileBytes;

struct Stage {
  u32x4 k[4];
  u32x4 v[4];
};

__device__ __forceinline__ void load_tile(Stage& st, const char* __restrict__ k_cache,
                                          const char* __restrict__ v_cache, const int32_t* __restrict__ bt_row,
                                          int it, int nblk_total, int L_total, size_t head_off, size_t blk_stride,
                                          int tid) {
#pragma unroll
  for (int jb = 0; jb < 4; ++jb) {
    const int j = it * 4 + jb;
    if (j < nblk_total) {
      const size_t off = (size_t)__builtin_amdgcn_readfirstlane(bt_row[j]) * blk_stride + head_off + (size_t)tid * 16;
      st.k[jb] = *reinterpret_cast<const u32x4*>(k_cache + off);
      u32x4 v = *reinterpret_cast<const u32x4*>(v_cache + off);
      const int tail = L_total - (j << 4);  // valid slots in this block
      if (tail < 16) {
        // stale slots of the sequence's last block: zero them so that 0 * garbage cannot
        // reach the accumulator.  This thread's unit holds slots 8*(tid&1) .. +7.
        const int s0 = (tid & 1) * 8;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int lo_slot = s0 + 2 * e;
          uint32_t w = v[e];
          if (lo_slot >= tail) w &= 0xffff0000u;
          if (lo_slot + 1 >= tail) w &= 0x0000ffffu;
          v[e] = w;
        }
      }
      st.v[jb] = v;
    } else {
      st.k[jb] = u32x4{0, 0, 0, 0};
      st.v[jb] = u32x4{0, 0, 0, 0};
    }
  }
}

__device__ __forceinline__ void store_tile(const Stage& st, char* buf, int tid) {
#pragma unroll
  for (int jb = 0; jb < 4; ++jb) {
    // K: thread's unit is (unit c = tid/16, token = tid%16) of block jb
    *reinterpret_cast<u32x4*>(buf + (((tid >> 4) * kTK) + jb * 16 + (tid & 15)) * 16) = st.k[jb];
    // V: thread's unit is (d = tid/2, half = tid%2) -> octet 2*jb + half
    *reinterpret_cast<u32x4*>(buf + kKTileBytes + (2 * jb + (tid & 1)) * kVOctStride + (tid >> 1) * 16) = st.v[jb];
  }
}

__global__ __launch_bounds__(256, 2) void prefill_mfma_kernel(
    const uint16_t* __restrict__ q, const char* __restrict__ k_cache, const char* __restrict__ v_cache,
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ ctx_before,
    const int32_t* __restrict__ block_table, int bt_stride, uint16_t* __restrict__ out, float* __restrict__ lse,
    int B, int Hq, int Hkv, int G, int n_qt_max, float scale_log2e) {
  __shared__ __attribute__((aligned(16))) char smem[2 * kBufBytes];

  int wg = blockIdx.x;
  const int g = wg % Hkv;  wg /= Hkv;
  const int hg = wg % G;   wg /= G;
  const int qt_rev = wg % n_qt_max;
  const int b = wg / n_qt_max;
  const int tok0 = cu_q[b];
  const int S = cu_q[b + 1] - tok0;
  const int n_qt = (S + kTQ - 1) / kTQ;
  const int qt = n_qt - 1 - qt_rev;
  if (qt < 0) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int h = g * G + hg;
  const int cb = ctx_before[b];
  const int L_total = cb + S;
  const int nblk_total = (L_total + 15) >> 4;
  const int q0 = qt * kTQ;
  const int kv_end = cb + min(S, q0 + kTQ);            // keys [0, kv_end) are needed by this workgroup
  const int n_tiles = (kv_end + kTK - 1) / kTK;
  const int row = q0 + wave * 32 + col;                // this lane's query row inside the sequence
  const bool row_valid = row < S;
  const int pos = cb + row;                            // absolute position = causal bound
  const int w_pmin = cb + q0 + wave * 32;              // smallest / largest bound in this wavefront
  const int w_pmax = cb + min(S - 1, q0 + wave * 32 + 31);

  // B operand of S^T: Q^T[d][row]; step t covers d = 16 t .. 16 t + 15
  bf16x8 qf[8];
  {
    const uint16_t* qrow = q + ((size_t)(tok0 + row) * Hq + h) * 128 + half * 8;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
      qf[t] = row_valid ? *reinterpret_cast<const bf16x8*>(qrow + t * 16) : z;
    }
  }

  f32x16 o[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[dt][i] = 0.f;
  float m = -INFINITY, l = 0.f;  // running max of raw scores (unscaled), per-lane partial sum

  const int32_t* bt_row = block_table + (size_t)b * bt_stride;
  const size_t head_off = (size_t)g * 4096;
  const size_t blk_stride = (size_t)Hkv * 4096;
  // A-operand row -> key inside a 32-key tile: swap bits 2 and 3
  const int krow = (col & 0x13) | ((col & 4) << 1) | ((col & 8) >> 1);

  Stage st;
  load_tile(st, k_cache, v_cache, bt_row, 0, nblk_total, L_total, head_off, blk_stride, tid);
  store_tile(st, smem, tid);
  __syncthreads();

  for (int it = 0; it < n_tiles; ++it) {
    const char* buf = smem + (it & 1) * kBufBytes;
    if (it + 1 < n_tiles)
      load_tile(st, k_cache, v_cache, bt_row, it + 1, nblk_total, L_total, head_off, blk_stride, tid);

    const int k0 = it * kTK;
    if (k0 <= w_pmax) {  // uniform per wavefront: tiles wholly above the diagonal are skipped
      f32x16 s[2];
#pragma unroll
      for (int sti = 0; sti < 2; ++sti) {
#pragma unroll
        for (int i = 0; i < 16; ++i) s[sti][i] = 0.f;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          const bf16x8 a =
              *reinterpret_cast<const bf16x8*>(buf + (((2 * t + half) * kTK) + sti * 32 + krow) * 16);
          s[sti] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[t], s[sti], 0, 0, 0);
        }
      }
      if (k0 + kTK - 1 > w_pmin) {  // diagonal tile: apply the causal bound
#pragma unroll
        for (int sti = 0; sti < 2; ++sti)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int key = k0 + sti * 32 + (i >> 3) * 16 + half * 8 + (i & 7);
            if (key > pos) s[sti][i] = -INFINITY;
          }
      }
      float bm = s[0][0];
#pragma unroll
      for (int sti = 0; sti < 2; ++sti)
#pragma unroll
        for (int i = 0; i < 16; ++i) bm = fmaxf(bm, s[sti][i]);
      bm = fmaxf(bm, __shfl_xor(bm, 32));
      const float m_new = fmaxf(m, bm);
      const float mc = m_new * scale_log2e;
      const float alpha = exp2f(m * scale_log2e - mc);
      float psum = 0.f;
#pragma unroll
      for (int sti = 0; sti < 2; ++sti)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float p = exp2f(__builtin_fmaf(s[sti][i], scale_log2e, -mc));
          s[sti][i] = p;
          psum += p;
        }
      l = l * alpha + psum;
      if (__any(m_new != m)) {
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) o[dt] *= alpha;
      }
      m = m_new;
      // B operand of O^T: P^T[key][row]; step u covers keys 16 u .. 16 u + 15 of the tile
      bf16x8 pf[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int e = 0; e < 8; ++e) pf[u][e] = (__bf16)s[u >> 1][(u & 1) * 8 + e];
      const char* vbuf = buf + kKTileBytes;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(vbuf + (2 * u + half) * kVOctStride + (dt * 32 + col) * 16);
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[u], o[dt], 0, 0, 0);
        }
    }

    if (it + 1 < n_tiles) store_tile(st, smem + ((it + 1) & 1) * kBufBytes, tid);
    __syncthreads();
  }

  l += __shfl_xor(l, 32);
  if (row_valid) {
    const float inv = 1.f / l;
    uint16_t* orow = out + ((size_t)(tok0 + row) * Hq + h) * 128;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        // registers 4*i4 .. 4*i4+3 hold d = 32 dt + 8 i4 + 4 half + (0..3)
        u32x2 w;
        w[0] = (uint32_t)float_to_bf16_bits(o[dt][4 * i4 + 0] * inv) |
               ((uint32_t)float_to_bf16_bits(o[dt][4 * i4 + 1] * inv) << 16);
        w[1] = (uint32_t)float_to_bf16_bits(o[dt][4 * i4 + 2] * inv) |
               ((uint32_t)float_to_bf16_bits(o[dt][4 * i4 + 3] * inv) << 16);
        *reinterpret_cast<u32x2*>(orow + dt * 32 + i4 * 8 + half * 4) = w;
      }
    if (lse && half == 0) lse[(size_t)(tok0 + row) * Hq + h] = (m * scale_log2e + log2f(l)) * kLn2;
  }
}

hipError_t launch_prefill_mfma(const AttnArgs& a, const int32_t* cu_q, const int32_t* ctx_before, int32_t /*T*/,
                               int32_t max_q_len, hipStream_t s) {
  const int G = a.Hq / a.Hkv;
  const int n_qt_max = (max_q_len + kTQ - 1) / kTQ;
  const int64_t n_wg = (int64_t)a.B * n_qt_max * G * a.Hkv;
  if (n_wg <= 0) return hipSuccess;
  if (n_wg > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(prefill_mfma_kernel, dim3((unsigned)n_wg), dim3(256), 0, s, (const uint16_t*)a.q,
                     (const char*)a.k_cache, (const char*)a.v_cache, cu_q, ctx_before, a.block_table, a.bt_stride,
                     (uint16_t*)a.out, a.lse, a.B, a.Hq, a.Hkv, G, n_qt_max, a.scale_log2e);
  return hipGetLastError();
}

}  // namespace eco
