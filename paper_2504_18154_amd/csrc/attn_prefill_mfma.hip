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
// each wavefront owns 32 rows; two workgroups share a CU so that one's softmax (VALU)
// runs under the other's matrix work.  Workgroup ids are laid out so that consecutive ids
// differ first in the K/V head (ids are dealt round-robin to the 8 XCDs, so with 8 K/V
// heads each XCD's L2 holds one head's K/V), then in the query head of the group, then in
// the query tile (heaviest, i.e. last, tile first), then in the sequence.
//
// Per 64-key step the four 16-token cache blocks of K and of V go straight from global
// memory into LDS (global_load ... lds, 16 bytes per lane, double buffered, one barrier per
// step); each lane picks the source address of the 16-byte unit that belongs at its LDS
// position, so the copy also performs the re-tiling.  The cache layouts were chosen so
// that no transposition is needed anywhere:
//   K block  [16 units][16 tokens][8 elems]  ->  LDS [unit][64 keys][16 B]:  A operand of
//            S^T = K Q^T   (v_mfma_f32_32x32x16_bf16, rows = keys, cols = query rows)
//   V block  [128 d][16 tokens]              ->  LDS [8-key octet][128 d][16 B]:  A operand
//            of O^T = V^T P^T (rows = d, cols = query rows)
// The rows of each S^T tile are assigned to keys with bits 2 and 3 swapped so that the
// accumulator registers a lane holds (rows 8*(i/4) + 4*half + i%4) are 8 consecutive keys,
// which is exactly the B-operand fragment of the second product: P stays in registers.
//
// Softmax is the online form per query row (= per accumulator column: in-lane over the
// lane's values, one v_permlane32_swap across the two halves), in the exp2 domain with the
// scale folded into one FMA.  The running maximum used in the exponent is only raised when
// a tile's maximum exceeds it by more than 2^8 (the accumulator and the row sum are then
// rescaled); weights can therefore reach 2^8, which bf16 and fp32 hold without loss of
// relative precision, and the rescale multiplications almost vanish from the loop.  The
// row sum is accumulated from the bf16-rounded weights with v_dot2_f32_bf16, so numerator
// and denominator see the same rounding.
//
// Lane layout relied upon for 32x32x16 (lane = 32*half + col):
//   A[row = col][k = 8*half .. +7],  B[k = 8*half .. +7][col],
//   C[row = 8*(i/4) + 4*half + i%4][col], i = 0..15.
#include "common.h"

namespace eco {

constexpr int kTQ = 128;                       // query rows per workgroup
constexpr int kTK = 64;                        // keys per step
constexpr int kKTileBytes = 16 * kTK * 16;     // [16 units][64 keys][16 B]
constexpr int kVOctStride = 128 * 16 + 64;     // one 8-key octet: [128 d][16 B] + pad
constexpr int kVTileBytes = 8 * kVOctStride;
constexpr int kBufBytes = kKTileBytes + kVTileBytes;
constexpr float kTau = 8.f;                    // lazy-rescale threshold, log2 units

typedef const void __attribute__((address_space(1)))* gptr_t;
typedef void __attribute__((address_space(3)))* lptr_t;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Physical block ids a lane needs to stage key tile `it`: idk for its K quarter (block
// lane/16 of the tile), idv for the V block its wavefront copies.  Blocks past the
// sequence's last one are replaced by the last one (their keys are beyond every causal
// bound; fix_tail() zeroes their values).
struct TileIds {
  int idk, idv;
};
__device__ __forceinline__ TileIds load_ids(const int32_t* __restrict__ bt_row, int it, int nblk_total, int wave,
                                            int lane) {
  const int last = nblk_total - 1;
  TileIds t;
  t.idk = bt_row[min(it * 4 + (lane >> 4), last)];
  t.idv = bt_row[min(it * 4 + wave, last)];
  return t;
}

// Issue the global->LDS copies of one key tile (64 keys).
__device__ __forceinline__ void stage_tile(char* buf, const char* __restrict__ k_cache,
                                           const char* __restrict__ v_cache, TileIds ids, size_t head_off,
                                           size_t blk_stride, int wave, int lane) {
  // K: this wavefront copies units u = 4*wave .. 4*wave+3 of all four blocks; a 1 KiB LDS
  // chunk is one unit of 64 keys, so lane l fetches (block l/16, token l%16)
  const char* ksrc = k_cache + (size_t)ids.idk * blk_stride + head_off + (size_t)(lane & 15) * 16;
  // V: this wavefront copies block `wave`: octets 2*wave, 2*wave+1; a 1 KiB LDS chunk is 64
  // consecutive d of one octet, so lane l fetches unit (d = 64 hd + l, half)
  const char* vsrc = v_cache + (size_t)ids.idv * blk_stride + head_off + (size_t)lane * 32;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int u = 4 * wave + i;
    __builtin_amdgcn_global_load_lds((gptr_t)(ksrc + u * 256), (lptr_t)(buf + u * 1024), 16, 0, 0);
  }
#pragma unroll
  for (int hf = 0; hf < 2; ++hf)
#pragma unroll
    for (int hd = 0; hd < 2; ++hd)
      __builtin_amdgcn_global_load_lds((gptr_t)(vsrc + hd * 2048 + hf * 16),
                                       (lptr_t)(buf + kKTileBytes + (2 * wave + hf) * kVOctStride + hd * 1024), 16,
                                       0, 0);
}

// Zero the V entries of keys >= first_bad of the tile in `buf` (slots past the end of the
// sequence may hold anything, and 0 * NaN must not reach the accumulator).
__device__ __forceinline__ void fix_tail(char* buf, int first_bad, int tid) {
  const int n = (kTK - first_bad) * 128;
  for (int idx = tid; idx < n; idx += 256) {
    const int key = first_bad + (idx >> 7), d = idx & 127;
    *reinterpret_cast<uint16_t*>(buf + kKTileBytes + (key >> 3) * kVOctStride + d * 16 + (key & 7) * 2) = 0;
  }
}

struct RowState {
  float m;  // maximum used in the exponent (raw score units); -inf before the first key
  float l;  // this lane's share of the row sum
};

// Online-softmax update for one 32-key S^T tile (16 accumulator values per lane): masks,
// raises the running maximum if needed (rescaling o and l), turns scores into bf16
// weights (two B-operand fragments of 8 keys each) and adds them to the row sum.
__device__ __forceinline__ void softmax_tile(f32x16& s, bf16x8 (&pf)[2], RowState& st, f32x16 (&o)[4], int key_base,
                                             int half, int pos, bool masked, float c) {
  if (masked) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int key = key_base + (i >> 3) * 16 + half * 8 + (i & 7);
      if (key > pos) s[i] = -INFINITY;
    }
  }
  float bm = fmaxf(s[0], s[1]);
#pragma unroll
  for (int i = 2; i < 16; i += 2) bm = fmaxf(bm, fmaxf(s[i], s[i + 1]));
  {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(bm), __float_as_uint(bm), false, false);
    bm = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
  }
  if (__any((bm - st.m) * c > kTau)) {
    const float m_new = fmaxf(st.m, bm);
    const float alpha = __builtin_amdgcn_exp2f((st.m - m_new) * c);
    st.l *= alpha;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) o[dt] *= alpha;
    st.m = m_new;
  }
  const float mc = st.m * c;
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
  float l0 = st.l, l1 = 0.f;
#pragma unroll
  for (int i = 0; i < 16; i += 4) {
    const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i + 0], c, -mc));
    const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i + 1], c, -mc));
    const float p2 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i + 2], c, -mc));
    const float p3 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i + 3], c, -mc));
    const bf16x2 a = {(__bf16)p0, (__bf16)p1};
    const bf16x2 b = {(__bf16)p2, (__bf16)p3};
    l0 = __builtin_amdgcn_fdot2_f32_bf16(a, ones, l0, false);
    l1 = __builtin_amdgcn_fdot2_f32_bf16(b, ones, l1, false);
    const int f = i >> 3, e = i & 7;
    pf[f][e + 0] = a[0];
    pf[f][e + 1] = a[1];
    pf[f][e + 2] = b[0];
    pf[f][e + 3] = b[1];
  }
  st.l = l0 + l1;
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

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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

  const int32_t* bt_row = block_table + (size_t)b * bt_stride;
  const size_t head_off = (size_t)g * 4096;
  const size_t blk_stride = (size_t)Hkv * 4096;

  stage_tile(smem, k_cache, v_cache, load_ids(bt_row, 0, nblk_total, wave, lane), head_off, blk_stride, wave, lane);
  TileIds next_ids = load_ids(bt_row, 1, nblk_total, wave, lane);  // ids run one tile ahead of the copies

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
  RowState st{-INFINITY, 0.f};

  // A-operand row -> key inside a 32-key tile: swap bits 2 and 3
  const int krow = (col & 0x13) | ((col & 4) << 1) | ((col & 8) >> 1);
  const int a_k_off = (half * kTK + krow) * 16;            // + (2 t * 64 + 32 sub) * 16
  const int a_v_off = half * kVOctStride + col * 16;       // + 2 u * stride + 32 dt * 16

  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (kTK > L_total) {  // the first tile already runs past the end of the sequence
    fix_tail(smem, L_total, tid);
    __syncthreads();
  }

  for (int it = 0; it < n_tiles; ++it) {
    const char* buf = smem + (it & 1) * kBufBytes;
    char* nbuf = smem + ((it + 1) & 1) * kBufBytes;
    if (it + 1 < n_tiles) {
      stage_tile(nbuf, k_cache, v_cache, next_ids, head_off, blk_stride, wave, lane);
      next_ids = load_ids(bt_row, it + 2, nblk_total, wave, lane);
    }

    const int k0 = it * kTK;
    if (k0 <= w_pmax) {  // uniform per wavefront: tiles wholly above the diagonal are skipped
      const bool masked = k0 + kTK - 1 > w_pmin;
      const bool second = k0 + 32 <= w_pmax;  // the second 32 keys are not wholly above the diagonal
      const char* kb = buf + a_k_off;
      const char* vb = buf + kKTileBytes + a_v_off;
      f32x16 s0, s1;
#pragma unroll
      for (int i = 0; i < 16; ++i) { s0[i] = 0.f; s1[i] = 0.f; }
      bf16x8 pf0[2], pf1[2];
      // keys 0..31: scores
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(kb + (2 * t * kTK) * 16);
        s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[t], s0, 0, 0, 0);
      }
      if (second) {
        // keys 32..63: scores, issued before the first half's softmax so the two overlap
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(kb + (2 * t * kTK + 32) * 16);
          s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[t], s1, 0, 0, 0);
        }
      }
      softmax_tile(s0, pf0, st, o, k0, half, pos, masked, scale_log2e);
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(vb + 2 * u * kVOctStride + dt * 32 * 16);
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf0[u], o[dt], 0, 0, 0);
        }
      if (second) {
        softmax_tile(s1, pf1, st, o, k0 + 32, half, pos, masked, scale_log2e);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(vb + (2 * u + 4) * kVOctStride + dt * 32 * 16);
            o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf1[u], o[dt], 0, 0, 0);
          }
      }
    }

    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (it + 1 < n_tiles && (it + 2) * kTK > L_total) {  // the next tile runs past the end of the sequence
      fix_tail(nbuf, L_total - (it + 1) * kTK, tid);
      __syncthreads();
    }
  }

  {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(st.l), __float_as_uint(st.l), false, false);
    st.l = __uint_as_float(r[0]) + __uint_as_float(r[1]);
  }
  if (row_valid) {
    const float inv = 1.f / st.l;
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
    if (lse && half == 0) lse[(size_t)(tok0 + row) * Hq + h] = (st.m * scale_log2e + log2f(st.l)) * kLn2;
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
