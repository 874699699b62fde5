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
// the query tile (heaviest, i.e. last, tile first), then in the sequence; only tiles that
// exist are launched (plus a few surplus workgroups that exit at once).
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
constexpr float kTau = 8.f;                    // lazy-rescale threshold, log2 units

typedef const void __attribute__((address_space(1)))* gptr_t;
typedef void __attribute__((address_space(3)))* lptr_t;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Physical block id for a tile's block index, clamped to the sequence's last block (keys
// past the end are beyond every causal bound; fix_tail() zeroes their values).
__device__ __forceinline__ int block_id(const int32_t* __restrict__ bt_row, int j, int nblk_total) {
  return bt_row[min(j, nblk_total - 1)];
}

// Issue the global->LDS copy of one 64-key K tile: this wavefront copies 16-byte units
// u = 4*wave .. 4*wave+3 of all four blocks; a 1 KiB LDS chunk is one unit of 64 keys, so
// lane l fetches (block l/16 [id in idk], token l%16).
__device__ __forceinline__ void stage_k(char* kbuf, const char* __restrict__ k_cache, int idk, size_t head_off,
                                        size_t blk_stride, int wave, int lane) {
  const char* ksrc = k_cache + (size_t)idk * blk_stride + head_off + (size_t)(lane & 15) * 16;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int u = 4 * wave + i;
    __builtin_amdgcn_global_load_lds((gptr_t)(ksrc + u * 256), (lptr_t)(kbuf + u * 1024), 16, 0, 0);
  }
}

// Same for a V tile: this wavefront copies block `wave` of the tile [id in idv]: octets
// 2*wave, 2*wave+1; a 1 KiB LDS chunk is 64 consecutive d of one octet, so lane l fetches
// unit (d = 64 hd + l, half).
__device__ __forceinline__ void stage_v(char* vbuf, const char* __restrict__ v_cache, int idv, size_t head_off,
                                        size_t blk_stride, int wave, int lane) {
  const char* vsrc = v_cache + (size_t)idv * blk_stride + head_off + (size_t)lane * 32;
#pragma unroll
  for (int hf = 0; hf < 2; ++hf)
#pragma unroll
    for (int hd = 0; hd < 2; ++hd)
      __builtin_amdgcn_global_load_lds((gptr_t)(vsrc + hd * 2048 + hf * 16),
                                       (lptr_t)(vbuf + (2 * wave + hf) * kVOctStride + hd * 1024), 16, 0, 0);
}

// Zero the V entries of keys >= first_bad of a V tile (slots past the end of the sequence
// may hold anything, and 0 * NaN must not reach the accumulator).
__device__ __forceinline__ void fix_tail(char* vbuf, int first_bad, int tid) {
  const int n = (kTK - first_bad) * 128;
  for (int idx = tid; idx < n; idx += 256) {
    const int key = first_bad + (idx >> 7), d = idx & 127;
    *reinterpret_cast<uint16_t*>(vbuf + (key >> 3) * kVOctStride + d * 16 + (key & 7) * 2) = 0;
  }
}

// v_max3_f32 as is (the C library's fmaxf also quiets signalling NaNs, one extra
// instruction per operand)
__device__ __forceinline__ float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// Causal mask (if the tile touches the diagonal) and row maximum of a 64-key S^T tile held
// as two 32-key accumulators; the maximum is combined across the two lane halves.
__device__ __forceinline__ float mask_and_max(f32x16 (&s)[2], int k0, int half, int pos, bool masked) {
  if (masked) {
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = k0 + sub * 32 + (i >> 3) * 16 + half * 8 + (i & 7);
        if (key > pos) s[sub][i] = -INFINITY;
      }
  }
  float bm = max3(s[0][0], s[0][1], s[0][2]);
#pragma unroll
  for (int i = 3; i < 15; i += 2) bm = max3(bm, s[0][i], s[0][i + 1]);
  bm = max3(bm, s[0][15], s[1][0]);
#pragma unroll
  for (int i = 1; i < 15; i += 2) bm = max3(bm, s[1][i], s[1][i + 1]);
  bm = fmaxf(bm, s[1][15]);
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(bm), __float_as_uint(bm), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Scores of one 32-key accumulator -> bf16 weights 2^(s c - mc) (two B-operand fragments of
// 8 keys each); the weights as rounded are added to this lane's share of the row sum.
__device__ __forceinline__ void exp_tile(const f32x16& s, bf16x8 (&pf)[2], float& l, float mc, float c) {
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
  float l0 = l, l1 = 0.f;
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
  l = l0 + l1;
}

__global__ __launch_bounds__(256, 2) void prefill_mfma_kernel(
    const uint16_t* __restrict__ q, const char* __restrict__ k_cache, const char* __restrict__ v_cache,
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ ctx_before,
    const int32_t* __restrict__ block_table, int bt_stride, uint16_t* __restrict__ out, float* __restrict__ lse,
    int B, int Hq, int Hkv, int G, float scale_log2e) {
  __shared__ __attribute__((aligned(16))) char smem[2 * kKTileBytes + 2 * kVTileBytes];
  static_assert((kMaxBatch + 1 + 4) * 4 <= 2 * kKTileBytes + 2 * kVTileBytes, "batch prefix sums must fit in the tile buffers");
  char* const kbufs = smem;
  char* const vbufs = smem + 2 * kKTileBytes;

  // Query tiles of the whole batch are numbered sequence after sequence, last (heaviest)
  // tile of a sequence first.  The grid covers an upper bound on their number that the host
  // can compute; every workgroup finds its (sequence, tile) from a prefix sum over the batch,
  // held in the LDS that the K/V buffers take over afterwards.
  int wg = blockIdx.x;
  const int g = wg % Hkv;  wg /= Hkv;
  const int hg = wg % G;   wg /= G;
  const int tile_id = wg;
  int b, qt;
  {
    int* pre = reinterpret_cast<int*>(smem);            // [B + 1]
    int* wsum = pre + kMaxBatch + 1;                    // [4]
    const int t = threadIdx.x, ln = t & 63, wv = t >> 6;
    const int per = (B + 255) / 256, b0 = t * per;
    int local = 0;
    for (int i = 0; i < per; ++i)
      if (b0 + i < B) local += (cu_q[b0 + i + 1] - cu_q[b0 + i] + kTQ - 1) / kTQ;
    int x = local;
#pragma unroll
    for (int o2 = 1; o2 < 64; o2 <<= 1) {
      const int y = __shfl_up(x, o2);
      if (ln >= o2) x += y;
    }
    if (ln == 63) wsum[wv] = x;
    __syncthreads();
    int run = x - local;
    for (int w = 0; w < wv; ++w) run += wsum[w];
    for (int i = 0; i < per; ++i)
      if (b0 + i < B) {
        pre[b0 + i] = run;
        run += (cu_q[b0 + i + 1] - cu_q[b0 + i] + kTQ - 1) / kTQ;
      }
    if (t == 0) pre[B] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
    __syncthreads();
    const bool live = tile_id < pre[B];
    int lo = 0, hi = B;
    while (live && hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (pre[mid] <= tile_id) lo = mid; else hi = mid;
    }
    b = lo;
    qt = live ? (pre[b + 1] - pre[b]) - 1 - (tile_id - pre[b]) : -1;
    __syncthreads();  // the prefix sums are dead: the same LDS now receives K/V tiles
  }
  if (qt < 0) return;
  const int tok0 = cu_q[b];
  const int S = cu_q[b + 1] - tok0;

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
  const int n_w = min(n_tiles, w_pmax / kTK + 1);      // tiles not wholly above this wavefront's diagonal
  const float c = scale_log2e;

  const int32_t* bt_row = block_table + (size_t)b * bt_stride;
  const size_t head_off = (size_t)g * 4096;
  const size_t blk_stride = (size_t)Hkv * 4096;
  const int kq = lane >> 4;  // which block of a tile this lane copies for K
  const int vq = tid >> 6;   // ... and for V (= wave, kept in a VGPR so that the id is fetched with a vector
                             // load: an outstanding scalar load would force full waits on every LDS read)

  stage_k(kbufs, k_cache, block_id(bt_row, kq, nblk_total), head_off, blk_stride, wave, lane);
  stage_v(vbufs, v_cache, __builtin_amdgcn_readfirstlane(block_id(bt_row, vq, nblk_total)), head_off, blk_stride,
          wave, lane);
  // K tile 1 goes out with tile 0 (both K buffers are free), which saves one memory round
  // trip in the prologue
  if (n_tiles > 1)
    stage_k(kbufs + kKTileBytes, k_cache, block_id(bt_row, 4 + kq, nblk_total), head_off, blk_stride, wave, lane);

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
  float m, l = 0.f;  // maximum used in the exponent (raw score units); this lane's share of the row sum

  // A-operand row -> key inside a 32-key tile: swap bits 2 and 3
  const int krow = (col & 0x13) | ((col & 4) << 1) | ((col & 8) >> 1);
  const int a_k_off = (half * kTK + krow) * 16;            // + (2 t * 64 + 32 sub) * 16
  const int a_v_off = half * kVOctStride + col * 16;       // + 2 u * stride + 32 dt * 16

  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (kTK > L_total) {  // the first tile already runs past the end of the sequence
    fix_tail(vbufs, L_total, tid);
    __syncthreads();
  }

  // ---- prologue: scores of tile 0 -----------------------------------------------------------
  int next_idk = block_id(bt_row, 8 + kq, nblk_total);     // K ids run two tiles ahead of the scores
  int next_idv = block_id(bt_row, 4 + vq, nblk_total);     // V ids one tile ahead
  f32x16 sa[2], sb[2];  // scores of the current / next tile, roles alternate
  {
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int i = 0; i < 16; ++i) sa[sub][i] = 0.f;
    const char* kb = kbufs + a_k_off;
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(kb + (2 * t * kTK + 32 * sub) * 16);
        sa[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[t], sa[sub], 0, 0, 0);
      }
    m = mask_and_max(sa, 0, half, pos, kTK - 1 > w_pmin);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  // ---- main loop: iteration j turns the scores of tile j into weights and accumulates
  // V(j) P(j), while the matrix cores already compute the scores of tile j+1 -----------------
  // One iteration; `sc` holds the (masked) scores of tile j on entry, `sn` receives those of
  // tile j+1.  The loop calls it with the two arrays swapped in turn, so no copy is needed.
  auto iteration = [&](int j, f32x16 (&sc)[2], f32x16 (&sn)[2]) {
    char* const kcur = kbufs + (j & 1) * kKTileBytes;          // held K(j), consumed: receives K(j+2)
    const char* const knext = kbufs + ((j + 1) & 1) * kKTileBytes;
    const char* const vcur = vbufs + (j & 1) * kVTileBytes;
    char* const vnext = vbufs + ((j + 1) & 1) * kVTileBytes;
#ifndef ECO_EXPERIMENT_NO_STAGE
    if (j + 2 < n_tiles) stage_k(kcur, k_cache, next_idk, head_off, blk_stride, wave, lane);
    if (j + 1 < n_tiles)
      stage_v(vnext, v_cache, __builtin_amdgcn_readfirstlane(next_idv), head_off, blk_stride, wave, lane);
#endif
    next_idk = block_id(bt_row, 4 * (j + 3) + kq, nblk_total);
    next_idv = block_id(bt_row, 4 * (j + 2) + vq, nblk_total);

    if (j < n_w) {  // uniform per wavefront
      const float mc = m * c;
      const char* kb = knext + a_k_off;
      const char* vb = vcur + a_v_off;
      bf16x8 pf0[2], pf1[2];
      const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
      float pv[2];
      // 32 matrix instructions per iteration, in this order:
      //   slots  0..15  scores of tile j+1: step t = slot/2, 32-key half = slot%2
      //   slots 16..23  O += V P, keys  0..31 of tile j: d tile = i%4, 16-key step = i/4
      //   slots 24..31  O += V P, keys 32..63
      // Consecutive slots write different accumulators (a dependent matrix instruction cannot
      // issue back to back).  Each slot is followed by the slice of softmax VALU work that
      // runs under it (one weight of keys 0..31 per slot in 0..15, two weights of keys 32..63
      // per slot in 16..23), and the LDS read of a slot's A fragment is issued kAhead slots
      // early.  The fences keep the compiler from regrouping the slots.
      constexpr int kAhead = 4;
      auto frag = [&](int slot) -> bf16x8 {
#ifdef ECO_EXPERIMENT_NO_LDS
        return qf[slot & 7];
#endif
        if (slot < 16) return *reinterpret_cast<const bf16x8*>(kb + (2 * (slot >> 1) * kTK + 32 * (slot & 1)) * 16);
        const int i = slot & 7;
        return *reinterpret_cast<const bf16x8*>(vb + (2 * (i >> 2) + (slot < 24 ? 0 : 4)) * kVOctStride +
                                                (i & 3) * 32 * 16);
      };
      // one weight: value e of accumulator s -> pv[e & 1]; every second one completes a pair
      auto weight = [&](const f32x16& s, bf16x8 (&pf)[2], int e) {
#ifdef ECO_EXPERIMENT_NO_SOFTMAX
        pv[e & 1] = s[e];
        if (e & 1) {
          const bf16x2 a = {(__bf16)pv[0], (__bf16)pv[1]};
          pf[e >> 3][(e & 7) - 1] = a[0];
          pf[e >> 3][(e & 7)] = a[1];
        }
        return;
#endif
        pv[e & 1] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[e], c, -mc));
        if (e & 1) {
          const bf16x2 a = {(__bf16)pv[0], (__bf16)pv[1]};
          l = __builtin_amdgcn_fdot2_f32_bf16(a, ones, l, false);
          pf[e >> 3][(e & 7) - 1] = a[0];
          pf[e >> 3][(e & 7)] = a[1];
        }
      };
      f32x16 zero;
#pragma unroll
      for (int i = 0; i < 16; ++i) zero[i] = 0.f;
      bf16x8 fr[2 * kAhead];
#pragma unroll
      for (int slot = 0; slot < kAhead; ++slot) fr[slot] = frag(slot);
#pragma unroll
      for (int slot = 0; slot < 32; ++slot) {
        if (slot + kAhead < 32) fr[(slot + kAhead) % (2 * kAhead)] = frag(slot + kAhead);
        const bf16x8 a = fr[slot % (2 * kAhead)];
        if (slot < 16) {
          sn[slot & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[slot >> 1], slot < 2 ? zero : sn[slot & 1], 0, 0, 0);
          weight(sc[0], pf0, slot);
        } else if (slot < 24) {
          const int i = slot - 16;
          o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf0[i >> 2], o[i & 3], 0, 0, 0);
          weight(sc[1], pf1, 2 * i);
          weight(sc[1], pf1, 2 * i + 1);
        } else {
          const int i = slot - 24;
          o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf1[i >> 2], o[i & 3], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      const int k0n = (j + 1) * kTK;
      const float bm = mask_and_max(sn, k0n, half, pos, k0n + kTK - 1 > w_pmin);
      if (__any((bm - m) * c > kTau)) {
        // the next tile's scores exceed the exponent offset by more than 2^kTau: raise it
        const float m_new = fmaxf(m, bm);
        const float alpha = __builtin_amdgcn_exp2f((m - m_new) * c);
        l *= alpha;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) o[dt] *= alpha;
        m = m_new;
      }
    }

#if defined(ECO_EXPERIMENT_NO_BARRIER) && defined(ECO_EXPERIMENT_NO_STAGE)
    return;
#endif
#ifndef ECO_EXPERIMENT_NO_WAIT
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#endif
    __syncthreads();
    if (j + 1 < n_tiles && (j + 2) * kTK > L_total) {  // the next V tile runs past the end of the sequence
      fix_tail(vnext, L_total - (j + 1) * kTK, tid);
      __syncthreads();
    }
  };
  for (int j = 0; j < n_tiles; j += 2) {
    iteration(j, sa, sb);
    if (j + 1 < n_tiles) iteration(j + 1, sb, sa);
  }

#ifdef ECO_EXPERIMENT_NO_WAIT
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#endif
  {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(l), __float_as_uint(l), false, false);
    l = __uint_as_float(r[0]) + __uint_as_float(r[1]);
  }
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
    if (lse && half == 0) lse[(size_t)(tok0 + row) * Hq + h] = (m * c + log2f(l)) * kLn2;
  }
}

hipError_t launch_prefill_mfma(const AttnArgs& a, const int32_t* cu_q, const int32_t* ctx_before, int32_t T,
                               int32_t /*max_q_len*/, hipStream_t s) {
  const int G = a.Hq / a.Hkv;
  // sum over sequences of ceil(S_b / kTQ) <= T / kTQ + (number of non-empty sequences)
  const int64_t max_tiles = (int64_t)T / kTQ + (a.B < T ? a.B : T);
  const int64_t n_wg = max_tiles * G * a.Hkv;
  if (n_wg <= 0) return hipSuccess;
  if (n_wg > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(prefill_mfma_kernel, dim3((unsigned)n_wg), dim3(256), 0, s, (const uint16_t*)a.q,
                     (const char*)a.k_cache, (const char*)a.v_cache, cu_q, ctx_before, a.block_table, a.bt_stride,
                     (uint16_t*)a.out, a.lse, a.B, a.Hq, a.Hkv, G, a.scale_log2e);
  return hipGetLastError();
}

}  // namespace eco
