// Causal variable-length prefill attention over the paged cache, bf16, head size 128,
// on gfx950 matrix cores.
//
// Eq. 2 of Section 2.1 for all new tokens of a prefill-only batch: the compute-bound
// phase of Table 2 (both attention products grow with S^2).  The new tokens' K/V are
// already in the paged cache; query i of sequence b sits at absolute position
// ctx_before[b] + i and sees keys 0..that position (a cached prefix is handled by the
// same loop).
//
// Work decomposition: one work item = 128 query rows (a query tile) of one query head,
// computed by one workgroup (4 wavefronts, 32 rows each).  A small plan kernel lists the
// batch's query tiles, heaviest (most key steps) first; the attention kernel is persistent:
// two workgroups per CU (one's softmax VALU work runs under the other's matrix work), each
// taking items from the list until it is empty.  While an item's last key step is being
// processed the workgroup already fetches the first K/V steps and the query rows of its next
// item, so a change of item costs no memory round trip: with the short prompts of a
// lognormal batch the start-up of a workgroup (tile lookup, block ids, first tiles, output
// write-back) would otherwise take a fifth of the kernel's time.  Consecutive items differ
// first in the K/V head, and a workgroup serves the items whose index is congruent to its
// XCD (workgroup ids are dealt round-robin to the 8 XCDs): with 8 K/V heads each XCD's L2
// holds one head's K/V.
// A prompt of at most 128 / G new tokens (G = query heads per K/V head) gets a packed tile
// instead: its rows are (query head of the group, position), so one item serves all G heads
// over the same K/V (see the plan kernel).
//
// Per 64-key step the four 16-token cache blocks of K and of V go straight from global
// memory into LDS (global_load ... lds, 16 bytes per lane, double buffered, one barrier per
// step, the eight copies of a wavefront issued one per slot under the step's first matrix
// instructions); each lane picks the source address of the 16-byte unit that belongs at its LDS
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
#include <type_traits>

#include "common.h"

namespace eco {

constexpr int kTQ = kPrefillTileRows;          // query rows per work item
constexpr int kTK = 64;                        // keys per step
constexpr int kKTileBytes = 16 * kTK * 16;     // [16 units][64 keys][16 B]
constexpr int kVOctStride = 128 * 16 + 64;     // one 8-key octet: [128 d][16 B] + pad
constexpr int kVTileBytes = 8 * kVOctStride;
constexpr float kTau = 8.f;                    // lazy-rescale threshold, log2 units
constexpr int kPlanThreads = 1024;
constexpr int kPlanBins = 4096;                // weight classes of the plan's counting sort
constexpr int kBalanceMinItems = 3072;          // batches with fewer items keep equal queues
constexpr float kShareGain = 2.5f, kShareMin = 0.5f, kShareMax = 1.5f;  // control of the queues' shares
constexpr int kQueues = 8;                     // work queues (a multiple of 8; more did not help)
static_assert(kQueues % 8 == 0 && kQueues <= kPlanMaxQueues, "queues come in multiples of the XCD count");

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

// One of the four copies of stage_k (I = 0..3), for callers that spread them out.  The instruction's immediate
// offset is added to the global address and to the LDS address alike, so with the LDS base moved back by the
// same amount the four copies share one address register pair.
template <int I>
__device__ __forceinline__ void stage_k_imm(char* kbuf, const char* ksrc_w, int wave) {
  __builtin_amdgcn_global_load_lds((gptr_t)ksrc_w, (lptr_t)(kbuf + wave * 4096 + I * (1024 - 256)), 16, I * 256, 0);
}
__device__ __forceinline__ void stage_k_one(char* kbuf, const char* ksrc_w, int wave, int i) {
  switch (i) {
    case 0: stage_k_imm<0>(kbuf, ksrc_w, wave); break;
    case 1: stage_k_imm<1>(kbuf, ksrc_w, wave); break;
    case 2: stage_k_imm<2>(kbuf, ksrc_w, wave); break;
    default: stage_k_imm<3>(kbuf, ksrc_w, wave); break;
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

// One of the four copies of stage_v (I = 0..3), with the immediate offset as in stage_k_imm.
template <int I>
__device__ __forceinline__ void stage_v_imm(char* vbuf, const char* vsrc, int wave) {
  constexpr int hf = I >> 1, hd = I & 1, imm = hd * 2048 + hf * 16;
  __builtin_amdgcn_global_load_lds((gptr_t)vsrc, (lptr_t)(vbuf + (2 * wave + hf) * kVOctStride + hd * 1024 - imm), 16, imm, 0);
}
__device__ __forceinline__ void stage_v_one(char* vbuf, const char* vsrc, int wave, int i) {
  switch (i) {
    case 0: stage_v_imm<0>(vbuf, vsrc, wave); break;
    case 1: stage_v_imm<1>(vbuf, vsrc, wave); break;
    case 2: stage_v_imm<2>(vbuf, vsrc, wave); break;
    default: stage_v_imm<3>(vbuf, vsrc, wave); break;
  }
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

// A row's keys are split between lane l and lane l ^ 32: the maximum over both.
__device__ __forceinline__ float across_halves(float bm) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(bm), __float_as_uint(bm), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Causal mask (if the tile touches the diagonal) and row maximum of a 64-key S^T tile held
// as two 32-key accumulators; the maximum is combined across the two lane halves.
__device__ __forceinline__ float mask_and_max(f32x16 (&s)[2], int k0, int half, int pos, bool masked) {
  if (masked) {
    // (an empty asm statement keeps this a real branch: turned into 32 unconditional selects it
    // would run on every step, and only the two steps at the diagonal of an item need it)
    asm volatile("" ::: "memory");
    // key index inside the step minus the lane-dependent part, against the bound moved the same
    // way: the comparisons take literal constants and one register
    const int bound = pos - k0 - half * 8;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (sub * 32 + (i >> 3) * 16 + (i & 7) > bound) s[sub][i] = -INFINITY;
  }
  float bm = max3(s[0][0], s[0][1], s[0][2]);
#pragma unroll
  for (int i = 3; i < 15; i += 2) bm = max3(bm, s[0][i], s[0][i + 1]);
  bm = max3(bm, s[0][15], s[1][0]);
#pragma unroll
  for (int i = 1; i < 15; i += 2) bm = max3(bm, s[1][i], s[1][i + 1]);
  bm = fmaxf(bm, s[1][15]);
  return across_halves(bm);
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

// ---- plan: the query tiles of a batch, heaviest first ------------------------------------------
//
// Plan layout (int32): [0] number of query tiles, [1] positions per packed tile and their reciprocal (0: no tile can be packed), [2] number of ordinary tiles (the packed ones follow them),
// [kPlanCounter0 + kPlanCounterStride * (kQueues * p
// + i)] ticket counter of work queue i in counter set p (one cache line each; launches alternate
// between the two sets and each launch leaves the other set ready for the next, so a tile list can
// serve many launches without being rebuilt), then from kPlanHeaderInts one record of kRecInts per
// query tile:
//   0 sequence, 1 tile inside the sequence, 2 first packed token of the sequence, 3 S,
//   4 ctx_before, 5 number of 64-key steps, 6 the tile's first query row, 7 the row behind its last,
//   8..19 physical ids of the sequence's first 12 blocks
// (clamped to its last block), i.e. everything a workgroup needs to start on the tile with one
// load.
// Where a prompt's tiles begin: a prompt of S = 128 n + r new tokens (0 < r < 128) has one ragged tile of r
// rows.  As the last tile it would cost as many key steps as a full one (its rows see the whole prompt);
// as the first tile it costs one or two.  Moving it to the front shifts the other tiles by r rows, which
// costs each of them ceil((ctx_before + r) / 64) - ceil(ctx_before / 64) steps more: without a cached
// prefix that is at most as many as the two steps saved per tile, and fewer when r <= 64.  tile_rows()
// takes whichever alignment has fewer key steps in total.  Records are sorted by the number of key steps, largest first, with a counting sort
// (tiles with kPlanBins - 1 or more steps share a class; the order inside a class is arbitrary).
__global__ __launch_bounds__(kPlanThreads) void prefill_plan_kernel(const int32_t* __restrict__ cu_q,
                                                                    const int32_t* __restrict__ ctx_before,
                                                                    const int32_t* __restrict__ block_table,
                                                                    int bt_stride, int B, int n_main_wgs,
                                                                    int max_tiles, int G, int32_t* __restrict__ plan) {
  __shared__ int pre[kMaxBatch + 1];
  __shared__ int bins[2 * kPlanBins];  // weight classes of the ordinary tiles, then of the packed ones
  __shared__ int wsum[kPlanThreads / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // exclusive prefix of one value per thread over the workgroup; `total` receives the sum
  auto block_scan = [&](int local, int& total) -> int {
    int x = local;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int y = __shfl_up(x, o);
      if (lane >= o) x += y;
    }
    if (lane == 63) wsum[wave] = x;
    __syncthreads();
    int run = x - local;
    total = 0;
    for (int w = 0; w < kPlanThreads / 64; ++w) {
      if (w < wave) run += wsum[w];
      total += wsum[w];
    }
    __syncthreads();
    return run;
  };
  auto tiles_of = [&](int b) { return (cu_q[b + 1] - cu_q[b] + kTQ - 1) / kTQ; };
  // rows [first, last) of tile qt of a prompt of S new tokens behind cb cached ones
  auto tile_rows = [&](int S, long long cb, int qt, int& first, int& last) {
    const int r = S % kTQ;
    const long long up = (cb + r + kTK - 1) / kTK - (cb + kTK - 1) / kTK;  // steps each full tile gains if shifted by r
    if (r > 0 && up < 2) {  // ragged tile first
      first = qt == 0 ? 0 : r + (qt - 1) * kTQ;
      last = qt == 0 ? r : first + kTQ;
    } else {
      first = qt * kTQ;
      last = min(S, first + kTQ);
    }
  };

  const int per = (B + kPlanThreads - 1) / kPlanThreads, b0 = tid * per;
  int local = 0;
  for (int i = 0; i < per; ++i)
    if (b0 + i < B) local += tiles_of(b0 + i);
  // Packed tiles: a prompt with at most P = kTQ / G new tokens fits a tile G times over, so its tile holds
  // all G query heads of a K/V head (row = head * P + position) and one item does what G items would, over
  // the same staged K/V: hundreds of 20-token prompts are otherwise one item per (prompt, query head) with a
  // sixth of its rows in use.  Packed tiles are listed behind the ordinary ones.
  const int P = G > 1 ? kTQ / G : 0;
  int n_tiles_all;
  int run = block_scan(local, n_tiles_all);
  // never more records than the host sized the launch (and the plan buffer) for, whatever cu_q says
  n_tiles_all = min(n_tiles_all, max_tiles);
  for (int i = 0; i < per; ++i)
    if (b0 + i < B) {
      pre[b0 + i] = run;
      run += tiles_of(b0 + i);
    }
  if (tid == 0) pre[B] = n_tiles_all;
  for (int i = tid; i < 2 * kPlanBins; i += kPlanThreads) bins[i] = 0;
  __syncthreads();

  // tile i of the batch (sequence after sequence) -> sequence, tile, key steps, weight class
  auto locate = [&](int i, int& b, int& qt, int& steps) -> int {
    int lo = 0, hi = B;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (pre[mid] <= i) lo = mid; else hi = mid;
    }
    b = lo;
    qt = i - pre[b];
    const int S = cu_q[b + 1] - cu_q[b];
    int first, last;
    tile_rows(S, ctx_before[b], qt, first, last);
    const long long kv_end = (long long)ctx_before[b] + last;
    steps = (int)((kv_end + kTK - 1) / kTK);
    const int cls = kPlanBins - 1 - min(steps, kPlanBins - 1);  // class 0 = heaviest
    return S <= P ? kPlanBins + cls : cls;
  };
  for (int i = tid; i < n_tiles_all; i += kPlanThreads) {
    int b, qt, steps;
    atomicAdd(&bins[locate(i, b, qt, steps)], 1);
  }
  __syncthreads();
  {
    constexpr int kPer = 2 * kPlanBins / kPlanThreads;
    int cnt[kPer], sum = 0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      cnt[i] = bins[tid * kPer + i];
      sum += cnt[i];
    }
    int total;
    int start = block_scan(sum, total);
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      bins[tid * kPer + i] = start;
      start += cnt[i];
    }
  }
  __syncthreads();
  if (tid == 0) {
    plan[1] = P ? (P | ((65536 / P + 1) << 8)) : 0;
    plan[2] = bins[kPlanBins];  // number of ordinary tiles = where the packed ones begin
  }
  __syncthreads();
  for (int i = tid; i < n_tiles_all; i += kPlanThreads) {
    int b, qt, steps;
    const int cls = locate(i, b, qt, steps);
    int32_t* rec = plan + kPlanHeaderInts + (size_t)atomicAdd(&bins[cls], 1) * kRecInts;
    const int cb = ctx_before[b], S = cu_q[b + 1] - cu_q[b];
    const int nblk_total = (int)(((long long)cb + S + 15) >> 4);
    rec[0] = b;
    rec[1] = qt;
    rec[2] = cu_q[b];
    rec[3] = S;
    rec[4] = cb;
    rec[5] = steps;
    tile_rows(S, cb, qt, rec[6], rec[7]);
    for (int j = 0; j < 12; ++j) rec[8 + j] = block_table[(size_t)b * bt_stride + min(j, nblk_total - 1)];
  }
  if (tid == 0) plan[0] = n_tiles_all;
  // each workgroup of the attention kernel owns the first two tickets of its queue outright
  if (tid < 2 * kQueues)
    plan[kPlanCounter0 + kPlanCounterStride * tid] = 2 * ((n_main_wgs - tid % kQueues + kQueues - 1) / kQueues);
}

// Wave-uniform description of one work item (a query tile of one query head).
constexpr int kPackedItem = 1 << 30;  // flag in the query head number handed to describe(): a packed tile
struct Item {
  int tok0, S, cb, q0, q_end, g, h, n_tiles;  // q0, q_end: the tile's query rows [q0, q_end) of the prompt's S
  bool pk;  // packed tile: rows are (query head h + row / P, position row % P)
  const int32_t* bt_row;
  __device__ __forceinline__ int L_total() const { return cb + S; }
  __device__ __forceinline__ int nblk_total() const { return (cb + S + 15) >> 4; }
};

// `rec` holds field l of the tile's plan record in lane l; g, h: the item's K/V and query head.
__device__ __forceinline__ Item describe(int rec, int g, int h, const int32_t* __restrict__ block_table,
                                         int bt_stride) {
  Item t;
  const int b = __builtin_amdgcn_readlane(rec, 0);
  t.tok0 = __builtin_amdgcn_readlane(rec, 2);
  t.S = __builtin_amdgcn_readlane(rec, 3);
  t.cb = __builtin_amdgcn_readlane(rec, 4);
  t.n_tiles = __builtin_amdgcn_readlane(rec, 5);
  t.g = g;
  t.h = h & (kPackedItem - 1);
  t.pk = (h & kPackedItem) != 0;
  t.q0 = __builtin_amdgcn_readlane(rec, 6);
  t.q_end = __builtin_amdgcn_readlane(rec, 7);
  t.bt_row = block_table + (size_t)b * bt_stride;
  return t;
}

template <bool kMayPack>
__global__ __launch_bounds__(256, 2) void prefill_mfma_kernel(
    const uint16_t* __restrict__ q, int q_row_stride, const char* __restrict__ k_cache,
    const char* __restrict__ v_cache, const int32_t* __restrict__ block_table, int bt_stride,
    uint16_t* __restrict__ out, float* __restrict__ lse, int32_t* __restrict__ plan, int parity, int Hq, int Hkv, int G, Divisor div_heads, Divisor div_hkv,
    float scale_log2e) {
  __shared__ __attribute__((aligned(16))) char smem[2 * kKTileBytes + 2 * kVTileBytes + 16 + 64];
  char* const kbufs = smem;
  char* const vbufs = smem + 2 * kKTileBytes;
  int* const slot = reinterpret_cast<int*>(smem + 2 * kKTileBytes + 2 * kVTileBytes);  // tickets from thread 0
  int* const qtab = slot + 4;  // [x]: items queue x works through, [8 + x]: items on its own list (wavefront 0 only)
  const long long t_begin = wall_clock64();

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31, half = lane >> 5;
  const int kq = lane >> 4;  // which block of a tile this lane copies for K
  const int vq = tid >> 6;   // ... and for V (= wave, kept in a VGPR so that the id is fetched with a vector
                             // load: an outstanding scalar load would force full waits on every LDS read)
  const float c = scale_log2e;
  const size_t blk_stride = (size_t)Hkv * 4096;
  // Packed tiles: P positions per tile (row = head * P + position) in the low byte, above it p_inv with
  // row / P == (row * p_inv) >> 16 for rows 0..127.  kMayPack false: every tile is taken as an ordinary one
  // and none of the packing code is compiled in (this kernel has no register to spare for it; the launcher
  // picks that variant for batches of long prompts); true: the tiles the plan lists as packed are.
  const int packing = kMayPack ? plan[1] : 0;
  const int heads = G * Hkv;  // items of an ordinary tile
  const int n_ord_tiles = packing ? plan[2] : plan[0];
  const int n_ordinary = n_ord_tiles * heads;  // items of the ordinary tiles; one per K/V head of the packed ones follow
  const int n_flat = n_ordinary + (plan[0] - n_ord_tiles) * Hkv;
  const int32_t* const recs = plan + kPlanHeaderInts;
  // Work items are dealt to kQueues queues (item f belongs to queue f % kQueues) and workgroup w
  // serves queue w % kQueues.  kQueues is a multiple of 8: workgroup ids are dealt round-robin to
  // the 8 XCDs and with eight K/V heads item f reads K/V head f % 8, so an XCD's L2 sees one head's
  // K/V.  The lists hold the same amount of work to within one item per weight class, and a
  // workgroup whose queue is empty is done.  Taking from other queues when one's own runs dry, or from
  // a pool shared by all, costs more than the imbalance it removes: atomics on one address are served
  // one after the other, and hundreds of workgroups asking the same counter at the same moment wait
  // tens of microseconds.  What does pay is decided before the first ticket: how many items each queue
  // works through (its quota, below), from the busy times of the launch before.
  const int queue = blockIdx.x % kQueues;
  int* const counter = plan + kPlanCounter0 + kPlanCounterStride * (kQueues * parity + queue);
  // the other counter set is idle (the launch that used it is over): start it for the next launch
  if (blockIdx.x == 0 && threadIdx.x < kQueues)
    plan[kPlanCounter0 + kPlanCounterStride * (kQueues * (parity ^ 1) + threadIdx.x)] =
        2 * (((int)gridDim.x - (int)threadIdx.x + kQueues - 1) / kQueues);
  auto resolve0 = [&](int k) -> int {  // ticket k of the own queue -> item of the own list, -1 past its end
    const int f = kQueues * k + queue;
    return f < n_flat ? f : -1;
  };
  // The same with the queues' quotas (qtab, set up below): a queue that gives items away stops short of the
  // end of its list, and the lists' ends so left over are dealt, in queue order, to the queues that take
  // more than their own.  Thread 0 only.
  auto resolve = [&](int k) -> int {
    const int quota = qtab[queue], own = qtab[kQueues + queue];
    if (k < min(quota, own)) return kQueues * k + queue;
    if (k >= quota) return -1;
    int p = k - own;  // index into the pool of left-over items
    for (int x = 0; x < queue; ++x) p += max(qtab[x] - qtab[kQueues + x], 0);
    for (int d = 0; d < kQueues; ++d) {
      const int cnt = qtab[kQueues + d] - qtab[d];
      if (cnt <= 0) continue;
      if (p < cnt) return kQueues * (qtab[d] + p) + d;
      p -= cnt;
    }
    return -1;
  };
  // What the previous launch left behind for this one (the other set): each workgroup's busy time, the
  // queues' shares and which batch they belong to.  Wavefront 0 asks for them now and uses them below.
  int prev_items = 0, prev_grid = 0;
  float busy_sum = 0.f, share = 0.f;  // (a float: 64 busy times of a long launch do not fit an int)
  if (wave == 0) {
    const int32_t* bp = plan + kPlanBusy0 + (parity ^ 1) * kPlanMaxWgs;
    for (int w = lane; w < (int)gridDim.x && w < kPlanMaxWgs; w += 64) busy_sum += (float)bp[w];
    share = reinterpret_cast<const float*>(plan)[kPlanShare0 + kQueues * (parity ^ 1) + (lane & 7)];
    prev_items = plan[kPlanMeta0 + (parity ^ 1)];
    prev_grid = plan[kPlanMeta0 + 2 + (parity ^ 1)];
  }
  // item f is query head f % (G Hkv) of tile f / (G Hkv), the K/V head varying fastest
  int tile_of_f, g_of_f, h_of_f;
  auto split = [&](int f) {
    if (kMayPack && f >= n_ordinary) {  // a packed tile: one item per K/V head, its G query heads share it
      const int fp = f - n_ordinary, t = fast_div(fp, div_hkv);
      tile_of_f = n_ord_tiles + t;
      g_of_f = fp - t * Hkv;
      h_of_f = (g_of_f * G) | kPackedItem;
      return;
    }
    tile_of_f = fast_div(f, div_heads);
    const int hp = f - tile_of_f * heads;
    const int hg = fast_div(hp, div_hkv);
    g_of_f = hp - hg * Hkv;
    h_of_f = g_of_f * G + hg;
  };
  auto load_rec = [&](int tile) { return recs[(size_t)tile * kRecInts + min(lane, kRecInts - 1)]; };

  // The first two tickets of every workgroup are fixed (the plan starts the counters behind them):
  // several hundred workgroups asking eight counters at once would wait on each other.
  if (tid == 0) {
    const int iq = blockIdx.x / kQueues;                                   // index in the queue's crew
    const int nq = ((int)gridDim.x - queue + kQueues - 1) / kQueues;       // size of the crew
    const int f0 = resolve0(iq);  // (a queue's quota is never below these two rounds)
    slot[0] = f0;
    slot[1] = f0 >= 0 ? resolve0(iq + nq) : -1;
  }
  __syncthreads();
  int f_cur = __builtin_amdgcn_readfirstlane(slot[0]);    // the item being computed
  int f_next = __builtin_amdgcn_readfirstlane(slot[1]);   // the one after it (-1: none)
  if (f_cur < 0) {
    if (tid == 0 && blockIdx.x < kPlanMaxWgs) plan[kPlanBusy0 + parity * kPlanMaxWgs + blockIdx.x] = 0;
    return;
  }

  split(f_cur);
  int rec_next = load_rec(tile_of_f);  // record of the next item (here: of the first)
  int pend = 0;                        // (thread 0) ticket on its way
  Item cur = describe(rec_next, g_of_f, h_of_f, block_table, bt_stride);
  int g_next = 0, h_next = 0;                    // heads of the next item

  // per-lane view of the current item
  int pos, w_pmin, n_w;
  size_t head_off;
  // tile row -> (query row inside the sequence, query head inside the group, row in use)
  auto map_row = [&](const Item& t, int& r, int& hq, bool& ok) {
    const int rr = wave * 32 + col;
    if (kMayPack && t.pk) {
      hq = (rr * (packing >> 8)) >> 16;
      r = rr - hq * (packing & 255);
      ok = hq < G && r < t.S;
    } else {
      hq = 0;
      r = t.q0 + rr;
      ok = r < t.q_end;
    }
  };
  auto enter = [&](const Item& t) {
    int row, hsel;
    bool row_valid;
    map_row(t, row, hsel, row_valid);
    pos = t.cb + row;                                      // absolute position = causal bound
    // smallest / largest bound in this wavefront (packed: of the tile, every wavefront sees every position)
    w_pmin = kMayPack && t.pk ? t.cb : t.cb + t.q0 + wave * 32;
    const int w_pmax = kMayPack && t.pk ? t.cb + t.S - 1 : t.cb + min(t.q_end - 1, t.q0 + wave * 32 + 31);
    // steps not wholly above this wavefront's diagonal; a wavefront none of whose rows exists (the ragged
    // last tile of a prompt) has nothing to compute at all
    const bool any_row = (kMayPack && t.pk) || t.q0 + wave * 32 < t.q_end;
    n_w = any_row ? min(t.n_tiles, w_pmax / kTK + 1) : 0;
    head_off = (size_t)t.g * 4096;
  };
  enter(cur);

  // B operand of S^T: Q^T[d][row]; step t covers d = 16 t .. 16 t + 15
  bf16x8 qf[8];
  auto load_q = [&](const Item& t) {
    int r, hq;
    bool ok;
    map_row(t, r, hq, ok);
    const uint16_t* qrow = q + (size_t)(t.tok0 + r) * q_row_stride + (t.h + hq) * 128 + half * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
      qf[i] = ok ? *reinterpret_cast<const bf16x8*>(qrow + i * 16) : z;
    }
  };
  // key steps 0 and 1 and value step 0 of an item (ids from its record) into the buffers of parity p
  auto stage_first = [&](const Item& t, int r, int p) {
    const size_t ho = (size_t)t.g * 4096;
    stage_k(kbufs + p * kKTileBytes, k_cache, __shfl(r, 8 + kq), ho, blk_stride, wave, lane);
    stage_v(vbufs + p * kVTileBytes, v_cache, __builtin_amdgcn_readlane(r, 8 + wave), ho, blk_stride, wave, lane);
    stage_k(kbufs + (p ^ 1) * kKTileBytes, k_cache, __shfl(r, 12 + kq), ho, blk_stride, wave, lane);
  };

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

  stage_first(cur, rec_next, 0);
  load_q(cur);
  int next_idk = __shfl(rec_next, 16 + kq);                // K ids run two steps ahead of the scores
  int next_idv = __shfl(rec_next, 12 + vq);                // V ids one step ahead
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (kTK > cur.L_total()) {  // the first step already runs past the end of the sequence
    fix_tail(vbufs, cur.L_total(), tid);
    __syncthreads();
  }
  // Quotas of the queues.  The XCDs of one device do not run this kernel equally fast (their workgroups end up
  // to 8% apart, in a pattern that holds from launch to launch), and a launch is over when the slowest is: so a
  // queue's share of the items follows its XCD's busy time in the previous launch of the same batch (one step
  // of proportional control per launch; the items that change hands are the lightest ones at the lists' ends,
  // hence the gain above one).  Which workgroup computes an item does not change its result.
  if (wave == 0) {
    // workgroup w runs on XCD w % 8, and lane l summed workgroups l, l + 64, ...: all of XCD l % 8
    float sum = busy_sum;
    sum += __shfl_xor(sum, 8);
    sum += __shfl_xor(sum, 16);
    sum += __shfl_xor(sum, 32);
    auto over_queues_i = [&](int v) { v += __shfl_xor(v, 1); v += __shfl_xor(v, 2); v += __shfl_xor(v, 4); return v; };
    auto over_queues_f = [&](float v) { v += __shfl_xor(v, 1); v += __shfl_xor(v, 2); v += __shfl_xor(v, 4); return v; };
    const int x = lane & 7;
    const int crew = ((int)gridDim.x - x + kQueues - 1) / kQueues;
    const int own = max(n_flat - x + kQueues - 1, 0) / kQueues;
    const float T = sum / (float)max(crew, 1);
    const float T_mean = over_queues_f(T) * 0.125f;
    const bool big = n_flat >= kBalanceMinItems && (int)gridDim.x <= kPlanMaxWgs && gridDim.x % kQueues == 0;
    const bool same = prev_items == n_flat && prev_grid == (int)gridDim.x;
    float sh = same && share > 0.f ? share : 1.f;
    if (big && same && __all(T > 0.f))
      sh = fminf(kShareMax, fmaxf(kShareMin, sh + kShareGain * (T_mean - T) / T_mean));
    sh *= 8.f / over_queues_f(sh);
    int quota = (int)((float)own * sh + 0.5f);
    const int quota_sum = over_queues_i(quota);
    if (x == kQueues - 1) quota += n_flat - quota_sum;  // the last queue takes the rounding
    const bool ok = big && __all(quota >= 2 * crew && own >= 2 * crew);
    if (!ok) quota = own;
    if (lane < kQueues) {
      qtab[lane] = quota;
      qtab[kQueues + lane] = own;
      if (blockIdx.x == 0) {
        reinterpret_cast<float*>(plan)[kPlanShare0 + kQueues * parity + lane] = ok ? sh : 1.f;
        if (lane == 0) {
          plan[kPlanMeta0 + parity] = n_flat;
          plan[kPlanMeta0 + 2 + parity] = (int)gridDim.x;
        }
      }
    }
  }
  int par = 0;  // buffer that holds step 0 of the current item

  f32x16 sa[2], sb[2];  // scores of the current / next step, roles alternate

  // One step of an item: turns the scores of step j (`sc`, masked) into weights and accumulates
  // V(j) P(j) while the matrix cores already compute the scores of step j+1 into `sn`.  The loop
  // calls it with the two arrays swapped in turn, so no copy is needed.  The last step of an item
  // has no next scores to compute; instead it brings in the first K/V steps and the query rows
  // of the next item, so that the only cost of changing items is the unoverlapped score product
  // of the new item's step 0.
  auto iteration = [&](auto last_tag, int j, f32x16 (&sc)[2], f32x16 (&sn)[2]) {
    constexpr bool is_last = decltype(last_tag)::value;
    const int pj = (j + par) & 1;
    char* const kcur = kbufs + pj * kKTileBytes;               // held K(j), consumed: receives K(j+2)
    const char* const knext = kbufs + (pj ^ 1) * kKTileBytes;
    const char* const vcur = vbufs + pj * kVTileBytes;
    char* const vnext = vbufs + (pj ^ 1) * kVTileBytes;
    // The eight global -> LDS copies of a step (K of step j + 2, V of step j + 1) are issued one per slot under
    // the first matrix instructions of the step instead of in a block before them (2.5% on long prompts); a
    // wavefront that has nothing to compute in this step issues them at once.  K past the item's last step
    // re-stages its last block into a buffer that nobody reads before the next item's first step overwrites it.
    const int idv_s = __builtin_amdgcn_readfirstlane(next_idv);
    // one address register pair for the four K copies and one for the four V copies: the pieces differ in the
    // instructions' immediate offsets (stage_k_imm)
    const char* const ksrc_w = k_cache + (size_t)next_idk * blk_stride + head_off + (size_t)(lane & 15) * 16 + wave * 1024;
    const char* const vsrc = v_cache + (size_t)idv_s * blk_stride + head_off + (size_t)lane * 32;
    auto copy = [&](int i) {
      if (i < 4) stage_k_one(kcur, ksrc_w, wave, i);
      else stage_v_one(vnext, vsrc, wave, i - 4);
    };
    auto next_ids = [&]() {
      next_idk = block_id(cur.bt_row, 4 * (j + 3) + kq, cur.nblk_total());
      next_idv = block_id(cur.bt_row, 4 * (j + 2) + vq, cur.nblk_total());
    };
    if constexpr (!is_last) {
      if (j >= n_w) {
#pragma unroll
        for (int i = 0; i < 8; ++i) copy(i);
        next_ids();
      }
    } else if (f_next >= 0) {
      const Item nxt = describe(rec_next, g_next, h_next, block_table, bt_stride);
      stage_first(nxt, rec_next, pj ^ 1);
      load_q(nxt);  // the current item's scores are all computed: its query rows make room
    }

    if (j < n_w) {  // uniform per wavefront
      const float mc = m * c;
      const char* kb = knext + a_k_off;
      const char* vb = vcur + a_v_off;
      bf16x8 pf0[2], pf1[2];
      const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
      float pv[2];
      float bmx = 0.f;
      // 32 matrix instructions per step, in this order:
      //   slots  0..15  scores of step j+1: d step t = slot/2, 32-key half = slot%2
      //   slots 16..23  O += V P, keys  0..31 of step j: d tile = i%4, 16-key step = i/4
      //   slots 24..31  O += V P, keys 32..63
      // Consecutive slots write different accumulators (a dependent matrix instruction cannot
      // issue back to back).  Each slot is followed by the slice of softmax VALU work that
      // runs under it (one weight of keys 0..31 per slot in 0..15, two weights of keys 32..63
      // per slot in 16..23), and the LDS read of a slot's A fragment is issued kAhead slots
      // early.  The fences keep the compiler from regrouping the slots.  The last step of an
      // item skips the matrix instructions of slots 0..15.
      constexpr int kAhead = 4;
      auto frag = [&](int s) -> bf16x8 {
        if (s < 16) return *reinterpret_cast<const bf16x8*>(kb + (2 * (s >> 1) * kTK + 32 * (s & 1)) * 16);
        const int i = s & 7;
        return *reinterpret_cast<const bf16x8*>(vb + (2 * (i >> 2) + (s < 24 ? 0 : 4)) * kVOctStride +
                                                (i & 3) * 32 * 16);
      };
      // one weight: value e of accumulator s -> pv[e & 1]; every second one completes a pair
      auto weight = [&](const f32x16& s, bf16x8 (&pf)[2], int e) {
        pv[e & 1] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[e], c, -mc));
        if (e & 1) {
          const bf16x2 a = {(__bf16)pv[0], (__bf16)pv[1]};
          l = __builtin_amdgcn_fdot2_f32_bf16(a, ones, l, false);
          asm volatile("" : "+v"(l));  // keeps the sum in its slot (it would otherwise sink below the loop)
          pf[e >> 3][(e & 7) - 1] = a[0];
          pf[e >> 3][(e & 7)] = a[1];
        }
      };
      f32x16 zero;
#pragma unroll
      for (int i = 0; i < 16; ++i) zero[i] = 0.f;
      bf16x8 fr[2 * kAhead];
#pragma unroll
      for (int s = 0; s < kAhead; ++s) fr[s] = frag(s);
#pragma unroll
      for (int s = 0; s < 32; ++s) {
        if (s + kAhead < 32) fr[(s + kAhead) % (2 * kAhead)] = frag(s + kAhead);
        const bf16x8 a = fr[s % (2 * kAhead)];
        if (s < 16) {
          if constexpr (!is_last) {
            sn[s & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[s >> 1], s < 2 ? zero : sn[s & 1], 0, 0, 0);
            if (s >= 1 && s <= 8) copy(s - 1);  // the step's copies ride in slots 1..8, the next block ids in slot 9
            if (s == 9) next_ids();
          }
          weight(sc[0], pf0, s);
        } else if (s < 24) {
          const int i = s - 16;
          o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf0[i >> 2], o[i & 3], 0, 0, 0);
          weight(sc[1], pf1, 2 * i);
          weight(sc[1], pf1, 2 * i + 1);
        } else {
          const int i = s - 24;
          o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf1[i >> 2], o[i & 3], 0, 0, 0);
          if constexpr (!is_last) {
            // the next step's scores are complete since slot 17: their maximum (without a mask) is
            // built here, four values per slot
            auto val = [&](int k) { return sn[k >> 4][k & 15]; };
            if (i == 0) {
              bmx = max3(val(0), val(1), val(2));
              bmx = max3(bmx, val(3), val(4));
            } else if (i < 7) {
              bmx = max3(bmx, val(4 * i + 1), val(4 * i + 2));
              bmx = max3(bmx, val(4 * i + 3), val(4 * i + 4));
            } else {
              bmx = max3(bmx, val(29), val(30));
              bmx = fmaxf(bmx, val(31));
            }
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      if constexpr (!is_last) {
        const int k0n = (j + 1) * kTK;
        // a step at the diagonal needs the mask first: its maximum is taken again from the masked scores
        const float bm = k0n + kTK - 1 > w_pmin ? mask_and_max(sn, k0n, half, pos, true) : across_halves(bmx);
        if (__any((bm - m) * c > kTau)) {
          // the next step's scores exceed the exponent offset by more than 2^kTau: raise it
          const float m_new = fmaxf(m, bm);
          const float alpha = __builtin_amdgcn_exp2f((m - m_new) * c);
          l *= alpha;
#pragma unroll
          for (int dt = 0; dt < 4; ++dt) o[dt] *= alpha;
          m = m_new;
        }
      }
    }

    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    // the ticket requested when this item began has arrived: publish the item it stands for
    if (j == 0 && tid == 0 && f_next >= 0) slot[0] = resolve(pend);
    __syncthreads();
    if constexpr (!is_last) {
      if ((j + 2) * kTK > cur.L_total()) {  // the next V step runs past the end of the sequence
        fix_tail(vnext, cur.L_total() - (j + 1) * kTK, tid);
        __syncthreads();
      }
    } else if (f_next >= 0) {
      const int L_next = __builtin_amdgcn_readlane(rec_next, 3) + __builtin_amdgcn_readlane(rec_next, 4);
      if (kTK > L_next) {
        fix_tail(vnext, L_next, tid);
        __syncthreads();
      }
    }
  };

  for (;;) {
    // K steps 0 and 1 and V step 0 of the current item are in LDS (step 0 in the buffers of
    // parity `par`), its query rows in qf.  Ask for the record of the next item and for the
    // ticket of the one after it; both arrive while this item is being computed.
    if (f_next >= 0) {
      split(f_next);
      g_next = g_of_f;
      h_next = h_of_f;
      rec_next = load_rec(tile_of_f);
      if (tid == 0) pend = atomicAdd(counter, 1);
    }
    if (n_w > 0) {
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int i = 0; i < 16; ++i) sa[sub][i] = 0.f;
      const char* kb = kbufs + par * kKTileBytes + a_k_off;
#pragma unroll
      for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(kb + (2 * t * kTK + 32 * sub) * 16);
          sa[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[t], sa[sub], 0, 0, 0);
        }
      m = mask_and_max(sa, 0, half, pos, kTK - 1 > w_pmin);
    }
    __syncthreads();  // K step 0 is consumed: its buffer receives step 2

    {
      // plain steps run in pairs (sa -> sb -> sa); the last step always takes its scores from sa, so a
      // left-over single plain step is followed by a copy
      int j = 0;
      for (; j + 2 < cur.n_tiles; j += 2) {
        iteration(std::false_type(), j, sa, sb);
        iteration(std::false_type(), j + 1, sb, sa);
      }
      if (j + 2 == cur.n_tiles) {
        iteration(std::false_type(), j, sa, sb);
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) sa[sub] = sb[sub];
        ++j;
      }
      iteration(std::true_type(), j, sa, sb);
    }

    {
      const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(l), __float_as_uint(l), false, false);
      l = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    }
    {
      // Registers 4 i4 .. 4 i4 + 3 of o[dt] hold d = 32 dt + 8 i4 + 4 half + (0..3): 8 bytes of output.
      // The two lanes of a row exchange halves (one v_permlane32_swap per register pair) so that
      // the lower lane holds the 16 bytes of d = 32 dt + 16 p .. + 7 and the upper lane the next 16.
      const float inv = 1.f / l;
      int row, hsel;  // (worked out again rather than kept in registers through the item)
      bool row_valid;
      map_row(cur, row, hsel, row_valid);
      uint16_t* orow = out + ((size_t)(cur.tok0 + row) * Hq + cur.h + hsel) * 128 + half * 8;
      auto pack = [&](float a, float b) {
        const bf16x2 v = {(__bf16)(a * inv), (__bf16)(b * inv)};
        return __builtin_bit_cast(uint32_t, v);
      };
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int p = 0; p < 2; ++p) {
          const f32x16& v = o[dt];
          const auto r0 = __builtin_amdgcn_permlane32_swap(pack(v[8 * p + 0], v[8 * p + 1]),
                                                           pack(v[8 * p + 4], v[8 * p + 5]), false, false);
          const auto r1 = __builtin_amdgcn_permlane32_swap(pack(v[8 * p + 2], v[8 * p + 3]),
                                                           pack(v[8 * p + 6], v[8 * p + 7]), false, false);
          u32x4 w;
          w[0] = r0[0];
          w[1] = r1[0];
          w[2] = r0[1];
          w[3] = r1[1];
          if (row_valid) *reinterpret_cast<u32x4*>(orow + dt * 32 + p * 16) = w;
        }
    }
    if (lse && half == 0) {
      int row, hsel;
      bool row_valid;
      map_row(cur, row, hsel, row_valid);
      if (row_valid) lse[(size_t)(cur.tok0 + row) * Hq + cur.h + hsel] = (m * c + log2f(l)) * kLn2;
    }
    if (f_next < 0) break;

    // next item: its first steps were staged by the last step above, into the other parity
    par = (par + cur.n_tiles) & 1;
    cur = describe(rec_next, g_next, h_next, block_table, bt_stride);
    f_next = __builtin_amdgcn_readfirstlane(slot[0]);
    enter(cur);
    next_idk = __shfl(rec_next, 16 + kq);
    next_idv = __shfl(rec_next, 12 + vq);
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[dt][i] = 0.f;
    l = 0.f;
  }
  if (tid == 0 && blockIdx.x < kPlanMaxWgs)
    plan[kPlanBusy0 + parity * kPlanMaxWgs + blockIdx.x] = (int)(wall_clock64() - t_begin);
}

// Workgroups of the attention launch: the persistent grid, or fewer if the batch cannot hold that
// many items (0: nothing to do, -1: too many items to number).
int32_t prefill_mfma_grid(const AttnArgs& a, int32_t T, int32_t n_persistent_wgs) {
  // sum over sequences of ceil(S_b / kTQ) <= T / kTQ + (number of non-empty sequences)
  const int64_t n_items = prefill_plan_tiles(a.B, T) * a.Hq;
  if (n_items <= 0) return 0;
  if (n_items > 0x7fffffffLL - (1 << 20)) return -1;
  return (int32_t)(n_items < n_persistent_wgs ? n_items : n_persistent_wgs);
}

hipError_t launch_prefill_mfma(const AttnArgs& a, const int32_t* cu_q, const int32_t* ctx_before, int32_t T,
                               int32_t max_q_len, int32_t* ws_plan, int32_t n_persistent_wgs, bool make_plan,
                               int parity, hipStream_t s) {
  const int G = a.Hq / a.Hkv;
  const int64_t max_tiles = prefill_plan_tiles(a.B, T);
  const int32_t n_wg = prefill_mfma_grid(a, T, n_persistent_wgs);
  if (n_wg == 0) return hipSuccess;
  if (n_wg < 0) return hipErrorInvalidValue;
  if (make_plan)
    hipLaunchKernelGGL(prefill_plan_kernel, dim3(1), dim3(kPlanThreads), 0, s, cu_q, ctx_before, a.block_table,
                       a.bt_stride, a.B, (int)n_wg, (int)max_tiles, G, ws_plan);
  auto launch = [&](auto kernel) {
    hipLaunchKernelGGL(kernel, dim3((unsigned)n_wg), dim3(256), 0, s, (const uint16_t*)a.q, a.q_row_stride,
                       (const char*)a.k_cache, (const char*)a.v_cache, a.block_table, a.bt_stride, (uint16_t*)a.out,
                       a.lse, ws_plan, parity, a.Hq, a.Hkv, G, make_divisor((uint32_t)(G * a.Hkv)),
                       make_divisor((uint32_t)a.Hkv), a.scale_log2e);
  };
  // The variant that can pack short prompts' tiles for batches that may hold many of them (few new tokens
  // per sequence on average); which tiles are packed is decided by the tile list, from the lengths themselves.
  (void)max_q_len;
  if (G > 1 && (int64_t)T <= (int64_t)a.B * 2 * (kTQ / G))
    launch(prefill_mfma_kernel<true>);
  else
    launch(prefill_mfma_kernel<false>);
  return hipGetLastError();
}

}  // namespace eco
