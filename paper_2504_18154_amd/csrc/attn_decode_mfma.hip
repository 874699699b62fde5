// Split-context paged decode attention, bf16, head size 128, on gfx950 matrix cores.
//
// Eq. 2 of Section 2.1 for one new token per sequence against the whole cached context:
// the memory-bound phase of Table 2 (every cached K and V byte is read once per step,
// arithmetic intensity = the GQA group size).  The kernel is organised around the HBM
// stream; the matrix cores are used only so that arithmetic never gets in its way.
//
// Work decomposition ("flat" split-context).  A unit of work is one 16-token cache block
// of one (sequence, K/V head): 4 KiB of K and 4 KiB of V serving all G query heads of the
// group.  Units are numbered sequence-major, then K/V head, then logical block (each
// (sequence, head) preceded by a few empty units that stand for the fixed cost of a piece), and the
// numbering is cut into equal chunks of C units, one chunk per wavefront of a persistent
// grid (one workgroup of 4 wavefronts per CU: one wavefront per SIMD, which is also the oldest
// and so never starved by the memory pipeline's oldest-first arbitration).  Context lengths live on the device, so every
// workgroup derives the numbering itself from a prefix sum over the batch (a few hundred
// integers).  All wavefronts therefore stream the same number of bytes whatever the mix of
// context lengths, start together and finish together.  A chunk may cover the tail of one
// (sequence, head), several whole ones and the head of another; each covered piece yields
// one partial softmax state.  On request the chunks are not equal but proportional to the
// speed of the XCD a wavefront runs on, as measured by the context's earlier launches (the
// XCDs of one device stream at rates several percent apart, stable over time): every
// wavefront records units and time, the merge kernel turns them into per-XCD shares for
// the next launch.
//
// Per piece, the wavefront streams whole cache blocks with fully coalesced per-lane loads
// (non-temporal buffer loads through a descriptor per block, see load_block) that land
// directly in MFMA operand layout - no LDS staging, no barriers, a register pipeline
// kDepth blocks deep, physical block ids prefetched 64 at a time into one VGPR:
//   scores  S^T[token][head] = K . Q^T   v_mfma_f32_16x16x32_bf16 (heads padded to 16 columns)
//   online softmax per column in the exp2 domain; the four 16-lane groups hold different
//   tokens of the same head, their maxima are combined with wavefront shuffles
//   values  O^T[d][head] += V^T . P^T    v_mfma_f32_16x16x16_bf16
// The accumulator layout of the first product is already the B-operand layout of the
// second, so P never leaves registers.  A piece that is a whole (sequence, head) writes the
// final output; otherwise (m, l, unnormalised o) go to the workspace and a small merge
// kernel combines them exactly.  With the step's append fused in (k_new given), the wavefront
// that reaches a sequence's last block takes the new token from the new rows, and the merge
// launch stores it into the cache.
//
// Lane layouts relied upon (lane = 16*quad + col):
//   16x16x32:  A[row=col][k = 8*quad .. 8*quad+7],  B[k = 8*quad..+7][col],
//   16x16x16:  A[row=col][k = 4*quad .. 4*quad+3],  B[k = 4*quad..+3][col],
//   both:      C[row = 4*quad + i][col], i = 0..3.
#include "common.h"

namespace eco {

constexpr int kWaves = 4;
// kDepth - 1 cache blocks of 8 KiB are in flight per wavefront behind the one being worked on.  One
// wavefront per SIMD: a second one buys nothing (the memory pipeline serves the older one first; a grid
// of two workgroups per CU was 4% slower on batches of a thousand short sequences once the pipeline ran
// through from piece to piece, and no faster on any other), and a fourth block in flight needs more
// registers than the pipeline's state leaves (the compiler then parks fragments in AGPRs and copies
// them back).
constexpr int kDecodeDepth = 3;

struct KVFrag {
  bf16x8 k[4];   // K block: unit (4*kk + quad, token = col)  ->  A operand of S^T step kk
  s16x4 v[8];    // V block: V^T[16*dt + col][tokens 4*quad..+3] ->  A operand of O^T tile dt
};

// Every cached K/V byte is read once per launch and by one wavefront only, so the loads carry
// the non-temporal hint: the caches then do not keep the lines, and the device streams them
// faster (a plain read of the same bytes in the same 8 KiB pieces: 7.0-7.2 TB/s with the
// hint against 6.0-6.4 TB/s without).  They are buffer loads through a descriptor of the one
// block (4 KiB of K, 4 KiB of V): the block's address is wavefront-uniform and lives in scalar
// registers, the lanes' offsets are two constants, and a load the pipeline issues past the end
// of a piece (`live` false) gets a descriptor of zero bytes, which the hardware answers with
// zeros without touching memory (the address it holds is a valid block all the same).
constexpr int kRsrcRaw = 0x00020000;  // untyped 32-bit data, no swizzle, no stride
constexpr int kAuxNonTemporal = 2;
__device__ __forceinline__ void load_block(KVFrag& f, const char* __restrict__ kbase, const char* __restrict__ vbase,
                                           bool live, int lane, int col, int quad) {
  const int bytes = live ? 4096 : 0;
  const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(kbase), 0, bytes, kRsrcRaw);
  const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(vbase), 0, bytes, kRsrcRaw);
  const int koff = lane * 16, voff = col * 32 + quad * 8;
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
    f.k[kk] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(rk, koff + kk * 1024, 0, kAuxNonTemporal));
#pragma unroll
  for (int dt = 0; dt < 8; ++dt)
    f.v[dt] = __builtin_bit_cast(s16x4, __builtin_amdgcn_raw_buffer_load_b64(rv, voff + dt * 512, 0, kAuxNonTemporal));
}

// One block's worth of work for one wavefront: scores, online softmax update, value
// accumulation.  `tail` is the number of valid slots in the block (16 unless it is the
// ragged last block of the sequence).
__device__ __forceinline__ void process_block(KVFrag& f, const bf16x8 (&qf)[4], f32x4 (&acc)[8], float& m, float& l,
                                              int tail, int quad, float scale_log2e) {
  // S^T[token = 4*quad+i][head = col]
  f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.k[kk], qf[kk], s, 0, 0, 0);
  s *= scale_log2e;
  if (tail < 16) {
    // ragged tail of the sequence: slots >= tail hold no token.  Their scores are excluded,
    // and their V entries zeroed so that stale bits (possibly NaN) times a zero weight
    // cannot reach the accumulator.
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (4 * quad + i >= tail) s[i] = -INFINITY;
#pragma unroll
    for (int dt = 0; dt < 8; ++dt)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (4 * quad + i >= tail) f.v[dt][i] = 0;
  }
  float bm = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
  bm = fmaxf(bm, __shfl_xor(bm, 16));
  bm = fmaxf(bm, __shfl_xor(bm, 32));
  const float m_new = fmaxf(m, bm);  // finite: every block of the slice holds >= 1 token
  const float alpha = __builtin_amdgcn_exp2f(m - m_new);
  f32x4 p;
#pragma unroll
  for (int i = 0; i < 4; ++i) p[i] = __builtin_amdgcn_exp2f(s[i] - m_new);
  l = l * alpha + ((p[0] + p[1]) + (p[2] + p[3]));  // per-lane partial; quads are summed at the end
  if (__any(m_new != m)) {
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) acc[dt] *= alpha;
  }
  m = m_new;
  const bf16x4 pb = __builtin_convertvector(p, bf16x4);
  const s16x4 pbits = __builtin_bit_cast(s16x4, pb);
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) acc[dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(f.v[dt], pbits, acc[dt], 0, 0, 0);
}

// A piece costs a wavefront several blocks' worth of time (finding it, its query rows, its result; before
// the block pipeline ran through from piece to piece also a fill and a drain: a wavefront's end time rose
// by ~3 us with every piece in its chunk), and some chunks hold a dozen pieces when others hold one.  So
// that equal chunks are equal work, every (sequence, K/V head) is numbered with kPieceCost units in front
// of its blocks that stand for that cost and hold no data (in units of a block's time).
// (a fit of the wavefronts' times against their blocks and pieces gives 2.7 to 3 block times per piece on
// three batch shapes; with 2, 3, 4 units 1024 sequences of ~120 tokens take 101.1, 99.9, 102.7 us and 512 of
// ~400 tokens 149.1, 148.5, 149.5 us; the benchmark batches do not care)
constexpr int kPieceCost = 3;

// Exclusive prefix sums of the per-sequence unit counts (blocks + kPieceCost) into LDS: pre[b] = units
// per K/V head of sequences 0..b-1, pre[B] = all; lens[b] = context length.  Called by all 256 threads.
__device__ __forceinline__ void scan_block_counts(int* pre, int* lens, int* wsum, const int32_t* __restrict__ ctx_len,
                                                  int B) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int per = (B + kWaves * 64 - 1) / (kWaves * 64);
  const int b0 = tid * per;
  int local = 0;
  for (int i = 0; i < per; ++i)
    if (b0 + i < B) local += ((ctx_len[b0 + i] + 15) >> 4) + kPieceCost;
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
      const int L = ctx_len[b0 + i];
      lens[b0 + i] = L;
      pre[b0 + i] = run;
      run += ((L + 15) >> 4) + kPieceCost;
    }
  if (tid == 0) pre[B] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
  __syncthreads();
}

// a / b for a >= 0, b > 0: the numbering's unit counts are 64-bit for the largest pools, but almost always fit
// 32 bits, where the division is a fraction of the instructions (the values are wavefront-uniform)
__device__ __forceinline__ long long div_units(long long a, int b) {
  return (a >> 31) == 0 ? (long long)((uint32_t)a / (uint32_t)b) : a / b;
}

// Chunk size in units: forced, or the equal share of the persistent grid's wavefronts.
__device__ __forceinline__ long long chunk_units(long long U, int n_waves, int c_forced) {
  if (c_forced > 0) return c_forced;
  const long long c = div_units(U + n_waves - 1, n_waves);
  return c < kMinSplitTokens / kBlockSize ? kMinSplitTokens / kBlockSize : c;
}

// The numbering of units is dealt to the wavefronts in rounds of 8 workgroups (workgroup ids go
// round-robin to the 8 XCDs, so position x of a round runs on XCD x): the 4 wavefronts of the
// workgroup at position x take c[x] units each, cum[x] = 4 (c[0] + .. + c[x-1]) units into the
// round, cum[8] units per round.  With equal c this is plain "wavefront w takes units
// [w c, (w + 1) c)"; unequal c let the XCDs carry shares of the stream in proportion to their
// measured speeds.
struct Chunking {
  const int* c;    // [8]
  const int* cum;  // [9]
  __device__ __forceinline__ long long begin(int gw) const {
    const int wg = gw >> 2, x = wg & 7;
    return (long long)(wg >> 3) * cum[8] + cum[x] + (gw & 3) * c[x];
  }
  __device__ __forceinline__ int size(int gw) const { return c[(gw >> 2) & 7]; }
  __device__ __forceinline__ int owner(long long u) const {  // the wavefront whose chunk holds unit u
    const long long r = div_units(u, cum[8]);
    const int off = (int)(u - r * cum[8]);
    int x = 0;
#pragma unroll
    for (int y = 1; y < 8; ++y)
      if (cum[y] <= off) x = y;
    return (int)((r * 8 + x) * 4 + (off - cum[x]) / c[x]);
  }
};
constexpr int kMetaPre = 18;  // ws_meta: [0..7] c, [8..16] cum, then the batch prefix sums

// Where a cut piece's partial states live.  A chunk holds at most two cut pieces: its first piece, if the
// (sequence, head) began in an earlier chunk (`begins` false), and its last piece, if the (sequence, head)
// begins here and runs on into later chunks (`begins` true); a piece that is cut at both ends is the chunk's
// only one.  So wavefront gw owns the two groups of G slots 2 gw and 2 gw + 1 (one slot per query head of the
// group: 128 floats in ws_acc, 2 in ws_ml), and the workspace grows with the grid, not with the batch.
// The k-th state of a (sequence, head) that begins in chunk w: group 2 w + 1 for k = 0, group 2 (w + k) after.
__device__ __forceinline__ size_t partial_slot(int gw, bool begins, int G) {
  return (size_t)(2 * gw + (begins ? 1 : 0)) * G;
}

template <int kDepth>
__global__ __launch_bounds__(kWaves * 64, 1) void decode_mfma_kernel(
    const uint16_t* __restrict__ q, int q_row_stride, const uint16_t* __restrict__ k_new,
    const uint16_t* __restrict__ v_new, int new_row_stride, const char* __restrict__ k_cache,
    const char* __restrict__ v_cache,
    const int32_t* __restrict__ block_table, int bt_stride, const int32_t* __restrict__ ctx_len,
    uint16_t* __restrict__ out, float* __restrict__ lse, float* __restrict__ ws_acc, float* __restrict__ ws_ml,
    int32_t* __restrict__ ws_meta, int c_forced, const float* __restrict__ share_in,
    float* __restrict__ share_out, const float* __restrict__ xcd_speed, int32_t* __restrict__ ws_wave,
    int32_t* __restrict__ ws_cut, int B, int Hq, int Hkv, int G, float scale_log2e) {
  __shared__ int pre[kMaxBatch + 1];
  __shared__ int lens[kMaxBatch];
  __shared__ int wsum[kWaves];
  __shared__ int s_c[8], s_cum[9];
  __shared__ __attribute__((aligned(16))) uint16_t s_new[kWaves][256];  // fused append: a token's K row, then its V row
  constexpr int kOutBytes = 16384;
  __shared__ __attribute__((aligned(16))) char s_out[kWaves][kOutBytes];  // final results on their way out
  const long long t_start = wall_clock64();
  scan_block_counts(pre, lens, wsum, ctx_len, B);

  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int col = lane & 15, quad = lane >> 4;
  const int n_waves = gridDim.x * kWaves;
  const long long U = (long long)pre[B] * Hkv;
  if (threadIdx.x == 0) {
    const long long C = chunk_units(U, n_waves, c_forced);
    // Per-XCD chunk sizes from the shares (mean 1); equal chunks if there are none, or if
    // rounding left the rounds short of covering all units.  The shares move half way from
    // their previous values towards the relative speeds that the previous launch measured
    // (every workgroup computes the same numbers; the first one stores them for the next launch).
    int c[8];
    long long sum = 0;
    if (share_in) {
      float share[8], mean = 0.f, total = 0.f;
      bool measured = true;
      for (int x = 0; x < 8; ++x) {
        share[x] = share_in[x];
        mean += xcd_speed[x];
        measured = measured && xcd_speed[x] > 0.f;
      }
      mean *= 0.125f;
      if (measured)
        for (int x = 0; x < 8; ++x) share[x] = fminf(1.5f, fmaxf(0.5f, 0.5f * share[x] + 0.5f * xcd_speed[x] / mean));
      for (int x = 0; x < 8; ++x) total += share[x];
      for (int x = 0; x < 8; ++x) {
        share[x] *= 8.f / total;
        if (blockIdx.x == 0) share_out[x] = share[x];
        c[x] = max(kMinSplitTokens / kBlockSize, (int)(share[x] * ((float)U / (float)n_waves)) + 1);
        sum += c[x];
      }
    }
    const bool ok = share_in && 4 * sum * (gridDim.x >> 3) >= U;
    int cum = 0;
    for (int x = 0; x < 8; ++x) {
      s_c[x] = ok ? c[x] : (int)C;
      s_cum[x] = cum;
      cum += 4 * s_c[x];
    }
    s_cum[8] = cum;
  }
  __syncthreads();
  const Chunking ch = {s_c, s_cum};
  if (blockIdx.x == 0) {
    // the merge kernel reads the numbering instead of recomputing it
    for (int i = threadIdx.x; i <= B; i += kWaves * 64) ws_meta[kMetaPre + i] = pre[i];
    if (threadIdx.x < 8) ws_meta[threadIdx.x] = s_c[threadIdx.x];
    if (threadIdx.x < 9) ws_meta[8 + threadIdx.x] = s_cum[threadIdx.x];
  }
  const int gw = blockIdx.x * kWaves + wave;
  const long long u_begin = ch.begin(gw);
  const long long u_end = min(U, u_begin + ch.size(gw));
  const size_t blk_stride = (size_t)Hkv * 4096;
  if (u_begin >= u_end) {
    if (ws_wave && lane == 0) ws_wave[2 * gw] = 0;  // no units: not a sample of this XCD's speed
    if (ws_cut && lane == 0) ws_cut[4 * gw] = 0;
    return;
  }

  // A piece: the blocks [blk0, blk0 + n) of one (sequence b, K/V head g) that fall into this
  // wavefront's chunk.  Everything a piece needs before its first K/V load - where it is
  // (LDS only), its query fragments and its first 64 block ids - is fetched while the
  // previous piece is still streaming, and so are its first blocks (see the pipeline below),
  // so a change of piece costs no memory round trip.
  struct Piece {
    int b, g, blk0, n, nb, L;  // blocks [blk0, blk0 + n) of the nb blocks of (b, g); n == 0: the chunk ends before block 0
    long long seg_u0;          // first unit of (b, g): kPieceCost cost units, then its blocks
    long long u_stop;          // where the piece ends in the numbering (chunk end or end of (b, g))
  };
  auto locate = [&](long long u) {
    Piece p;
    const int key = (int)div_units(u, Hkv);  // largest b with pre[b] <= u / Hkv
    // every lane probes one candidate per round (pre is increasing and pre[lo] <= key throughout, so the lanes
    // that see pre <= key are the first few): two rounds for the largest batch instead of twelve LDS round trips
    int lo = 0, n_cand = B;
    while (n_cand > 1) {
      const int stride = (n_cand + 63) >> 6;
      const int idx = lo + lane * stride;
      const bool le = idx < lo + n_cand && pre[idx] <= key;
      const int last = __popcll(__ballot(le)) - 1;
      const int new_lo = lo + last * stride;
      n_cand = min(stride, lo + n_cand - new_lo);
      lo = new_lo;
    }
    p.b = lo;
    const int nu = pre[lo + 1] - pre[lo];  // units of one (sequence, head)
    p.nb = nu - kPieceCost;
    const long long seq_u0 = (long long)pre[lo] * Hkv;
    p.g = (int)div_units(u - seq_u0, nu);
    p.seg_u0 = seq_u0 + (long long)p.g * nu;
    p.u_stop = min(u_end, p.seg_u0 + nu);
    p.blk0 = max((int)(u - p.seg_u0) - kPieceCost, 0);
    p.n = max((int)(p.u_stop - p.seg_u0) - kPieceCost, 0) - p.blk0;
    p.L = lens[lo];
    return p;
  };
  // The piece after p, which ended at the end of its (sequence, head) with units left in the chunk: the
  // next K/V head, or head 0 of the next sequence - two LDS reads instead of a search.  A sequence without
  // tokens (not a valid decode input, but it must not cost its neighbours their results) has no blocks and
  // is passed over.
  auto following = [&](const Piece& p) {
    Piece q = p;
    do {
      const long long seg = q.seg_u0 + q.nb + kPieceCost;
      if (++q.g == Hkv) {
        q.g = 0;
        ++q.b;
      }
      const int nu = pre[q.b + 1] - pre[q.b];
      q.nb = nu - kPieceCost;
      q.seg_u0 = seg;
      q.u_stop = min(u_end, seg + nu);
      q.blk0 = 0;
      q.n = max((int)(q.u_stop - seg) - kPieceCost, 0);
      q.L = lens[q.b];
    } while (q.n == 0 && q.u_stop < u_end);
    return q;
  };
  // B operand of S^T: Q^T[d][head], heads beyond the group are zero columns
  auto load_q = [&](bf16x8 (&qf)[4], const Piece& p) {
    const uint16_t* qrow = q + (size_t)p.b * q_row_stride + ((size_t)p.g * G + col) * 128;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
      qf[kk] = col < G ? *reinterpret_cast<const bf16x8*>(qrow + kk * 32 + quad * 8) : z;
    }
  };
  // A piece is not streamed front to back: position i of the piece is block (start + i * step) mod (n - 1)
  // of its first n - 1 blocks, with a start of its own and a step co-prime to n - 1, and its last block
  // comes last (it may be the ragged end of the sequence, which only the closing rounds of the loop below
  // handle).  The softmax does not care about the order, and the memory system does: with block tables
  // that hand a sequence consecutive physical blocks (a fresh allocator), wavefronts that walk their
  // sequences front to back advance by the same 4 KiB * Hkv from load to load, and the stream is 6-9%
  // slower than over a shuffled table (128 sequences of 8192 tokens: 730 vs 664 us; with staggered starts
  // alone 690 us); with the strided walk it is as fast as the best (639 us), and a shuffled table is
  // unaffected.
  auto start_of = [&](const Piece& p) {
    const uint32_t h = ((uint32_t)p.b * 0x9E3779B1u + (uint32_t)p.g * 0x85EBCA77u) >> 8;
    return (int)(((unsigned long long)(h & 0xffffffu) * (unsigned)(p.n - 1)) >> 24);  // in [0, n - 1), 0 for n = 1
  };
  auto step_of = [&](const Piece& p) {  // the first of 37, 41, 43 (7, 5, 11 for short pieces) that does not divide n - 1
    const int m = p.n - 1;
    if (m <= 12) return 1;
    if (m <= 40) return m % 7 != 0 ? 7 : m % 5 != 0 ? 5 : 11;
    return m % 37 != 0 ? 37 : m % 41 != 0 ? 41 : 43;
  };
  auto block_at = [&](const Piece& p, int start, int step, int i) {  // i in [0, n)
    const int m = p.n - 1;
    if (i == m) return p.blk0 + i;
    return p.blk0 + (int)(((unsigned)start + (unsigned)i * (unsigned)step) % (unsigned)m);
  };
  // physical ids of up to 64 consecutive positions of a piece, lane i holding position base + i
  auto load_ids = [&](const Piece& p, int start, int step, int base) {
    int id = 0;
    if (base + lane < p.n) id = block_table[(size_t)p.b * bt_stride + block_at(p, start, step, base + lane)];
    return id;
  };

  // Final results wait in LDS and go out together (when the wavefront's buffer is full, and at the end of
  // its chunk): a global store in the middle of the stream would make the next wait for a K/V load a full
  // drain (loads and stores pending together count as unordered), and the block pipeline below runs through
  // piece after piece without one.  An entry: G output rows of 256 bytes (contiguous in `out` too), G
  // log-sum-exps, (sequence, K/V head).
  const int entry_bytes = G * 256 + 64 + 16;
  const int k_entries = kOutBytes / entry_bytes;  // >= 1: G <= 16
  char* const obuf = s_out[wave];
  int n_buf = 0;
  auto flush = [&]() {
    for (int e = 0; e < n_buf; ++e) {
      const char* ent = obuf + e * entry_bytes;
      const int eb = *reinterpret_cast<const int*>(ent + G * 256 + 64);
      const int eg = *reinterpret_cast<const int*>(ent + G * 256 + 68);
      char* orow = reinterpret_cast<char*>(out + ((size_t)eb * Hq + (size_t)eg * G) * 128);
      for (int idx = lane; idx < G * 16; idx += 64)
        *reinterpret_cast<u32x4*>(orow + idx * 16) = *reinterpret_cast<const u32x4*>(ent + idx * 16);
      if (lse && lane < G) lse[(size_t)eb * Hq + eg * G + lane] = *reinterpret_cast<const float*>(ent + G * 256 + lane * 4);
    }
    n_buf = 0;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // nothing but loads pending from here on
  };

  Piece cur = locate(u_begin);
  if (cur.n == 0 && cur.u_stop < u_end) cur = following(cur);  // (the chunk begins at an empty sequence)
  if (cur.n > 0) {  // (else: only the cost units of a (sequence, head) fall into this chunk)
    bf16x8 qf[4];
    load_q(qf, cur);
    int start = start_of(cur), step = step_of(cur);
    int ids = load_ids(cur, start, step, 0);
    // Register pipeline kDepth blocks deep, running without a break through the whole chunk.  Blocks are
    // taken in windows of up to 64 (the ids one VGPR holds); a window of n blocks occupies np = n rounded
    // up to kDepth pipeline slots (the slots behind its last block do no work and their loads are loads of
    // nothing), so every window starts on f[0] and the loop has one shape.  Slot t's load is issued
    // kDepth - 1 slots early; the issue slots that reach past a window fetch the first blocks of what
    // follows it (the piece's next 64 blocks, or the next piece), which therefore arrive while this
    // window's last blocks are worked on: a change of window or piece does not drain the pipeline.  Every
    // slot issues the same twelve loads, so the number in flight never varies and waits stay precise.
    KVFrag f[kDepth];
    {
      const int n0 = min(64, cur.n);
#pragma unroll
      for (int d = 0; d < kDepth - 1; ++d) {
        const size_t off = (size_t)__builtin_amdgcn_readlane(ids, min(d, n0 - 1)) * blk_stride + (size_t)cur.g * 4096;
        load_block(f[d], k_cache + off, v_cache + off, d < n0, lane, col, quad);
      }
    }
    for (;;) {
      const bool has_next = cur.u_stop < u_end;
      Piece nxt = cur;
      bf16x8 qn[4];
      int ids_n = 0, start_n = 0, step_n = 1;
      if (has_next) {
        nxt = following(cur);
        load_q(qn, nxt);
        start_n = start_of(nxt);
        step_n = step_of(nxt);
        ids_n = load_ids(nxt, start_n, step_n, 0);
      }
      const size_t head_off = (size_t)cur.g * 4096;
      const int L = cur.L;
      // fused append: if this piece reaches the end of its sequence, the new token's K and V rows (512 bytes)
      // are fetched now, 8 bytes per lane, and wait in two registers until the last block is worked on
      u32x2 new_row = {0u, 0u};
      if (k_new != nullptr && cur.blk0 + cur.n == cur.nb) {
        const size_t row = (size_t)cur.b * new_row_stride + (size_t)cur.g * 128 + (lane & 31) * 4;
        new_row = *reinterpret_cast<const u32x2*>((lane < 32 ? k_new : v_new) + row);
      }

      f32x4 acc[8];
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
      float m = -INFINITY, l = 0.f;

      int base = 0;
      do {  // (bottom-tested loops: the compiler then knows that loads were issued since the piece began)
        const int n = min(64, cur.n - base);
        const int my_id = ids;
        const bool more = base + 64 < cur.n;
        if (more) ids = load_ids(cur, start, step, base + 64);  // ids of the following 64 blocks, early
        // what follows this window: the piece's next 64 blocks, or the first blocks of the next piece
        const size_t nhead = more ? head_off : (size_t)nxt.g * 4096;
        const int nn = more ? min(64, cur.n - base - 64) : (has_next ? min(64, nxt.n) : 0);
        const int np = (n + kDepth - 1) / kDepth * kDepth;
        auto issue = [&](KVFrag& fr, int t, bool may_follow) {  // the load of pipeline slot t (t < np + kDepth - 1)
          size_t off;
          bool live = t < n;
          if (may_follow && t >= np && t - np < nn) {
            // (kept a real branch: taken only behind a window's end, and reading the ids earlier would
            // wait for a load that has only just been issued)
            asm volatile("" ::: "memory");
            int id;
            if (more) {
              id = __builtin_amdgcn_readlane(ids, t - np);
            } else {
              asm volatile("" ::: "memory");
              id = __builtin_amdgcn_readlane(ids_n, t - np);
            }
            off = (size_t)id * blk_stride + nhead;
            live = true;
          } else {
            off = (size_t)__builtin_amdgcn_readlane(my_id, min(t, n - 1)) * blk_stride + head_off;
          }
          load_block(fr, k_cache + off, v_cache + off, live, lane, col, quad);
        };
        auto tail_of = [&](int i) { return L - (block_at(cur, start, step, base + i) << 4); };  // > 16 except in the sequence's last block
        // Fused append (k_new given): the sequence's newest token, slot t of its last block, is not in the
        // cache yet.  The wavefront that streams that block (exactly one per K/V head) takes the token's K
        // and V from the new rows instead, in the operand layout the block's loads produce.  The slot itself
        // is written by the merge launch that follows.
        auto append_token = [&](KVFrag& fr, int t) {
          // through LDS into the operand layout: lane l holds bytes [8 l, 8 l + 8) of (K row, V row)
          uint16_t* const st = s_new[wave];
          *reinterpret_cast<u32x2*>(st + lane * 4) = new_row;
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
          __builtin_amdgcn_wave_barrier();
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
          if (col == t) {
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) fr.k[kk] = *reinterpret_cast<const bf16x8*>(st + kk * 32 + quad * 8);
          }
          if (quad == (t >> 2)) {
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
              const short x = (short)st[128 + dt * 16 + col];
#pragma unroll
              for (int e = 0; e < 4; ++e)
                if (e == (t & 3)) fr.v[dt][e] = x;
            }
          }
        };
        int i = 0;
        // the body of a window: every slot it issues lies inside the window and no block is the sequence's last
        for (; i + 2 * kDepth - 1 <= n; i += kDepth) {
#pragma unroll
          for (int d = 0; d < kDepth; ++d) {
            const size_t off = (size_t)__builtin_amdgcn_readlane(my_id, i + d + kDepth - 1) * blk_stride + head_off;
            load_block(f[(d + kDepth - 1) % kDepth], k_cache + off, v_cache + off, true, lane, col, quad);
            process_block(f[d], qf, acc, m, l, 16, quad, scale_log2e);
          }
        }
        // its last one or two rounds (at least kDepth - 1 blocks are left): the general form
        do {
#pragma unroll
          for (int d = 0; d < kDepth; ++d) {
            issue(f[(d + kDepth - 1) % kDepth], i + d + kDepth - 1, d > 0);  // (slot i + kDepth - 1 is never past the window)
            if (i + d < n) {
              const int tail = tail_of(i + d);
              if (k_new != nullptr && tail <= 16) {
                asm volatile("" ::: "memory");  // (a real branch: once per (sequence, head))
                append_token(f[d], tail - 1);
              }
              process_block(f[d], qf, acc, m, l, tail, quad, scale_log2e);
            }
          }
          i += kDepth;
        } while (i < np);
        base += 64;
      } while (base < cur.n);

      // ---- this piece's result: lanes (col = head, quad) hold o[d = 16 dt + 4 quad + i] --------
      l += __shfl_xor(l, 16);
      l += __shfl_xor(l, 32);
      if (cur.n == cur.nb) {  // the whole (sequence, head): final, into the LDS buffer
        if (n_buf == k_entries) flush();
        char* ent = obuf + n_buf * entry_bytes;
        if (col < G) {
          const float inv = 1.f / l;
#pragma unroll
          for (int dt = 0; dt < 8; ++dt) {
            u32x2 w;
            w[0] = pack_bf16x2(acc[dt][0] * inv, acc[dt][1] * inv);
            w[1] = pack_bf16x2(acc[dt][2] * inv, acc[dt][3] * inv);
            *reinterpret_cast<u32x2*>(ent + col * 256 + (dt * 16 + 4 * quad) * 2) = w;
          }
          if (quad == 0) *reinterpret_cast<float*>(ent + G * 256 + col * 4) = (m + log2f(l)) * kLn2;
        }
        if (lane == 0) {
          *reinterpret_cast<int*>(ent + G * 256 + 64) = cur.b;
          *reinterpret_cast<int*>(ent + G * 256 + 68) = cur.g;
        }
        ++n_buf;
      } else {  // a cut (sequence, head): at most the first and the last piece of a chunk
        if (col < G) {
          const size_t slot = partial_slot(gw, cur.blk0 == 0, G) + col;
#pragma unroll
          for (int dt = 0; dt < 8; ++dt) *reinterpret_cast<f32x4*>(ws_acc + slot * 128 + dt * 16 + 4 * quad) = acc[dt];
          if (quad == 0) {
            ws_ml[slot * 2 + 0] = m;
            ws_ml[slot * 2 + 1] = l;
          }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // (see flush)
      }
      if (!has_next || nxt.n == 0) break;  // n == 0: only the cost units of the next (sequence, head) are left
      cur = nxt;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) qf[kk] = qn[kk];
      ids = ids_n;
      start = start_n;
      step = step_n;
    }
    flush();
  }
  if (ws_cut && lane == 0) {
    // For the merge kernel: a (sequence, K/V head) that starts in this chunk and runs on into later ones
    // is this chunk's last piece; its partial states are those of this wavefront and the following
    // n_split - 1.  Every cut (sequence, head) is reported exactly once, by the chunk it starts in.
    const bool cut = cur.n > 0 && cur.blk0 == 0 && cur.n < cur.nb;
    ws_cut[4 * gw] = cut ? ch.owner(cur.seg_u0 + kPieceCost + cur.nb - 1) - gw + 1 : 0;
    ws_cut[4 * gw + 1] = cur.b;
    ws_cut[4 * gw + 2] = cur.g;
  }
  if (ws_wave && lane == 0) {  // units streamed and time taken (100 MHz ticks), for the XCD shares
    ws_wave[2 * gw] = (int)(u_end - u_begin);
    ws_wave[2 * gw + 1] = (int)(wall_clock64() - t_start);
  }
}

// Feedback for the next launch: the speed of XCD x is the mean over its wavefronts of units
// streamed per tick (0 if most of them had nothing to stream: then the launch is too small to
// tell).  One wavefront per XCD.
__device__ __forceinline__ void measure_xcd_speed(float* __restrict__ xcd_speed, const int32_t* __restrict__ ws_wave,
                                                  int n_waves, int x) {
  float v = 0.f, n = 0.f, idle = 0.f;
  for (int i = threadIdx.x; 32 * (i >> 2) + 4 * x + (i & 3) < n_waves; i += 64) {
    const int w = 32 * (i >> 2) + 4 * x + (i & 3);  // wavefront i of XCD x
    const int units = ws_wave[2 * w], ticks = ws_wave[2 * w + 1];
    if (units > 0 && ticks > 0) {
      v += (float)units / (float)ticks;
      n += 1.f;
    } else {
      idle += 1.f;
    }
  }
  v = wave_sum(v);
  n = wave_sum(n);
  idle = wave_sum(idle);
  if (threadIdx.x == 0) xcd_speed[x] = n > idle ? v / n : 0.f;
}

// The fused append's stores, carried by the merge launch: token b of the new rows goes to position
// ctx_len[b] - 1 of sequence b.  k_new == NULL: nothing to do.
struct AppendJob {
  const uint16_t* k_new;
  const uint16_t* v_new;
  int new_row_stride;
  uint16_t* k_cache;
  uint16_t* v_cache;
  const int32_t* block_table;
  int bt_stride;
  const int32_t* ctx_len;
  int B, Hkv;
};
// Workgroup `bid` of `n_blocks` (64 threads each) takes the (sequence, K/V head) pairs bid, bid + n_blocks, ...
__device__ __forceinline__ void append_new_tokens(const AppendJob& j, int bid, int n_blocks) {
  if (j.k_new == nullptr) return;
  for (int pair = bid; pair < j.B * j.Hkv; pair += n_blocks) {
    const int b = pair / j.Hkv, g = pair % j.Hkv, lane = (int)threadIdx.x;
    // the token's rows are asked for first: they do not depend on where the token goes, and the two
    // dependent reads that tell (length, block table) are then answered alongside them
    const size_t row = (size_t)b * j.new_row_stride + (size_t)g * 128;
    u32x4 kval = {0u, 0u, 0u, 0u};
    if (lane < 16) kval = *reinterpret_cast<const u32x4*>(j.k_new + row + lane * 8);
    const uint16_t v0 = j.v_new[row + lane], v1 = j.v_new[row + 64 + lane];
    const int p = j.ctx_len[b] - 1;
    if (p < 0) continue;  // an empty sequence has no new token (and no output row worth reading)
    const int64_t blk = j.block_table[(size_t)b * j.bt_stride + (p >> 4)];
    const int slot = p & 15;
    const size_t base = ((size_t)blk * j.Hkv + g) * 2048;  // elements of one (block, head): 16 slots x 128
    // K: unit c of the row goes to [c][slot][8 elements]; V: element d to [d][slot]
    if (lane < 16) *reinterpret_cast<u32x4*>(j.k_cache + base + (size_t)lane * 128 + slot * 8) = kval;
    j.v_cache[base + (size_t)lane * 16 + slot] = v0;
    j.v_cache[base + (size_t)(64 + lane) * 16 + slot] = v1;
  }
}

// The n_split partial states of one query head (number i of its group) of a (sequence, K/V head) that begins
// in chunk w, into its output row (and log-sum-exp); one wavefront, lanes own pairs of head-vector elements.
__device__ __forceinline__ void merge_partials(const float* __restrict__ ws_acc, const float* __restrict__ ws_ml,
                                               int w, int i, int G, int n_split, uint16_t* __restrict__ orow,
                                               float* __restrict__ lse_out) {
  const int lane = threadIdx.x;
  auto slot = [&](int k) { return partial_slot(w + k, k == 0, G) + i; };
  float M = -INFINITY;
  float lsum = 0.f, o0 = 0.f, o1 = 0.f;
  if (n_split <= 4) {
    // the usual case (a chunk boundary or two inside the sequence): every state is asked for at once
    float mk[4], lk[4];
    float2 ak[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const bool in = k < n_split;
      mk[k] = in ? ws_ml[slot(k) * 2] : -INFINITY;
      lk[k] = in ? ws_ml[slot(k) * 2 + 1] : 0.f;
      ak[k] = in ? *reinterpret_cast<const float2*>(ws_acc + slot(k) * 128 + 2 * lane) : float2{0.f, 0.f};
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) M = fmaxf(M, mk[k]);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float wk = k < n_split ? exp2f(mk[k] - M) : 0.f;
      lsum += lk[k] * wk;
      o0 += ak[k].x * wk;
      o1 += ak[k].y * wk;
    }
  } else {
    for (int k = 0; k < n_split; ++k) M = fmaxf(M, ws_ml[slot(k) * 2]);
    for (int k = 0; k < n_split; ++k) {
      const float wk = exp2f(ws_ml[slot(k) * 2] - M);
      lsum += ws_ml[slot(k) * 2 + 1] * wk;
      const float2 a = *reinterpret_cast<const float2*>(ws_acc + slot(k) * 128 + 2 * lane);
      o0 += a.x * wk;
      o1 += a.y * wk;
    }
  }
  const float inv = 1.f / lsum;
  const uint32_t packed = pack_bf16x2(o0 * inv, o1 * inv);
  *reinterpret_cast<uint32_t*>(orow + 2 * lane) = packed;
  if (lse_out && lane == 0) *lse_out = (M + log2f(lsum)) * kLn2;
}

// Merge of the partial softmax states of every (sequence, query head) that was cut:
//   M = max_k m_k;  l = sum_k l_k 2^(m_k - M);  o = sum_k acc_k 2^(m_k - M) / l.
// grid (Hq, B), 64 threads; lanes own pairs of head-vector elements.
__global__ __launch_bounds__(64) void decode_flat_merge_kernel(const float* __restrict__ ws_acc,
                                                              const float* __restrict__ ws_ml,
                                                              const int32_t* __restrict__ ws_meta,
                                                              uint16_t* __restrict__ out, float* __restrict__ lse,
                                                              float* __restrict__ xcd_speed,
                                                              const int32_t* __restrict__ ws_wave, int n_waves,
                                                              int Hq, int Hkv, int G, AppendJob job) {
  const int h = blockIdx.x, b = blockIdx.y, g = h / G;
  append_new_tokens(job, b * Hq + h, (int)(gridDim.x * gridDim.y));
  if (xcd_speed && b * Hq + h < 8) measure_xcd_speed(xcd_speed, ws_wave, n_waves, b * Hq + h);
  const Chunking ch = {ws_meta, ws_meta + 8};
  const int p0 = ws_meta[kMetaPre + b], nu = ws_meta[kMetaPre + b + 1] - p0;  // units: kPieceCost + blocks
  const long long seg_u0 = (long long)p0 * Hkv + (long long)g * nu;
  const int w0 = ch.owner(seg_u0 + kPieceCost);  // the chunk that holds block 0
  const int n_split = ch.owner(seg_u0 + nu - 1) - w0 + 1;
  if (n_split <= 1) return;  // written in final form by the decode kernel
  merge_partials(ws_acc, ws_ml, w0, h - g * G, G, n_split, out + ((size_t)b * Hq + h) * 128,
                 lse ? lse + (size_t)b * Hq + h : nullptr);
}

// The same merge for the persistent grid, where the decode kernel has listed the cut (sequence, K/V head)s:
// grid (wavefronts of the decode launch, G), 64 threads; block (w, i) merges query head i of the group that
// chunk w reported, if it reported one.  A batch of many short sequences has far more (sequence, head)s than
// cuts, and this grid does not grow with it.
__global__ __launch_bounds__(64) void decode_cut_merge_kernel(const float* __restrict__ ws_acc,
                                                             const float* __restrict__ ws_ml,
                                                             const int32_t* __restrict__ ws_cut,
                                                             uint16_t* __restrict__ out, float* __restrict__ lse,
                                                             float* __restrict__ xcd_speed,
                                                             const int32_t* __restrict__ ws_wave, int n_waves,
                                                             int Hq, int G, AppendJob job) {
  const int w = blockIdx.x;
  const int n_split = ws_cut[4 * w];  // (asked for before the append's own chain of loads, answered alongside it)
  const int b = ws_cut[4 * w + 1], h = ws_cut[4 * w + 2] * G + blockIdx.y;
  append_new_tokens(job, w * G + (int)blockIdx.y, (int)(gridDim.x * gridDim.y));
  if (xcd_speed && w * G + (int)blockIdx.y < 8) measure_xcd_speed(xcd_speed, ws_wave, n_waves, w * G + blockIdx.y);
  if (n_split <= 1) return;
  merge_partials(ws_acc, ws_ml, w, (int)blockIdx.y, G, n_split, out + ((size_t)b * Hq + h) * 128,
                 lse ? lse + (size_t)b * Hq + h : nullptr);
}

int64_t decode_mfma_waves(int32_t B, int32_t Hkv, int32_t max_ctx_len, int32_t split_tokens,
                          int32_t n_persistent_wgs) {
  if (split_tokens <= 0) return (int64_t)n_persistent_wgs * kWaves;
  // forced chunk size: the grid must cover the largest possible number of units
  const int64_t c_forced = split_tokens / kBlockSize;
  const int64_t u_max = (int64_t)B * Hkv * ((max_ctx_len + kBlockSize - 1) / kBlockSize + kPieceCost);
  const int64_t waves = (u_max + c_forced - 1) / c_forced;
  return (waves + kWaves - 1) / kWaves * kWaves;
}

hipError_t launch_decode_mfma(const AttnArgs& a, const int32_t* ctx_len, int32_t split_tokens, int32_t max_ctx_len,
                              int32_t n_persistent_wgs, float* ws_acc, float* ws_ml, int32_t* ws_meta,
                              int64_t ws_waves, const float* share_in, float* share_out, const float* xcd_speed,
                              int32_t* ws_wave, int32_t* ws_cut, hipStream_t s) {
  const int G = a.Hq / a.Hkv;
  const int64_t n_waves = decode_mfma_waves(a.B, a.Hkv, max_ctx_len, split_tokens, n_persistent_wgs);
  if (n_waves > ws_waves || n_waves / kWaves > 0x7fffffffLL) return hipErrorInvalidValue;  // the workspace holds two slot groups per wavefront
  const int n_wg = (int)(n_waves / kWaves);
  int c_forced = 0;
  if (split_tokens > 0) {
    c_forced = split_tokens / kBlockSize;
    share_in = nullptr;
    ws_cut = nullptr;  // sized for the persistent grid only
  }
  if (n_wg % 8 != 0) share_in = nullptr;  // the rounds of 8 workgroups would not line up with the XCDs
  if (!share_in) ws_wave = nullptr;
  auto launch = [&](auto kernel) {
    hipLaunchKernelGGL(kernel, dim3((unsigned)n_wg), dim3(kWaves * 64), 0, s, (const uint16_t*)a.q, a.q_row_stride,
                       (const uint16_t*)a.k_new, (const uint16_t*)a.v_new, a.new_row_stride, (const char*)a.k_cache, (const char*)a.v_cache, a.block_table, a.bt_stride, ctx_len,
                       (uint16_t*)a.out, a.lse, ws_acc, ws_ml, ws_meta, c_forced, share_in, share_out,
                       xcd_speed, ws_wave, ws_cut, a.B, a.Hq, a.Hkv, G, a.scale_log2e);
  };
  launch(decode_mfma_kernel<kDecodeDepth>);
  return hipGetLastError();
}

hipError_t launch_decode_mfma_merge(const AttnArgs& a, const int32_t* ctx_len, const float* ws_acc, const float* ws_ml,
                                    const int32_t* ws_meta, float* xcd_speed,
                                    const int32_t* ws_wave, const int32_t* ws_cut, int32_t n_waves, hipStream_t s) {
  const AppendJob job = {(const uint16_t*)a.k_new, (const uint16_t*)a.v_new, a.new_row_stride,
                         (uint16_t*)const_cast<void*>(a.k_cache), (uint16_t*)const_cast<void*>(a.v_cache),
                         a.block_table, a.bt_stride, ctx_len, a.B, a.Hkv};
  if (ws_cut) {
    hipLaunchKernelGGL(decode_cut_merge_kernel, dim3((unsigned)n_waves, (unsigned)(a.Hq / a.Hkv)), dim3(64), 0, s,
                       ws_acc, ws_ml, ws_cut, (uint16_t*)a.out, a.lse, xcd_speed, ws_wave, n_waves, a.Hq,
                       a.Hq / a.Hkv, job);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(decode_flat_merge_kernel, dim3((unsigned)a.Hq, (unsigned)a.B), dim3(64), 0, s, ws_acc, ws_ml,
                     ws_meta, (uint16_t*)a.out, a.lse, xcd_speed, ws_wave, n_waves, a.Hq, a.Hkv,
                     a.Hq / a.Hkv, job);
  return hipGetLastError();
}

}  // namespace eco
