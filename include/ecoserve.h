/*
 * ecoserve.h -- C ABI of the paged-attention hot path of an EcoServe instance
 * (arXiv 2504.18154) for AMD MI355X (gfx950).
 *
 * An EcoServe instance alternates between phase-pure prefill-only and
 * decode-only batches (Section 3.2, temporal disaggregation).  In both modes
 * the device time of the attention layer is Eq. 2 of Section 2.1,
 *     Attention(Q,K,V) = softmax(Q K^T / sqrt(d_k)) V,
 * evaluated over a KV cache (Section 2.1) that is organised in fixed-size
 * blocks addressed through a per-sequence block table (Section 5, "KV cache
 * management"), with grouped-query head sharing (Section 4.1).  This library
 * is that path and nothing else: append new K/V rows to the paged cache,
 * causal variable-length prefill attention, split-context decode attention.
 *
 * General rules
 *   - Plain C.  No exception crosses the boundary; every call returns a
 *     status code (ECOSERVE_OK == 0) and ecoserve_strerror() names it.
 *   - "dev" pointers are device (HBM) addresses on the context's GPU, "host"
 *     pointers are ordinary host memory.  Every buffer is caller-owned.  The
 *     library allocates device memory only in ecoserve_create() and
 *     ecoserve_set_option() and frees it in ecoserve_destroy().
 *   - The three hot calls validate what the host can see (pointers, sizes,
 *     alignment, limits) BEFORE launching anything, then enqueue their kernels
 *     on the given HIP stream and return without synchronising.
 *   - Contents of device arrays (block-table entries, lengths) are not
 *     checked by the hot calls; out-of-range contents are undefined
 *     behaviour.  ecoserve_debug_validate() checks them synchronously.
 *   - One call handles one layer; callers loop over layers.
 *   - Calls that share a context must be issued on one stream (or be ordered
 *     by the caller): they share the context's workspace (split-context partial
 *     states of decode, the query-tile list of prefill).
 *   - With the default options the hot calls may be recorded into a HIP graph
 *     (they neither allocate nor synchronise, and record no memset nodes).
 *     Options whose state advances on the host from call to call
 *     (ECOSERVE_OPT_PROFILE, ECOSERVE_OPT_DECODE_ADAPTIVE,
 *     ECOSERVE_OPT_PREFILL_REUSE_PLAN) are for eager calls: a recorded launch
 *     replays the arguments it was recorded with.
 *
 * Notation (Table 1 of the paper, extended): B sequences in the batch, Hq
 * query heads (M in the paper), Hkv key/value heads, G = Hq/Hkv, D per-head
 * size, bs tokens per cache block.  Query head h uses K/V head h / G.
 *
 * Cache layout (fixed, one pool for K and one for V per layer; E = element
 * type, x = 16 / sizeof(E) elements = one 16-byte unit):
 *
 *   k_cache : E[num_blocks][Hkv][D / x][bs][x]
 *             (block, K/V head, 16-byte unit of the head vector, slot, element)
 *   v_cache : E[num_blocks][Hkv][D][bs]
 *             (block, K/V head, element of the head vector, slot)
 *
 * Each (block, head) is one contiguous piece of bs*D*sizeof(E) bytes (4 KiB
 * for bf16, D = 128, bs = 16), so a wavefront streams it with fully coalesced
 * 16-byte (K) and 8-byte (V) per-lane loads that land directly in the operand
 * layout of the gfx950 matrix instructions.  ecoserve_k_cache_index() and
 * ecoserve_v_cache_index() give the element offset of a logical coordinate.
 */
#ifndef ECOSERVE_H
#define ECOSERVE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ecoserve_ctx ecoserve_ctx; /* opaque; owns a device workspace and timing events */

enum {
  ECOSERVE_OK = 0,
  ECOSERVE_EINVAL = 1,       /* NULL / negative / inconsistent / misaligned argument */
  ECOSERVE_EUNSUPPORTED = 2, /* valid in principle, not built (head size, block size, dtype) */
  ECOSERVE_ENOMEM = 3,       /* device or host allocation failed */
  ECOSERVE_EHIP = 4,         /* a HIP runtime call or kernel launch failed */
  ECOSERVE_ECONTENT = 5      /* ecoserve_debug_validate(): device-resident contents are out of range */
};

enum { ECOSERVE_BF16 = 0, ECOSERVE_F32 = 1 };

/* Head layout and paging of one layer's cache.
 * Supported: block_size == 16; num_q_heads % num_kv_heads == 0 with
 * G = Hq/Hkv <= 16; dtype BF16 with head_dim 128 (matrix-core kernels) or any
 * head_dim that is a multiple of 8 up to 256 (plain kernels); dtype F32 with
 * head_dim a multiple of 4 up to 256 (plain kernels). */
typedef struct {
  int32_t num_q_heads;
  int32_t num_kv_heads;
  int32_t head_dim;
  int32_t block_size;
  int32_t num_blocks;   /* physical blocks in one layer's pool */
  int32_t dtype;        /* ECOSERVE_BF16 | ECOSERVE_F32: type of q, k, v, caches and out */
  float softmax_scale;  /* 0 => 1/sqrt(head_dim), the scale of Eq. 2 */
} ecoserve_layout;

/* Tuning and test knobs for ecoserve_set_option(). */
enum {
  /* Tokens of context per decode split (multiple of 64, 64..4096).  0 restores
   * the built-in choice, which depends on B and max_ctx_len. */
  ECOSERVE_OPT_DECODE_SPLIT_TOKENS = 1,
  /* 1: use the plain (non matrix-core) kernels even where the fast ones apply. */
  ECOSERVE_OPT_FORCE_PLAIN = 2,
  /* n >= 1: bracket the dominant kernel of every n-th hot call of each kind
   * (counted from the last ecoserve_profile_reset(), the first one included)
   * with HIP events on the call's stream; read the sums with
   * ecoserve_profile_read().  0 (default): off.  An event pair delays the
   * stream by a few microseconds, so a timed loop samples (n around 7)
   * rather than bracketing every launch.  Negative: ECOSERVE_EINVAL. */
  ECOSERVE_OPT_PROFILE = 3,
  /* 1: decode (bf16, head size 128, built-in split) cuts the K/V stream into per-XCD shares that
   * follow the speeds measured in the context's earlier decode calls (the XCDs of one device
   * differ by several percent and finish together only with unequal shares).  Results stay
   * within the tolerance of the split-context merge but are no longer bit-identical from call
   * to call, because the cut points move with the measurements.  0 (default): equal shares,
   * bit-reproducible. */
  ECOSERVE_OPT_DECODE_ADAPTIVE = 4,
  /* 1: consecutive ecoserve_attn_prefill calls (bf16, head size 128) that pass the same cu_q,
   * ctx_before and block_table pointers, bt_stride, B and T are taken to describe the same
   * batch - the caller vouches that the arrays' contents have not changed - and share the list
   * of query tiles that the first of them builds, instead of each building its own (the layers
   * of one step of a model: the list depends only on these arrays).  0 (default): every call
   * builds its list.  Setting the option, to either value, forgets the current list: a caller
   * whose allocator may hand the same addresses to a new batch sets it again at every step.
   * With the option on, ecoserve_attn_prefill on a stream that is being captured returns
   * ECOSERVE_EINVAL (a recorded launch cannot decide at replay whether its list is current). */
  ECOSERVE_OPT_PREFILL_REUSE_PLAN = 5
};

enum { ECOSERVE_KERNEL_APPEND = 0, ECOSERVE_KERNEL_PREFILL = 1, ECOSERVE_KERNEL_DECODE = 2 };

/* Create a context on `device` for batches of at most max_batch sequences whose
 * block tables have at most max_blocks_per_seq entries per sequence.
 * Allocates the decode workspace (split-context partial results).  On failure
 * *out is NULL. */
int ecoserve_create(ecoserve_ctx** out, int device, const ecoserve_layout* layout,
                    int32_t max_batch, int32_t max_blocks_per_seq);

/* Frees the workspace and events.  Synchronises the device first.  NULL is OK. */
int ecoserve_destroy(ecoserve_ctx* ctx);

/* Set a knob (see ECOSERVE_OPT_*).  May reallocate the workspace, so it
 * synchronises the device; not for use between dependent hot calls in flight. */
int ecoserve_set_option(ecoserve_ctx* ctx, int32_t option, int32_t value);

/* Host-only helpers (no GPU needed). */
const char* ecoserve_strerror(int status);
/* Bytes of one layer's k_cache (== v_cache); 0 if the layout is invalid. */
size_t ecoserve_cache_bytes(const ecoserve_layout* layout);
/* Element offset of logical coordinate (blk, kv_head, slot, d) in k_cache / v_cache. */
size_t ecoserve_k_cache_index(const ecoserve_layout* layout, int32_t blk, int32_t kv_head, int32_t slot, int32_t d);
size_t ecoserve_v_cache_index(const ecoserve_layout* layout, int32_t blk, int32_t kv_head, int32_t slot, int32_t d);
/* Bytes of device workspace the context currently holds. */
size_t ecoserve_workspace_bytes(const ecoserve_ctx* ctx);

/*
 * KV-cache append (Section 2.1: the key and value embeddings of processed
 * tokens are saved in memory and reused by later steps; Section 5: fixed-size
 * blocks).  New token i of sequence b is stored at absolute position
 * p = ctx_before[b] + i: block block_table[b][p / bs], slot p % bs.  Bit-exact
 * copy.  Slots not addressed keep their contents.
 *
 *   k_cache, v_cache : dev, in/out, layout above, 16-byte aligned
 *   k_new, v_new     : dev, E[T][Hkv][D], sequences packed back to back, 16-byte aligned
 *   cu_q             : dev, int32[B+1], prefix sums of new-token counts, cu_q[0] = 0, cu_q[B] = T
 *   ctx_before       : dev, int32[B], tokens of each sequence already cached
 *   block_table      : dev, int32[B][bt_stride]; entries beyond a sequence's blocks are never read
 *   B, T             : batch size and total new tokens (B <= max_batch); B == 0 or T == 0 is a no-op
 *   max_new_len      : upper bound on any sequence's new-token count, in 1..T (sizes the launch;
 *                      <= 1 selects the one-token-per-sequence kernel); 0 with T > 0: ECOSERVE_EINVAL
 *   stream           : hipStream_t (NULL = the default stream)
 */
int ecoserve_kv_append(ecoserve_ctx* ctx, void* k_cache, void* v_cache, const void* k_new,
                       const void* v_new, const int32_t* cu_q, const int32_t* ctx_before,
                       const int32_t* block_table, int32_t bt_stride, int32_t B, int32_t T,
                       int32_t max_new_len, void* stream);

/*
 * Prefill attention (Section 2.1, Eq. 2; prefill phase: all prompt tokens at
 * once).  Causal, variable-length, grouped-query.  The new tokens' K/V must
 * already be in the cache (call ecoserve_kv_append first).  New token i of
 * sequence b sits at absolute position p = ctx_before[b] + i and attends to
 * cached keys 0..p of its own sequence.
 *
 *   q           : dev, E[T][Hq][D], packed by sequence like k_new
 *   k_cache, v_cache, cu_q, ctx_before, block_table, bt_stride, B, T : as in ecoserve_kv_append
 *   out         : dev, E[T][Hq][D] (rounded to E with round-to-nearest-even)
 *   lse         : dev, float[T][Hq] natural-log sum-exp of the scaled scores, or NULL
 *   max_q_len   : upper bound on any sequence's new-token count, in 1..T (checked; the kernels
 *                 take every length from cu_q, so a loose bound costs nothing)
 *   Sequences with zero new tokens are skipped.  B == 0 or T == 0 is a no-op.
 *   T / 128 + min(B, T) must not exceed num_blocks / 8 + max_batch (a batch cannot bring more
 *   new tokens than the pool holds; the context's list of query tiles is sized for that), else
 *   ECOSERVE_EINVAL.  The list lives in the context's workspace: see the rule on sharing a context.
 *   The workspace also carries, from one launch to the next, how long each workgroup was busy and
 *   the work queues' shares (ecoserve_debug_prefill_queue_shares): they decide which workgroup
 *   computes which query tile, never a result; out and lse of a call are the same bits whatever
 *   ran before it.
 */
int ecoserve_attn_prefill(ecoserve_ctx* ctx, const void* q, const void* k_cache, const void* v_cache,
                          const int32_t* cu_q, const int32_t* ctx_before, const int32_t* block_table,
                          int32_t bt_stride, void* out, float* lse, int32_t B, int32_t T,
                          int32_t max_q_len, void* stream);

/*
 * Decode attention (Section 2.1, Eq. 2; decode phase: one new token per
 * sequence attends to the whole cached context, which is what makes the phase
 * memory-bound, Table 2).  The new token's K/V must already be appended;
 * ctx_len[b] >= 1 counts it, and the query attends to keys 0..ctx_len[b]-1.
 * The context of a sequence is split across workgroups; partial softmax
 * states go through the context's workspace and are merged exactly.
 * A sequence with ctx_len[b] == 0 has no defined result: its rows of out and
 * lse hold unspecified values afterwards, the other sequences are unaffected.
 *
 *   q           : dev, E[B][Hq][D]
 *   ctx_len     : dev, int32[B]
 *   out         : dev, E[B][Hq][D];  lse : dev, float[B][Hq] or NULL
 *   max_ctx_len : upper bound on ctx_len[] (sizes the launch);
 *                 must be <= max_blocks_per_seq * block_size and <= bt_stride * block_size
 */
int ecoserve_attn_decode(ecoserve_ctx* ctx, const void* q, const void* k_cache, const void* v_cache,
                         const int32_t* block_table, int32_t bt_stride, const int32_t* ctx_len,
                         void* out, float* lse, int32_t B, int32_t max_ctx_len, void* stream);

/*
 * Synchronous check of device-resident arguments (tests and debugging; copies
 * the arrays to the host).  Verifies cu_q monotone from 0 (if given), every
 * length non-negative (decode: ctx_len >= 1 when cu_q == NULL), every block
 * table entry that a call would dereference inside [0, num_blocks), and that
 * no physical block is referenced twice.  `ctx_total[b]` is the number of
 * tokens of sequence b the call would touch (ctx_before + new, or ctx_len).
 * Returns ECOSERVE_ECONTENT on a violation.
 */
int ecoserve_debug_validate(ecoserve_ctx* ctx, const int32_t* cu_q, const int32_t* ctx_total,
                            const int32_t* block_table, int32_t bt_stride, int32_t B);

/*
 * The work queues' shares of the last ecoserve_attn_prefill launch of this
 * context (tests and debugging; waits for the device).  The matrix-core
 * prefill kernel deals its work items to eight queues, one per XCD of the
 * device; the XCDs do not run equally fast, so from the second launch on the
 * same batch (same item count) each queue's share of the items follows the
 * busy time its XCD's workgroups recorded in the launch before (Table 2 and
 * Section 2.1: prefill attention is the compute-bound phase, a launch is
 * over when its slowest part is).  Which workgroup computes an item does not
 * change any result.  shares[q] == 1 for every queue while no measurement
 * applies: the first launch of a batch, batches below 3072 items, the plain
 * kernels.
 *
 *   shares : host, float[8]; mean 1 over the queues
 */
int ecoserve_debug_prefill_queue_shares(ecoserve_ctx* ctx, float* shares);

/*
 * With ECOSERVE_OPT_PROFILE on: synchronise, then return the summed duration
 * (milliseconds) and the number of the bracketed launches of the dominant
 * kernel of `kernel` (ECOSERVE_KERNEL_*) since the last
 * ecoserve_profile_reset().
 */
int ecoserve_profile_read(ecoserve_ctx* ctx, int32_t kernel, double* ms_total, int64_t* launches);
int ecoserve_profile_reset(ecoserve_ctx* ctx);

/*
 * The three hot calls on rows that are not packed: Q, K and V read in place
 * from the output of the projection of Eq. 1 (Section 2.1), which a fused
 * projection writes as one row [Hq + 2 Hkv][D] per token.  The heads of one
 * token stay contiguous ([H][D]); consecutive tokens are `*_row_stride`
 * ELEMENTS apart: at least H * D, a multiple of 16 bytes, below 2^31.  For a
 * fused row, k_new = qkv + Hq * D, v_new = qkv + (Hq + Hkv) * D and all three
 * strides are (Hq + 2 Hkv) * D: no split copy of the projection output is
 * needed before the cache append.  Everything else (outputs packed
 * [T][Hq][D], errors, ownership) is as in the packed calls, which are these
 * with the strides Hkv * D and Hq * D.  A stride that breaks the rules above:
 * ECOSERVE_EINVAL.
 */
int ecoserve_kv_append_strided(ecoserve_ctx* ctx, void* k_cache, void* v_cache, const void* k_new,
                               const void* v_new, int64_t new_row_stride, const int32_t* cu_q,
                               const int32_t* ctx_before, const int32_t* block_table, int32_t bt_stride,
                               int32_t B, int32_t T, int32_t max_new_len, void* stream);
int ecoserve_attn_prefill_strided(ecoserve_ctx* ctx, const void* q, int64_t q_row_stride, const void* k_cache,
                                  const void* v_cache, const int32_t* cu_q, const int32_t* ctx_before,
                                  const int32_t* block_table, int32_t bt_stride, void* out, float* lse,
                                  int32_t B, int32_t T, int32_t max_q_len, void* stream);
int ecoserve_attn_decode_strided(ecoserve_ctx* ctx, const void* q, int64_t q_row_stride, const void* k_cache,
                                 const void* v_cache, const int32_t* block_table, int32_t bt_stride,
                                 const int32_t* ctx_len, void* out, float* lse, int32_t B, int32_t max_ctx_len,
                                 void* stream);

/*
 * Decode attention with the step's cache append fused in (Section 2.1: in the
 * decode phase every sequence brings exactly one new token, whose key and
 * value join the cache and whose query attends to the whole context).
 * Equivalent, bit for bit in cache and output, to ecoserve_kv_append_strided
 * of one token per sequence at position ctx_len[b] - 1 followed by
 * ecoserve_attn_decode_strided, in one launch less: the wavefront that
 * streams a sequence's last cache block takes the new token's K and V from
 * the new rows, and the small launch that merges the split contexts also
 * stores them into the block.  The cache holds the new tokens when the
 * call's work on `stream` is complete, like every other result.
 *
 *   k_new, v_new     : dev, row b = the new token of sequence b, [Hkv][D], rows
 *                      new_row_stride elements apart (rules of the strided calls)
 *   k_cache, v_cache : dev, in/out
 *   ctx_len          : dev, int32[B], context lengths INCLUDING the new token (>= 1)
 *   everything else as in ecoserve_attn_decode_strided.
 */
int ecoserve_attn_decode_append(ecoserve_ctx* ctx, const void* q, int64_t q_row_stride, const void* k_new,
                                const void* v_new, int64_t new_row_stride, void* k_cache, void* v_cache,
                                const int32_t* block_table, int32_t bt_stride, const int32_t* ctx_len,
                                void* out, float* lse, int32_t B, int32_t max_ctx_len, void* stream);

/*
 * ecoserve_attn_decode for callers that cannot allocate device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  No context: the layout is passed directly, and the scratch
 * memory of the two launches (partial softmax states of the split contexts,
 * the launch's numbering, the list of cut sequences) is a fixed array of
 * 16.3 MiB inside the library's device code, one copy per GPU, held until the
 * process ends.  The call allocates nothing (no hipMalloc / hipFree, no
 * events), does not synchronise, and launches the same kernels as
 * ecoserve_attn_decode with its default options (persistent grid, equal
 * shares), so the results are the same bits.
 *
 *   device      : ordinal of the GPU that holds every buffer (0 .. 63)
 *   layout      : host; dtype BF16 with head_dim 128 only (the matrix-core
 *                 kernels), else ECOSERVE_EUNSUPPORTED
 *   q, k_cache, v_cache, block_table, bt_stride, ctx_len, out, lse,
 *   max_ctx_len, stream : as in ecoserve_attn_decode (q and out packed
 *                 [B][Hq][D]); max_ctx_len <= bt_stride * block_size
 *   B           : at most 4096, else ECOSERVE_EINVAL (the array is sized for
 *                 that batch, any group size up to 16 and a grid of up to 256
 *                 workgroups; nothing else about the inputs is limited)
 *
 * All calls on one GPU share that GPU's array: calls that overlap there (two
 * streams, two threads) race; order them.  The array needs no clearing
 * between calls (a launch writes every word it later reads), and a call may
 * follow a larger one.
 */
int ecoserve_attn_decode_noalloc(int device, const ecoserve_layout* layout, const void* q, const void* k_cache,
                                 const void* v_cache, const int32_t* block_table, int32_t bt_stride,
                                 const int32_t* ctx_len, void* out, float* lse, int32_t B, int32_t max_ctx_len,
                                 void* stream);

/*
 * Machine ceilings for the roofline reasoning of Section 2.1 (Table 2 prices
 * decode attention in bytes read, prefill attention in matrix FLOPs): what
 * `device` sustains on each resource, to be reported beside the published
 * peaks.  Measurement helpers, not hot calls: they allocate their own device
 * memory, run on the null stream, synchronise the device and free everything
 * before they return.  `reps` in [1, 1000] timed launches after one untimed.
 *
 * ecoserve_probe_hbm_read: reads a buffer of `bytes` (a multiple of 8192, at
 *   least 1 MiB; use more than the 256 MiB last-level cache, e.g. 4 GiB) once
 *   per launch, each wavefront taking whole 8 KiB pieces with coalesced
 *   16-byte non-temporal loads (the fastest read pattern known to this
 *   library, and the decode kernel's); *gb_per_s = bytes / mean launch time,
 *   in 1e9 B/s.
 *   ECOSERVE_ENOMEM if the buffer cannot be allocated.
 * ecoserve_probe_mfma_bf16: a register-only loop of 32x32x16 bf16 matrix
 *   instructions, four wavefronts per SIMD; `random_operands` != 0 feeds every
 *   accumulator chain its own pseudo-random operands (the chip then holds a
 *   lower clock under its power limit than with smooth ones);
 *   *tflop_per_s = FLOPs / mean launch time, in 1e12 FLOP/s.
 */
int ecoserve_probe_hbm_read(int device, size_t bytes, int32_t reps, double* gb_per_s);
int ecoserve_probe_mfma_bf16(int device, int32_t random_operands, int32_t reps, double* tflop_per_s);

/*
 * How much vector-ALU work the matrix cores of `device` hide (Section 2.1 counts only the
 * matrix FLOPs of attention, calling the softmax "a small fraction of the total execution time"; on this
 * chip the softmax's vector instructions decide how busy the matrix cores can be).  Every wavefront
 * runs slots of one 32x32x16 bf16 matrix instruction (if with_mfma != 0), fma_per_slot independent
 * v_fma_f32 and exp_per_slot independent v_exp_f32, register operands only, waves_per_simd (1 or 2)
 * wavefronts on every SIMD.  *clocks_per_slot = shader clocks one SIMD spends per slot (32 = the
 * matrix instruction alone; if the vector work were hidden the figure would stay there);
 * *ghz = the shader clock during the run.  (fma_per_slot, exp_per_slot) must be one of
 * (0,0) (2,0) (4,0) (8,0) (0,2) (2,2) (4,2), and not (0,0) without the matrix instruction:
 * else ECOSERVE_EINVAL.  Allocates, synchronises, frees: a measurement helper like the two above.
 */
int ecoserve_probe_mfma_valu(int device, int32_t with_mfma, int32_t fma_per_slot, int32_t exp_per_slot,
                             int32_t waves_per_simd, double* clocks_per_slot, double* ghz);

#ifdef __cplusplus
}
#endif
#endif /* ECOSERVE_H */
