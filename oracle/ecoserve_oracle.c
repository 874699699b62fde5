/*
 * ecoserve_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, fp64 CPU statement of what the paged-attention hot path
 * computes.  Only the tests, the smoke check and the benchmark's
 * "cpu_baseline" leg may call it; the GPU library never does and shares no
 * code, header, table or helper with this file.
 *
 * What it follows (EcoServe, arXiv 2504.18154):
 *   - Section 2.1, Eq. 2: Attention(Q,K,V) = softmax(Q K^T / sqrt(d_k)) V,
 *     with d_k = the per-head size D of Table 1.
 *   - Section 2.1, first paragraph: generation is autoregressive over the
 *     accumulated context, and the key/value embeddings of earlier tokens
 *     are kept in memory (the KV cache) and reused.  Hence a query token at
 *     absolute position p sees exactly the keys 0..p of its own sequence.
 *   - Section 4.1 (model setup): grouped-query attention shares one K/V head
 *     among several query heads.  Reading taken here: query head h uses
 *     K/V head h div (Hq/Hkv).
 *   - Section 5 (KV cache management): the cache is organised in fixed-size
 *     blocks; a per-sequence block table maps logical block j of the
 *     sequence to a physical block of the pool.
 *
 * The method (tiling, online softmax, split context, paging) reaches the
 * plain definition exactly up to rounding order, so the oracle IS the
 * definition: gather the sequence's keys and values through the block
 * table, form all scores, subtract the maximum, exponentiate, normalise,
 * take the weighted sum of values.  Two passes, no blocking, no fusion.
 *
 * Storage types: inputs arrive in the bit patterns the GPU gets (bf16 as
 * uint16, or fp32) and are widened exactly to double before any arithmetic.
 * All arithmetic is double.
 *
 * Logical cache view used here: cache[num_blocks][Hkv][bs][D], one array for
 * K and one for V.  (This is the oracle's own container; how the GPU library
 * orders the bytes of a block is its business and is compared through a
 * logical view in the tests.)
 *
 * Parity pins (tests, CPU only): dense brute force written independently in
 * NumPy, a library SDPA routine on the case that reduces to it, the closed
 * forms for a single-token context and for equal keys, rows of the weight
 * matrix summing to one, and invariance under re-drawing the physical block
 * permutation.  No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_BF16 = 0, ORACLE_F32 = 1 };

enum {
  ORACLE_OK = 0,
  ORACLE_EINVAL = 1,  /* bad shapes / unsupported dtype */
  ORACLE_ERANGE = 2,  /* a block-table entry or position outside the pool */
  ORACLE_ENOMEM = 3
};

static size_t elem_size(int dtype) { return dtype == ORACLE_BF16 ? 2u : 4u; }

/* Exact widening of one stored element to double. */
static double widen(const void *base, size_t idx, int dtype) {
  if (dtype == ORACLE_BF16) {
    uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
  }
  return (double)((const float *)base)[idx];
}

/* Element index of (blk, g, slot, d) in the logical cache view. */
static size_t cache_index(int64_t blk, int g, int slot, int d, int Hkv, int bs,
                          int D) {
  return ((((size_t)blk * (size_t)Hkv + (size_t)g) * (size_t)bs + (size_t)slot) *
          (size_t)D) + (size_t)d;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/*
 * KV-cache append (Section 2.1: the key and value embeddings of processed
 * tokens are kept in memory for later steps; Section 5: fixed-size blocks).
 *
 * New token i of sequence b lands at absolute position p = ctx_before[b] + i,
 * i.e. in physical block block_table[b][p div bs], slot p mod bs.  The copy is
 * a byte copy of the stored elements, so it is exact by construction.
 *
 *   k_cache, v_cache : [num_blocks][Hkv][bs][D] in the storage dtype (in/out)
 *   k_new, v_new     : [T][Hkv][D], sequences packed back to back
 *   cu_q             : [B+1] prefix sums of new-token counts, cu_q[0] = 0
 *   ctx_before       : [B] tokens of the sequence already in the cache
 *   block_table      : [B][bt_stride] physical block ids
 */
int oracle_kv_append(void *k_cache, void *v_cache, const void *k_new,
                     const void *v_new, const int32_t *cu_q,
                     const int32_t *ctx_before, const int32_t *block_table,
                     int32_t bt_stride, int32_t B, int32_t Hkv, int32_t D,
                     int32_t bs, int32_t num_blocks, int32_t dtype) {
  if (B < 0 || Hkv <= 0 || D <= 0 || bs <= 0 || num_blocks < 0) return ORACLE_EINVAL;
  if (dtype != ORACLE_BF16 && dtype != ORACLE_F32) return ORACLE_EINVAL;
  const size_t es = elem_size(dtype);
  for (int b = 0; b < B; ++b) {
    const int S = cu_q[b + 1] - cu_q[b];
    if (S < 0 || ctx_before[b] < 0) return ORACLE_EINVAL;
    for (int i = 0; i < S; ++i) {
      const int p = ctx_before[b] + i;
      const int j = p / bs;
      const int slot = p % bs;
      if (j >= bt_stride) return ORACLE_ERANGE;
      const int64_t blk = block_table[(size_t)b * (size_t)bt_stride + (size_t)j];
      if (blk < 0 || blk >= num_blocks) return ORACLE_ERANGE;
      const size_t t = (size_t)cu_q[b] + (size_t)i;
      for (int g = 0; g < Hkv; ++g) {
        const size_t src = (t * (size_t)Hkv + (size_t)g) * (size_t)D;
        const size_t dst = cache_index(blk, g, slot, 0, Hkv, bs, D);
        memcpy((char *)k_cache + dst * es, (const char *)k_new + src * es, (size_t)D * es);
        memcpy((char *)v_cache + dst * es, (const char *)v_new + src * es, (size_t)D * es);
      }
    }
  }
  return ORACLE_OK;
}

/*
 * Gather the first L keys (or values) of sequence b, K/V head g, through the
 * block table into a dense double array dst[L][D]  (Section 5: block-table
 * indirection; Section 2.1: the cache holds the sequence's K and V).
 */
static int gather_dense(double *dst, const void *cache, const int32_t *bt_row,
                        int32_t bt_stride, int L, int g, int Hkv, int D, int bs,
                        int num_blocks, int dtype) {
  for (int j = 0; j < L; ++j) {
    const int lb = j / bs;
    if (lb >= bt_stride) return ORACLE_ERANGE;
    const int64_t blk = bt_row[lb];
    if (blk < 0 || blk >= num_blocks) return ORACLE_ERANGE;
    const size_t base = cache_index(blk, g, j % bs, 0, Hkv, bs, D);
    for (int d = 0; d < D; ++d) dst[(size_t)j * (size_t)D + (size_t)d] = widen(cache, base + (size_t)d, dtype);
  }
  return ORACLE_OK;
}

/*
 * Eq. 2 for one query vector against keys/values 0..p (inclusive):
 *   s_j = scale * <q, K_j>;  m = max_j s_j;  w_j = exp(s_j - m);
 *   Z = sum_j w_j;  P_j = w_j / Z;  o = sum_j P_j V_j;  lse = m + log Z.
 * scratch holds p+1 doubles.  If probs != NULL the weights P_j are stored.
 */
static void attend_one(const double *qv, const double *Kd, const double *Vd,
                       int p, int D, double scale, double *scratch,
                       double *o, double *lse, double *probs) {
  const int n = p + 1;
  double m = -INFINITY;
  for (int j = 0; j < n; ++j) {
    double acc = 0.0;
    const double *kj = Kd + (size_t)j * (size_t)D;
    for (int d = 0; d < D; ++d) acc += qv[d] * kj[d];
    scratch[j] = scale * acc;
    if (scratch[j] > m) m = scratch[j];
  }
  double Z = 0.0;
  for (int j = 0; j < n; ++j) {
    scratch[j] = exp(scratch[j] - m);
    Z += scratch[j];
  }
  for (int d = 0; d < D; ++d) o[d] = 0.0;
  for (int j = 0; j < n; ++j) {
    const double Pj = scratch[j] / Z;
    if (probs) probs[j] = Pj;
    const double *vj = Vd + (size_t)j * (size_t)D;
    for (int d = 0; d < D; ++d) o[d] += Pj * vj[d];
  }
  if (lse) *lse = m + log(Z);
}

/*
 * Attention for a list of query rows (the general form; prefill and decode
 * below are thin callers).
 *
 * Row r belongs to sequence row_seq[r], takes its query vector from token
 * row_tok[r] of q ([n_q_tokens][Hq][D]) and sits at absolute position
 * row_pos[r] of its sequence, so it attends to keys 0..row_pos[r]
 * (Section 2.1: next-token prediction over the accumulated context).
 * Rows must be grouped by sequence: rows of sequence b are
 * seq_row_start[b] .. seq_row_start[b+1]-1.
 *
 *   out   : [R][Hq][D] double
 *   lse   : [R][Hq] double, or NULL
 *   probs : [R][Hq][probs_stride] double (weights P_j, zero beyond p), or NULL
 *   scale : 1/sqrt(D) for Eq. 2; passed in so tests can vary it
 */
int oracle_attn_rows(const void *q, const void *k_cache, const void *v_cache,
                     const int32_t *block_table, int32_t bt_stride,
                     const int32_t *seq_row_start, const int32_t *row_tok,
                     const int32_t *row_pos, int32_t B, int32_t Hq, int32_t Hkv,
                     int32_t D, int32_t bs, int32_t num_blocks, int32_t dtype,
                     double scale, double *out, double *lse, double *probs,
                     int32_t probs_stride) {
  if (B < 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || bs <= 0) return ORACLE_EINVAL;
  if (Hq % Hkv != 0) return ORACLE_EINVAL;
  if (dtype != ORACLE_BF16 && dtype != ORACLE_F32) return ORACLE_EINVAL;
  const int G = Hq / Hkv;
  int status = ORACLE_OK;

#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b) {
    for (int g = 0; g < Hkv; ++g) {
      const int r0 = seq_row_start[b], r1 = seq_row_start[b + 1];
      if (r1 <= r0) continue;
      int pmax = -1;
      for (int r = r0; r < r1; ++r)
        if (row_pos[r] > pmax) pmax = row_pos[r];
      int bad = 0;
      for (int r = r0; r < r1; ++r)
        if (row_pos[r] < 0 || row_tok[r] < 0) bad = 1;
      if (bad || (probs && pmax >= probs_stride)) {
#pragma omp critical
        status = ORACLE_EINVAL;
        continue;
      }
      const int L = pmax + 1;
      double *Kd = (double *)malloc((size_t)L * (size_t)D * sizeof(double));
      double *Vd = (double *)malloc((size_t)L * (size_t)D * sizeof(double));
      double *scratch = (double *)malloc((size_t)L * sizeof(double));
      double *qv = (double *)malloc((size_t)D * sizeof(double));
      if (!Kd || !Vd || !scratch || !qv) {
#pragma omp critical
        status = ORACLE_ENOMEM;
        free(Kd); free(Vd); free(scratch); free(qv);
        continue;
      }
      const int32_t *bt_row = block_table + (size_t)b * (size_t)bt_stride;
      int rc = gather_dense(Kd, k_cache, bt_row, bt_stride, L, g, Hkv, D, bs, num_blocks, dtype);
      if (rc == ORACLE_OK)
        rc = gather_dense(Vd, v_cache, bt_row, bt_stride, L, g, Hkv, D, bs, num_blocks, dtype);
      if (rc != ORACLE_OK) {
#pragma omp critical
        status = rc;
      } else {
        for (int r = r0; r < r1; ++r) {
          for (int hh = 0; hh < G; ++hh) {
            const int h = g * G + hh;  /* GQA: query head h reads K/V head h div G */
            const size_t qbase = ((size_t)row_tok[r] * (size_t)Hq + (size_t)h) * (size_t)D;
            for (int d = 0; d < D; ++d) qv[d] = widen(q, qbase + (size_t)d, dtype);
            const size_t obase = ((size_t)r * (size_t)Hq + (size_t)h);
            double *pr = probs ? probs + obase * (size_t)probs_stride : NULL;
            if (pr) memset(pr, 0, (size_t)probs_stride * sizeof(double));
            attend_one(qv, Kd, Vd, row_pos[r], D, scale, scratch,
                       out + obase * (size_t)D, lse ? lse + obase : NULL, pr);
          }
        }
      }
      free(Kd); free(Vd); free(scratch); free(qv);
    }
  }
  return status;
}

/*
 * Prefill attention (Section 2.1: the prefill phase processes all prompt
 * tokens at once).  The K/V of the new tokens must already be in the cache.
 * New token i of sequence b is at absolute position ctx_before[b] + i and
 * attends causally to keys 0..ctx_before[b]+i.
 *
 *   q   : [T][Hq][D] packed by sequence (cu_q as in oracle_kv_append)
 *   out : [T][Hq][D] double;  lse : [T][Hq] double or NULL
 */
int oracle_attn_prefill(const void *q, const void *k_cache, const void *v_cache,
                        const int32_t *cu_q, const int32_t *ctx_before,
                        const int32_t *block_table, int32_t bt_stride, int32_t B,
                        int32_t Hq, int32_t Hkv, int32_t D, int32_t bs,
                        int32_t num_blocks, int32_t dtype, double scale,
                        double *out, double *lse) {
  if (B < 0) return ORACLE_EINVAL;
  const int T = B > 0 ? cu_q[B] : 0;
  int32_t *tok = (int32_t *)malloc(((size_t)T + 1) * sizeof(int32_t));
  int32_t *pos = (int32_t *)malloc(((size_t)T + 1) * sizeof(int32_t));
  if (!tok || !pos) { free(tok); free(pos); return ORACLE_ENOMEM; }
  for (int b = 0; b < B; ++b)
    for (int t = cu_q[b]; t < cu_q[b + 1]; ++t) {
      tok[t] = t;
      pos[t] = ctx_before[b] + (t - cu_q[b]);
    }
  /* rows == tokens, already grouped by sequence: seq_row_start == cu_q */
  int rc = oracle_attn_rows(q, k_cache, v_cache, block_table, bt_stride, cu_q, tok,
                            pos, B, Hq, Hkv, D, bs, num_blocks, dtype, scale, out,
                            lse, NULL, 0);
  free(tok); free(pos);
  return rc;
}

/*
 * Decode attention (Section 2.1: each decode step produces one token per
 * sequence from the accumulated context).  The new token's K/V has already
 * been appended, ctx_len[b] counts it, and its query sits at position
 * ctx_len[b]-1, so it also attends to itself.
 *
 *   q   : [B][Hq][D];  out : [B][Hq][D] double;  lse : [B][Hq] double or NULL
 */
int oracle_attn_decode(const void *q, const void *k_cache, const void *v_cache,
                       const int32_t *block_table, int32_t bt_stride,
                       const int32_t *ctx_len, int32_t B, int32_t Hq, int32_t Hkv,
                       int32_t D, int32_t bs, int32_t num_blocks, int32_t dtype,
                       double scale, double *out, double *lse) {
  if (B < 0) return ORACLE_EINVAL;
  int32_t *start = (int32_t *)malloc(((size_t)B + 1) * sizeof(int32_t));
  int32_t *tok = (int32_t *)malloc(((size_t)B + 1) * sizeof(int32_t));
  int32_t *pos = (int32_t *)malloc(((size_t)B + 1) * sizeof(int32_t));
  if (!start || !tok || !pos) { free(start); free(tok); free(pos); return ORACLE_ENOMEM; }
  int rc = ORACLE_OK;
  for (int b = 0; b < B; ++b) {
    start[b] = b;
    tok[b] = b;
    pos[b] = ctx_len[b] - 1;
    if (ctx_len[b] < 1) rc = ORACLE_EINVAL;  /* an empty context has no softmax */
  }
  start[B] = B;
  if (rc == ORACLE_OK)
    rc = oracle_attn_rows(q, k_cache, v_cache, block_table, bt_stride, start, tok,
                          pos, B, Hq, Hkv, D, bs, num_blocks, dtype, scale, out, lse,
                          NULL, 0);
  free(start); free(tok); free(pos);
  return rc;
}
