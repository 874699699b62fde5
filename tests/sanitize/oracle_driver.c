/* Runs the C oracle (oracle/ecoserve_oracle.c, compiled into this program with
 * -fsanitize=address,undefined) over small seeded batches that touch every entry point and the ragged
 * cases: zero-length sequences, cached prefixes, blocks filled to the last slot, fp32 and bf16 storage.
 * Checks only that every call succeeds and every output is finite; the sanitizers check the rest. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_num_threads(void);
int oracle_kv_append(void *k_cache, void *v_cache, const void *k_new, const void *v_new, const int32_t *cu_q,
                     const int32_t *ctx_before, const int32_t *block_table, int32_t bt_stride, int32_t B, int32_t Hkv,
                     int32_t D, int32_t bs, int32_t num_blocks, int32_t dtype);
int oracle_attn_prefill(const void *q, const void *k_cache, const void *v_cache, const int32_t *cu_q,
                        const int32_t *ctx_before, const int32_t *block_table, int32_t bt_stride, int32_t B, int32_t Hq,
                        int32_t Hkv, int32_t D, int32_t bs, int32_t num_blocks, int32_t dtype, double scale, double *out,
                        double *lse);
int oracle_attn_decode(const void *q, const void *k_cache, const void *v_cache, const int32_t *block_table,
                       int32_t bt_stride, const int32_t *ctx_len, int32_t B, int32_t Hq, int32_t Hkv, int32_t D,
                       int32_t bs, int32_t num_blocks, int32_t dtype, double scale, double *out, double *lse);

static uint32_t rng_state = 12345u;
static uint32_t rnd(void) {
  rng_state = rng_state * 1664525u + 1013904223u;
  return rng_state >> 8;
}
static float rnd_unit(void) { return (float)(rnd() % 20001) / 10000.0f - 1.0f; }

static void fill(void *dst, size_t n, int dtype) {
  for (size_t i = 0; i < n; ++i) {
    const float f = rnd_unit();
    if (dtype == 0) {
      uint32_t u;
      memcpy(&u, &f, 4);
      ((uint16_t *)dst)[i] = (uint16_t)(u >> 16);
    } else {
      ((float *)dst)[i] = f;
    }
  }
}

static int run_case(int dtype, int Hq, int Hkv, int D, const int *first, const int *second, int B) {
  const int bs = 16;
  const size_t es = dtype == 0 ? 2 : 4;
  int total_blocks = 0, stride = 0;
  for (int b = 0; b < B; ++b) {
    const int nb = (first[b] + second[b] + 1 + bs - 1) / bs;
    total_blocks += nb;
    if (nb > stride) stride = nb;
  }
  const int num_blocks = total_blocks + 3;
  int32_t *table = malloc(sizeof(int32_t) * (size_t)B * stride);
  int next = num_blocks - 1;  /* hand the blocks out from the top: logical and physical order differ */
  for (int b = 0; b < B; ++b)
    for (int j = 0; j < stride; ++j) table[b * stride + j] = j < (first[b] + second[b] + 1 + bs - 1) / bs ? next-- : -1;
  const size_t pool = (size_t)num_blocks * Hkv * bs * D;
  void *kc = calloc(pool, es), *vc = calloc(pool, es);
  int rc = 0;
  int32_t *cu = malloc(sizeof(int32_t) * (B + 1)), *before = malloc(sizeof(int32_t) * B), *len = malloc(sizeof(int32_t) * B);
  for (int round = 0; round < 2 && !rc; ++round) {  /* a first chunk, then a second one behind it */
    const int *n_new = round == 0 ? first : second;
    cu[0] = 0;
    for (int b = 0; b < B; ++b) {
      cu[b + 1] = cu[b] + n_new[b];
      before[b] = round == 0 ? 0 : first[b];
    }
    const int T = cu[B];
    void *kn = malloc((size_t)(T ? T : 1) * Hkv * D * es), *vn = malloc((size_t)(T ? T : 1) * Hkv * D * es);
    void *q = malloc((size_t)(T ? T : 1) * Hq * D * es);
    fill(kn, (size_t)T * Hkv * D, dtype);
    fill(vn, (size_t)T * Hkv * D, dtype);
    fill(q, (size_t)T * Hq * D, dtype);
    double *out = malloc(sizeof(double) * (size_t)(T ? T : 1) * Hq * D), *lse = malloc(sizeof(double) * (size_t)(T ? T : 1) * Hq);
    rc = oracle_kv_append(kc, vc, kn, vn, cu, before, table, stride, B, Hkv, D, bs, num_blocks, dtype);
    if (!rc) rc = oracle_attn_prefill(q, kc, vc, cu, before, table, stride, B, Hq, Hkv, D, bs, num_blocks, dtype,
                                     1.0 / sqrt((double)D), out, lse);
    for (size_t i = 0; !rc && i < (size_t)T * Hq * D; ++i)
      if (!isfinite(out[i])) rc = 100;
    free(kn); free(vn); free(q); free(out); free(lse);
  }
  if (!rc) {  /* one decode step for the sequences that hold tokens */
    int Bd = 0;
    for (int b = 0; b < B; ++b) cu[b + 1] = cu[b] = 0;
    int32_t *rows = malloc(sizeof(int32_t) * (size_t)B * stride);
    for (int b = 0; b < B; ++b)
      if (first[b] + second[b] > 0) {
        memcpy(rows + (size_t)Bd * stride, table + (size_t)b * stride, sizeof(int32_t) * stride);
        before[Bd] = first[b] + second[b];
        len[Bd] = before[Bd] + 1;
        ++Bd;
      }
    for (int b = 0; b <= Bd; ++b) cu[b] = b;
    void *kn = malloc((size_t)(Bd ? Bd : 1) * Hkv * D * es), *vn = malloc((size_t)(Bd ? Bd : 1) * Hkv * D * es);
    void *q = malloc((size_t)(Bd ? Bd : 1) * Hq * D * es);
    fill(kn, (size_t)Bd * Hkv * D, dtype);
    fill(vn, (size_t)Bd * Hkv * D, dtype);
    fill(q, (size_t)Bd * Hq * D, dtype);
    double *out = malloc(sizeof(double) * (size_t)(Bd ? Bd : 1) * Hq * D), *lse = malloc(sizeof(double) * (size_t)(Bd ? Bd : 1) * Hq);
    rc = oracle_kv_append(kc, vc, kn, vn, cu, before, rows, stride, Bd, Hkv, D, bs, num_blocks, dtype);
    if (!rc) rc = oracle_attn_decode(q, kc, vc, rows, stride, len, Bd, Hq, Hkv, D, bs, num_blocks, dtype,
                                    1.0 / sqrt((double)D), out, lse);
    for (size_t i = 0; !rc && i < (size_t)Bd * Hq * D; ++i)
      if (!isfinite(out[i])) rc = 101;
    free(kn); free(vn); free(q); free(out); free(lse); free(rows);
  }
  free(table); free(kc); free(vc); free(cu); free(before); free(len);
  return rc;
}

int main(void) {
  const int first[] = {37, 0, 16, 1, 100, 15, 64}, second[] = {11, 5, 0, 31, 28, 1, 0};
  int rc = oracle_num_threads() >= 1 ? 0 : 1;
  if (!rc) rc = run_case(1, 4, 2, 64, first, second, 7);    /* fp32, the tiny configuration's heads */
  if (!rc) rc = run_case(0, 10, 2, 128, first, second, 7);  /* bf16, group size 5 */
  if (!rc) rc = run_case(0, 3, 3, 24, first, second, 7);    /* no K/V sharing, an odd head size */
  /* errors are reported, not crashed on: a table entry outside the pool */
  {
    int32_t table[1] = {7}, cu[2] = {0, 1}, before[1] = {0};
    uint16_t kc[16 * 8] = {0}, vc[16 * 8] = {0}, kn[8] = {0};
    if (!rc && oracle_kv_append(kc, vc, kn, kn, cu, before, table, 1, 1, 1, 8, 16, 1, 0) == 0) rc = 102;
  }
  printf(rc ? "oracle driver FAILED (%d)\n" : "oracle driver ok\n", rc);
  return rc;
}
