/* Driver for the AddressSanitizer / UndefinedBehaviorSanitizer build of the CPU oracle
 * (oracle/fedattn_oracle.c): runs every entry point on small exact-size heap buffers - ragged
 * and empty segments, keep-lists, empty caches, both decode readings - so that any access
 * outside a buffer or any undefined operation aborts the program.  Exit status 0 = clean. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int fedattn_oracle_is_sync(int32_t H, int32_t block_idx);
int fedattn_oracle_threads(void);
void fedattn_oracle_attend_rows(const float* q, const float* k, const float* v, int32_t total, int32_t Hq, int32_t Hkv,
                                int32_t D, const int32_t* seg_off, int32_t N, double scale, int32_t is_sync,
                                int32_t causal, const uint8_t* keep_tok, const int32_t* rows, const int32_t* heads,
                                int64_t n_rows, double* out, double* prob);
void fedattn_oracle_decode(const float* q, const float* k_cache, const float* v_cache, int32_t N, int32_t Hq, int32_t Hkv,
                           int32_t D, const int32_t* seg_off, const int32_t* seg_lens, const int32_t* remote_lens,
                           double scale, int32_t is_sync, double* out);

static float* randf(size_t n, unsigned* state) {
  float* p = (float*)malloc(sizeof(float) * (n ? n : 1));
  for (size_t i = 0; i < n; ++i) {
    *state = *state * 1664525u + 1013904223u;
    p[i] = (float)((*state >> 8) & 0xffff) / 32768.0f - 1.0f;
  }
  return p;
}

static int finite_all(const double* x, size_t n) {
  for (size_t i = 0; i < n; ++i)
    if (!isfinite(x[i])) return 0;
  return 1;
}

int main(void) {
  unsigned st = 12345u;
  int bad = 0;
  if (fedattn_oracle_is_sync(4, 3) != 1 || fedattn_oracle_is_sync(4, 4) != 0 || fedattn_oracle_is_sync(0, 7) != 0) bad = 1;
  if (fedattn_oracle_is_sync(-3, 2) != 0 || fedattn_oracle_threads() < 1) bad = 1;

  /* prefill: 4 participants, one empty, ragged lengths */
  const int32_t seg[5] = {0, 7, 7, 20, 33};
  const int total = 33, Hq = 4, Hkv = 2, D = 8, N = 4;
  float *q = randf((size_t)total * Hq * D, &st), *k = randf((size_t)total * Hkv * D, &st), *v = randf((size_t)total * Hkv * D, &st);
  uint8_t* keep = (uint8_t*)malloc(total);
  for (int i = 0; i < total; ++i) keep[i] = (uint8_t)(i % 3 == 0);
  const int n_rows = total * Hq;
  int32_t* rows = (int32_t*)malloc(sizeof(int32_t) * n_rows);
  int32_t* heads = (int32_t*)malloc(sizeof(int32_t) * n_rows);
  for (int i = 0; i < n_rows; ++i) { rows[i] = i / Hq; heads[i] = i % Hq; }
  double* out = (double*)malloc(sizeof(double) * (size_t)n_rows * D);
  double* prob = (double*)malloc(sizeof(double) * (size_t)n_rows * total);
  for (int sync = 0; sync < 2; ++sync)
    for (int causal = 0; causal < 2; ++causal)
      for (int with_keep = 0; with_keep < 2; ++with_keep)
        for (int with_prob = 0; with_prob < 2; ++with_prob) {
          fedattn_oracle_attend_rows(q, k, v, total, Hq, Hkv, D, seg, N, 0.35, sync, causal, with_keep ? keep : NULL, rows,
                                     heads, n_rows, out, with_prob ? prob : NULL);
          if (!finite_all(out, (size_t)n_rows * D)) bad = 1;
          if (with_prob) {
            for (int r = 0; r < n_rows; ++r) {   /* probability rows sum to one */
              double s = 0;
              for (int j = 0; j < total; ++j) s += prob[(size_t)r * total + j];
              if (fabs(s - 1.0) > 1e-12) bad = 1;
            }
          }
        }
  /* no rows requested, and a problem without tokens */
  fedattn_oracle_attend_rows(q, k, v, total, Hq, Hkv, D, seg, N, 0.35, 1, 1, NULL, rows, heads, 0, out, NULL);
  const int32_t seg0[2] = {0, 0};
  fedattn_oracle_attend_rows(q, k, v, 0, Hq, Hkv, D, seg0, 1, 0.35, 1, 1, NULL, rows, heads, 0, out, NULL);

  /* decode: capacity layout with an empty cache, both readings of the remote rows */
  const int32_t cap[5] = {0, 10, 20, 30, 33};
  const int32_t lens[4] = {10, 0, 4, 3};
  const int32_t remote[4] = {6, 0, 4, 1};
  float* qd = randf((size_t)N * Hq * D, &st);
  double* od = (double*)malloc(sizeof(double) * (size_t)N * Hq * D);
  for (int sync = 0; sync < 2; ++sync) {
    fedattn_oracle_decode(qd, k, v, N, Hq, Hkv, D, cap, lens, NULL, 0.35, sync, od);
    if (!finite_all(od, (size_t)N * Hq * D)) bad = 1;
    fedattn_oracle_decode(qd, k, v, N, Hq, Hkv, D, cap, lens, remote, 0.35, sync, od);
    if (!finite_all(od, (size_t)N * Hq * D)) bad = 1;
  }
  free(q); free(k); free(v); free(keep); free(rows); free(heads); free(out); free(prob); free(qd); free(od);
  if (bad) { fprintf(stderr, "oracle driver: a check failed\n"); return 1; }
  printf("oracle driver: clean\n");
  return 0;
}
