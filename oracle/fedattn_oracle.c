/*
 * FedAttn attention oracle: plain, slow, fp64, CPU only.
 *
 * TEST INFRASTRUCTURE.  This file is the reference the GPU library is checked
 * against.  It shares no code with the GPU library and must never be called
 * from it; only the tests, the smoke check and the benchmark's CPU-baseline leg
 * use it.
 *
 * What it computes is the definition itself, one query row at a time:
 *   scores  S_j = scale * <q_i, k_j>           (Section III-B, scaled dot-product attention)
 *   weights p_j = exp(S_j - max) / sum         (row-wise softmax; every row is a distribution)
 *   output  o_i = sum_j p_j v_j                (value aggregation)
 * over the keys j that query i may see:
 *   causal:        j <= i                      (Section III-B causal mask, read as "a token
 *                                               attends to itself and to preceding tokens";
 *                                               the printed case condition has i and j
 *                                               swapped relative to the prose)
 *   local block:   j in the query's own segment          (Phase I, local self-attention)
 *   sync block:    j anywhere in the aggregated KV        (Phase II, global self-attention),
 *                  under the causal order of the global sequence
 *   sparse exchange: a remote j only if its row was sent  (adaptive KV aggregation:
 *                  unselected remote rows are absent from the global KV matrix;
 *                  a participant's own rows are always complete)
 * Multi-head / GQA: heads are independent, scale = 1/sqrt(head_dim) unless given,
 * query head h reads KV head floor(h / (Hq/Hkv)).
 *
 * Rows are independent, so the loop over requested rows runs under OpenMP; there
 * is no blocking, fusion or reordering inside a row.
 *
 * Inputs are float32 (bf16 workloads pass bf16-representable float32 values); the
 * upcast to double is exact.  Outputs are double, unrounded.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Algorithm 1: block m = H t + h (1-based) runs global attention iff h = H, i.e.
 * m mod H == 0.  With 0-based block_idx = m - 1: (block_idx + 1) mod H == 0.
 * H <= 0 means no block ever synchronises. */
int fedattn_oracle_is_sync(int32_t H, int32_t block_idx) {
  if (H <= 0) return 0;
  return ((block_idx + 1) % H) == 0;
}

int fedattn_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* participant that owns global token i: the n with seg_off[n] <= i < seg_off[n+1]
 * (index sets L_n are contiguous runs of the global sequence, Section IV-A). */
static int owner(const int32_t* seg_off, int N, int i) {
  for (int n = 0; n < N; ++n)
    if (i >= seg_off[n] && i < seg_off[n + 1]) return n;
  return -1;
}

/* May query i see key j? */
static int allowed(int i, int j, int seg_i, int seg_j, int is_sync, int causal,
                   const uint8_t* keep_tok) {
  if (causal && j > i) return 0;
  if (seg_i == seg_j) return 1;                 /* own rows: always complete */
  if (!is_sync) return 0;                       /* local block: nothing remote */
  if (keep_tok && !keep_tok[j]) return 0;       /* remote row not exchanged */
  return 1;
}

/*
 * Attention output for the requested (row, head) pairs of one block.
 *   q [total,Hq,D], k,v [total,Hkv,D] float32, token-major.
 *   seg_off [N+1]; keep_tok [total] or NULL (all kept).
 *   rows/heads [n_rows]; out [n_rows,D]; prob [n_rows,total] or NULL.
 * A row with no visible key yields zeros.
 */
void fedattn_oracle_attend_rows(const float* q, const float* k, const float* v,
                                int32_t total, int32_t Hq, int32_t Hkv, int32_t D,
                                const int32_t* seg_off, int32_t N, double scale,
                                int32_t is_sync, int32_t causal, const uint8_t* keep_tok,
                                const int32_t* rows, const int32_t* heads, int64_t n_rows,
                                double* out, double* prob) {
  const int group = Hq / Hkv;
  int* seg = (int*)malloc(sizeof(int) * (size_t)(total > 0 ? total : 1));
  for (int j = 0; j < total; ++j) seg[j] = owner(seg_off, N, j);

#pragma omp parallel
  {
    double* s = (double*)malloc(sizeof(double) * (size_t)(total > 0 ? total : 1));
#pragma omp for schedule(dynamic, 4)
    for (int64_t r = 0; r < n_rows; ++r) {
      const int i = rows[r], h = heads[r], g = h / group;
      const float* qi = q + ((size_t)i * Hq + h) * D;
      double* o = out + (size_t)r * D;
      double* pr = prob ? prob + (size_t)r * total : NULL;
      for (int d = 0; d < D; ++d) o[d] = 0.0;
      if (pr) for (int j = 0; j < total; ++j) pr[j] = 0.0;

      double mx = -INFINITY;
      int any = 0;
      for (int j = 0; j < total; ++j) {
        if (!allowed(i, j, seg[i], seg[j], is_sync, causal, keep_tok)) continue;
        const float* kj = k + ((size_t)j * Hkv + g) * D;
        double acc = 0.0;
        for (int d = 0; d < D; ++d) acc += (double)qi[d] * (double)kj[d];
        s[j] = scale * acc;
        if (s[j] > mx) mx = s[j];
        any = 1;
      }
      if (!any) continue;
      double denom = 0.0;
      for (int j = 0; j < total; ++j) {
        if (!allowed(i, j, seg[i], seg[j], is_sync, causal, keep_tok)) continue;
        s[j] = exp(s[j] - mx);
        denom += s[j];
      }
      for (int j = 0; j < total; ++j) {
        if (!allowed(i, j, seg[i], seg[j], is_sync, causal, keep_tok)) continue;
        const double p = s[j] / denom;
        if (pr) pr[j] = p;
        const float* vj = v + ((size_t)j * Hkv + g) * D;
        for (int d = 0; d < D; ++d) o[d] += p * (double)vj[d];
      }
    }
    free(s);
  }
  free(seg);
}

/*
 * One decoding step of one block (Section IV-C: blocks that ran local attention
 * kept the local KV cache, blocks that ran global attention kept the global one,
 * and decoding reuses them).  One query per participant; the step's own k,v are
 * already the last valid cache row, so the query sees itself.
 *   q [N,Hq,D]; k_cache,v_cache [capacity_total,Hkv,D];
 *   seg_off [N+1] = capacity layout; seg_lens [N] = valid rows per segment;
 *   remote_lens [N] or NULL (= seg_lens): rows of segment m visible to the
 *   queries of participants other than m in a sync block.
 *   out [N,Hq,D].  Everything cached is in the past, so there is no further mask.
 */
void fedattn_oracle_decode(const float* q, const float* k_cache, const float* v_cache,
                           int32_t N, int32_t Hq, int32_t Hkv, int32_t D,
                           const int32_t* seg_off, const int32_t* seg_lens,
                           const int32_t* remote_lens, double scale, int32_t is_sync,
                           double* out) {
  const int group = Hq / Hkv;
  const int cap = seg_off[N];
#pragma omp parallel
  {
    double* s = (double*)malloc(sizeof(double) * (size_t)(cap > 0 ? cap : 1));
    uint8_t* vis = (uint8_t*)malloc((size_t)(cap > 0 ? cap : 1));
#pragma omp for schedule(dynamic, 1) collapse(2)
    for (int n = 0; n < N; ++n) {
      for (int h = 0; h < Hq; ++h) {
        const int g = h / group;
        const float* qn = q + ((size_t)n * Hq + h) * D;
        double* o = out + ((size_t)n * Hq + h) * D;
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        /* visible rows of the cache for participant n */
        memset(vis, 0, (size_t)(cap > 0 ? cap : 1));
        for (int m = 0; m < N; ++m) {
          int len;
          if (m == n) len = seg_lens[m];
          else if (!is_sync) len = 0;
          else len = remote_lens ? remote_lens[m] : seg_lens[m];
          for (int r = 0; r < len; ++r) vis[seg_off[m] + r] = 1;
        }
        double mx = -INFINITY;
        int any = 0;
        for (int j = 0; j < cap; ++j) {
          if (!vis[j]) continue;
          const float* kj = k_cache + ((size_t)j * Hkv + g) * D;
          double acc = 0.0;
          for (int d = 0; d < D; ++d) acc += (double)qn[d] * (double)kj[d];
          s[j] = scale * acc;
          if (s[j] > mx) mx = s[j];
          any = 1;
        }
        if (!any) continue;
        double denom = 0.0;
        for (int j = 0; j < cap; ++j)
          if (vis[j]) { s[j] = exp(s[j] - mx); denom += s[j]; }
        for (int j = 0; j < cap; ++j) {
          if (!vis[j]) continue;
          const double p = s[j] / denom;
          const float* vj = v_cache + ((size_t)j * Hkv + g) * D;
          for (int d = 0; d < D; ++d) o[d] += p * (double)vj[d];
        }
      }
    }
    free(s);
    free(vis);
  }
}
