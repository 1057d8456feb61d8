/*
 * CPU oracle for the decode path of PQ-based KV-cache retrieval.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * GPU library must compute.  It shares no code, header, table or helper with the
 * HIP sources; only tests, the smoke check and the benchmark's CPU-baseline leg
 * may load it.  Everything is written as the definition reads: one loop nest per
 * formula, no blocking, no tables, no fusion.
 *
 * Notation (paper, Table "Notations" and Section 3.1): B sequences, Hq query
 * heads, Hkv key/value heads, G = Hq/Hkv, D = d_h, N cached tokens, M partitions,
 * C = 2^b centroids per partition, Dm = D/M.  I / L are the sizes of the always
 * kept initial and local windows, K the number of retrieved middle tokens.
 *
 * Layouts (all row-major, host memory):
 *   q          [B][Hq][D]          f32 or bf16 bits (uint16)
 *   k, v       [B][Hkv][N][D]      same type as q
 *   centroids  [B][Hkv][M][C][Dm]  f32
 *   codes      [B][Hkv][N][M]      uint8
 *
 * Pins (tests/test_oracle_*.py): scores against exact q.k when every token is its
 * own centroid, against a numpy reconstruction of the quantised keys, against a
 * hand-worked example; selection against numpy sorting and a quadratic brute
 * force; attention against dense numpy softmax when every token is selected and
 * against closed forms; K-Means against brute-force argmin / member means /
 * monotone inertia.  No function here is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { PQO_F32 = 0, PQO_BF16 = 1 };

int pqo_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Value of element i of a stored tensor; bf16 widens exactly to float. */
static float elem(const void* base, int dtype, int64_t i) {
  if (dtype == PQO_F32) return ((const float*)base)[i];
  uint32_t bits = (uint32_t)((const uint16_t*)base)[i] << 16;
  float f;
  memcpy(&f, &bits, 4);
  return f;
}

/* ------------------------------------------------------------------ K-Means
 * Section 2.2 / Section 3.1 step 2: every partition of the per-head keys is
 * clustered on its own into C centroids; a token's code is the index of the
 * cluster it belongs to.  Lloyd iterations, fixed count, squared L2 distance,
 * lowest index wins ties, an empty cluster keeps its centroid.  The starting
 * centroids are the sub-vectors at init_idx (drawn by the caller).
 *
 *   x        [n][dm] f32      cent  [c][dm] f32 (out)     codes [n] uint8 (out)
 *   inertia  [iters+1] (out): sum of squared distances at each assignment; the
 *            last entry belongs to the returned codes and centroids.
 */
static void assign_all(const float* x, int64_t n, int dm, int c, const float* cent,
                       uint8_t* codes, double* dist_out) {
#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < n; ++t) {
    double best = INFINITY;
    int arg = 0;
    for (int a = 0; a < c; ++a) {
      double d2 = 0.0;
#pragma omp simd reduction(+ : d2)
      for (int e = 0; e < dm; ++e) {
        double diff = (double)x[t * dm + e] - (double)cent[a * dm + e];
        d2 += diff * diff;
      }
      if (d2 < best) {
        best = d2;
        arg = a;
      }
    }
    codes[t] = (uint8_t)arg;
    dist_out[t] = best;
  }
}

int pqo_kmeans(const float* x, int64_t n, int dm, int c, int iters, const int32_t* init_idx,
               float* cent, uint8_t* codes, double* inertia) {
  if (n <= 0 || dm <= 0 || c <= 0 || c > 256 || iters < 0) return -1;
  double* dist = (double*)malloc(sizeof(double) * (size_t)n);
  double* sum = (double*)malloc(sizeof(double) * (size_t)c * dm);
  int64_t* cnt = (int64_t*)malloc(sizeof(int64_t) * (size_t)c);
  if (!dist || !sum || !cnt) return -2;
  for (int a = 0; a < c; ++a)
    for (int e = 0; e < dm; ++e) cent[a * dm + e] = x[(int64_t)init_idx[a] * dm + e];
  for (int it = 0;; ++it) {
    assign_all(x, n, dm, c, cent, codes, dist);
    double total = 0.0;
    for (int64_t t = 0; t < n; ++t) total += dist[t];
    inertia[it] = total;
    if (it == iters) break;
    memset(sum, 0, sizeof(double) * (size_t)c * dm);
    memset(cnt, 0, sizeof(int64_t) * (size_t)c);
    for (int64_t t = 0; t < n; ++t) {
      cnt[codes[t]] += 1;
      for (int e = 0; e < dm; ++e) sum[codes[t] * dm + e] += (double)x[t * dm + e];
    }
    for (int a = 0; a < c; ++a)
      if (cnt[a] > 0)
        for (int e = 0; e < dm; ++e) cent[a * dm + e] = (float)(sum[a * dm + e] / (double)cnt[a]);
  }
  free(dist);
  free(sum);
  free(cnt);
  return 0;
}

/* PQ construction for a whole layer: one clustering per (sequence, KV head,
 * partition), Section 3.3 ("h_kv * m per layer per sample").
 *   init_idx [B][Hkv][M][C] int32      inertia [B][Hkv][M][iters+1]
 */
int pqo_pq_build(const void* keys, int dtype, int B, int Hkv, int64_t N, int D, int M, int C,
                 int iters, const int32_t* init_idx, float* centroids, uint8_t* codes,
                 double* inertia) {
  if (M <= 0 || D % M) return -1;
  int Dm = D / M;
  float* x = (float*)malloc(sizeof(float) * (size_t)N * Dm);
  uint8_t* cd = (uint8_t*)malloc((size_t)N);
  if (!x || !cd) return -2;
  for (int u = 0; u < B * Hkv; ++u)
    for (int j = 0; j < M; ++j) {
      for (int64_t t = 0; t < N; ++t)
        for (int e = 0; e < Dm; ++e) x[t * Dm + e] = elem(keys, dtype, ((int64_t)u * N + t) * D + j * Dm + e);
      int rc = pqo_kmeans(x, N, Dm, C, iters, init_idx + ((int64_t)u * M + j) * C,
                          centroids + ((int64_t)u * M + j) * C * Dm, cd,
                          inertia + ((int64_t)u * M + j) * (iters + 1));
      if (rc) return rc;
      for (int64_t t = 0; t < N; ++t) codes[((int64_t)u * N + t) * M + j] = cd[t];
    }
  free(x);
  free(cd);
  return 0;
}

/* Code of one new key per (sequence, KV head): nearest centroid in every partition
 * (Section 3.1, tokens leaving the local window; Algorithm 2 "PQArgNearest").
 *   key [B][Hkv][D]  ->  code [B][Hkv][M]
 */
int pqo_nearest_codes(const void* key, int dtype, const float* centroids, int B, int Hkv, int D,
                      int M, int C, uint8_t* code) {
  if (M <= 0 || D % M) return -1;
  int Dm = D / M;
  for (int u = 0; u < B * Hkv; ++u)
    for (int j = 0; j < M; ++j) {
      double best = INFINITY;
      int arg = 0;
      for (int a = 0; a < C; ++a) {
        double d2 = 0.0;
        for (int e = 0; e < Dm; ++e) {
          double diff = (double)elem(key, dtype, (int64_t)u * D + j * Dm + e) -
                        (double)centroids[(((int64_t)u * M + j) * C + a) * Dm + e];
          d2 += diff * diff;
        }
        if (d2 < best) {
          best = d2;
          arg = a;
        }
      }
      code[u * M + j] = (uint8_t)arg;
    }
  return 0;
}

/* ------------------------------------------------------- approximate scores
 * Section 2.2 (search) and Section 3.1 step 4: the query is cut into M
 * partitions, each partition is multiplied with the centroid the token's code
 * names, and the M products are added.  With grouped-query attention one
 * selection serves the G query heads that share a KV head; the group's score is
 * the sum of its heads' scores, i.e. the PQ score of the summed query.
 *
 * Brute force per token, no table.  Two results:
 *   score64  everything in double;
 *   score32  the fp32 evaluation whose order the GPU path reproduces, because a
 *            ranking decided in floating point must be decided in one precision
 *            on both sides:  qs[d] = ((q_0[d] + q_1[d]) + ...) over the group's
 *            heads in head order;  part_j = fma chain over e = 0..Dm-1 starting
 *            from 0;  score = ((part_0 + part_1) + part_2) + ...
 *   score32, score64: [B][Hkv][N]  (either may be NULL)
 */
int pqo_scores(const void* q, int dtype, const float* centroids, const uint8_t* codes, int B,
               int Hq, int Hkv, int64_t N, int D, int M, int C, float* score32, double* score64) {
  if (Hkv <= 0 || Hq % Hkv || M <= 0 || D % M || D > 1024) return -1;
  int G = Hq / Hkv, Dm = D / M;
#pragma omp parallel for schedule(static)
  for (int u = 0; u < B * Hkv; ++u) {
    int b = u / Hkv, g = u % Hkv;
    float qs32[1024];
    double qs64[1024];
    for (int d = 0; d < D; ++d) {
      float a32 = 0.0f;
      double a64 = 0.0;
      for (int h = 0; h < G; ++h) {
        float qv = elem(q, dtype, ((int64_t)b * Hq + g * G + h) * D + d);
        a32 = (h == 0) ? qv : a32 + qv;
        a64 += (double)qv;
      }
      qs32[d] = a32;
      qs64[d] = a64;
    }
    for (int64_t t = 0; t < N; ++t) {
      float s32 = 0.0f;
      double s64 = 0.0;
      for (int j = 0; j < M; ++j) {
        int code = codes[((int64_t)u * N + t) * M + j];
        const float* cv = centroids + (((int64_t)u * M + j) * C + code) * Dm;
        float p32 = 0.0f;
        double p64 = 0.0;
        for (int e = 0; e < Dm; ++e) {
          p32 = fmaf(qs32[j * Dm + e], cv[e], p32);
          p64 += qs64[j * Dm + e] * (double)cv[e];
        }
        s32 = (j == 0) ? p32 : s32 + p32;
        s64 += p64;
      }
      if (score32) score32[(int64_t)u * N + t] = s32;
      if (score64) score64[(int64_t)u * N + t] = s64;
    }
  }
  return 0;
}

/* Exact group scores qs . k_t in double: the ideal the PQ scores approximate
 * (the paper's "Oracle" baseline, Section 4.1).  Used for recall reports only. */
int pqo_exact_scores(const void* q, const void* k, int dtype, int B, int Hq, int Hkv, int64_t N,
                     int D, double* score) {
  if (Hkv <= 0 || Hq % Hkv) return -1;
  int G = Hq / Hkv;
#pragma omp parallel for schedule(static)
  for (int u = 0; u < B * Hkv; ++u) {
    int b = u / Hkv, g = u % Hkv;
    for (int64_t t = 0; t < N; ++t) {
      double s = 0.0;
      for (int d = 0; d < D; ++d) {
        double qs = 0.0;
        for (int h = 0; h < G; ++h) qs += (double)elem(q, dtype, ((int64_t)b * Hq + g * G + h) * D + d);
        s += qs * (double)elem(k, dtype, ((int64_t)u * N + t) * D + d);
      }
      score[(int64_t)u * N + t] = s;
    }
  }
  return 0;
}

/* ---------------------------------------------------------------- selection
 * Section 3.1 step 4 and Section 3.2: the K largest approximate scores among the
 * middle tokens [I, N-L).  Full sort by (score descending, token ascending): a
 * lower token index wins a tie.  The attended set is initial + top-k + local
 * (Algorithm 2, "AllKV").
 *   score [B][Hkv][N] f32  ->  idx [B][Hkv][I+K+L] int32:
 *   initial tokens ascending, then the K retrieved tokens best first, then the
 *   local tokens ascending.
 */
typedef struct {
  float s;
  int32_t t;
} scored;

static int by_score_then_index(const void* a, const void* b) {
  const scored* x = (const scored*)a;
  const scored* y = (const scored*)b;
  if (x->s > y->s) return -1;
  if (x->s < y->s) return 1;
  return (x->t > y->t) - (x->t < y->t);
}

int pqo_select(const float* score, int B, int Hkv, int64_t N, int64_t K, int64_t I, int64_t L,
               int32_t* idx) {
  if (I < 0 || L < 0 || K < 0 || I + K + L > N) return -1;
  int64_t mid = N - I - L, tot = I + K + L;
  int fail = 0;
#pragma omp parallel for schedule(dynamic)
  for (int u = 0; u < B * Hkv; ++u) {
    scored* arr = (scored*)malloc(sizeof(scored) * (size_t)(mid > 0 ? mid : 1));
    if (!arr) {
      fail = 1;
      continue;
    }
    for (int64_t t = 0; t < mid; ++t) {
      arr[t].s = score[(int64_t)u * N + I + t];
      arr[t].t = (int32_t)(I + t);
    }
    qsort(arr, (size_t)mid, sizeof(scored), by_score_then_index);
    int32_t* o = idx + (int64_t)u * tot;
    for (int64_t t = 0; t < I; ++t) o[t] = (int32_t)t;
    for (int64_t t = 0; t < K; ++t) o[I + t] = arr[t].t;
    for (int64_t t = 0; t < L; ++t) o[I + K + t] = (int32_t)(N - L + t);
    free(arr);
  }
  return fail ? -2 : 0;
}

/* ---------------------------------------------------------------- attention
 * Section 2.1 restricted to the selected tokens (Section 3.1 step 6): for each
 * query head h of KV head g,
 *   w_t = exp(scale * q_h . K_t - max),   out_h = sum_t w_t V_t / sum_t w_t,
 * t ranging over the n_idx listed tokens of (b, g).  Double precision.
 *   idx [B][Hkv][n_idx] int32  ->  out [B][Hq][D] double
 */
int pqo_attention(const void* q, const void* k, const void* v, int dtype, int B, int Hq, int Hkv,
                  int64_t N, int D, const int32_t* idx, int64_t n_idx, double scale, double* out) {
  if (Hkv <= 0 || Hq % Hkv || n_idx <= 0) return -1;
  int G = Hq / Hkv;
  int fail = 0;
#pragma omp parallel for schedule(static)
  for (int bh = 0; bh < B * Hq; ++bh) {
    int b = bh / Hq, h = bh % Hq, g = h / G;
    int64_t u = (int64_t)b * Hkv + g;
    double* logit = (double*)malloc(sizeof(double) * (size_t)n_idx);
    if (!logit) {
      fail = 1;
      continue;
    }
    double mx = -INFINITY;
    for (int64_t i = 0; i < n_idx; ++i) {
      int64_t t = idx[u * n_idx + i];
      if (t < 0 || t >= N) {
        fail = 2;
        t = 0;
      }
      double s = 0.0;
      for (int d = 0; d < D; ++d)
        s += (double)elem(q, dtype, (int64_t)bh * D + d) * (double)elem(k, dtype, (u * N + t) * D + d);
      logit[i] = scale * s;
      if (logit[i] > mx) mx = logit[i];
    }
    double den = 0.0;
    for (int64_t i = 0; i < n_idx; ++i) {
      logit[i] = exp(logit[i] - mx);
      den += logit[i];
    }
    for (int d = 0; d < D; ++d) {
      double acc = 0.0;
      for (int64_t i = 0; i < n_idx; ++i) {
        int64_t t = idx[u * n_idx + i];
        if (t < 0 || t >= N) t = 0;
        acc += logit[i] * (double)elem(v, dtype, (u * N + t) * D + d);
      }
      out[(int64_t)bh * D + d] = acc / den;
    }
    free(logit);
  }
  return fail ? -2 : 0;
}

/* The whole decode step (Algorithm 2, PQSearch + AllKV + attention), as the three
 * functions above in order.  This is what the benchmark times as its CPU baseline.
 *   score32 [B][Hkv][N] scratch, idx [B][Hkv][I+K+L], out [B][Hq][D] double
 */
int pqo_decode(const void* q, const float* centroids, const uint8_t* codes, const void* k,
               const void* v, int dtype, int B, int Hq, int Hkv, int64_t N, int D, int M, int C,
               int64_t K, int64_t I, int64_t L, double scale, float* score32, int32_t* idx,
               double* out) {
  int rc = pqo_scores(q, dtype, centroids, codes, B, Hq, Hkv, N, D, M, C, score32, NULL);
  if (rc) return rc;
  rc = pqo_select(score32, B, Hkv, N, K, I, L, idx);
  if (rc) return rc;
  return pqo_attention(q, k, v, dtype, B, Hq, Hkv, N, D, idx, I + K + L, scale, out);
}

/* Per-block counts of selected tokens (Section 3.4: the cache is refreshed with
 * the blocks that hold most of the retrieved tokens).
 *   idx [B][Hkv][n_idx]  ->  counts [B][Hkv][ceil(N/block)] int32
 */
int pqo_block_counts(const int32_t* idx, int B, int Hkv, int64_t N, int64_t n_idx, int block,
                     int32_t* counts) {
  if (block <= 0) return -1;
  int64_t nb = (N + block - 1) / block;
  memset(counts, 0, sizeof(int32_t) * (size_t)(B * Hkv) * nb);
  for (int64_t u = 0; u < (int64_t)B * Hkv; ++u)
    for (int64_t i = 0; i < n_idx; ++i) {
      int64_t t = idx[u * n_idx + i];
      if (t < 0 || t >= N) return -2;
      counts[u * nb + t / block] += 1;
    }
  return 0;
}

/* The blocks to refresh the cache with (Section 3.4): the k_cache blocks that hold the
 * most selected tokens.  The paper does not say how equal counts are ordered: a lower
 * block index ranks first here.  Plain selection sort of the best k_cache blocks.
 *   counts [B][Hkv][nb]  ->  blocks [B][Hkv][k_cache] int32, best first
 */
int pqo_block_topk(const int32_t* counts, int B, int Hkv, int64_t nb, int64_t k_cache, int32_t* blocks) {
  if (k_cache < 0 || k_cache > nb) return -1;
  unsigned char* used = (unsigned char*)malloc((size_t)(nb > 0 ? nb : 1));
  if (!used) return -3;
  for (int64_t u = 0; u < (int64_t)B * Hkv; ++u) {
    const int32_t* c = counts + u * nb;
    memset(used, 0, (size_t)nb);
    for (int64_t r = 0; r < k_cache; ++r) {
      int64_t best = -1;
      for (int64_t j = 0; j < nb; ++j)
        if (!used[j] && (best < 0 || c[j] > c[best])) best = j; /* strict >: the lowest index wins a tie */
      used[best] = 1;
      blocks[u * k_cache + r] = (int32_t)best;
    }
  }
  free(used);
  return 0;
}
