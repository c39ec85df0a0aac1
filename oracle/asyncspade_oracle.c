/*
 * CPU oracle for the KV-selection hot path of AsyncSpade.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64, written from the paper's
 * definitions; it shares no code with the HIP library and must never be called
 * from the product path (only tests, the smoke check and the cpu_baseline leg
 * of the benchmark may load it).
 *
 * All pointers are HOST pointers.  bf16 values travel as uint16_t bit patterns.
 * Values cross stage boundaries in the representation the device path uses
 * (q_hat fp32, scores fp32, attention output bf16 round-to-nearest-even) so each
 * stage can be compared in isolation.
 *
 * Stages (Sec. 4.2, Sec. 4.3, Appendix C Alg. 1):
 *   predict  Eq. 2-5: ridge regression of Q_t on its k newest predecessors,
 *            softmax of the solved weights, applied to the window shifted by
 *            one token; one candidate per window size k = 1..W; mean over k.
 *   score    Alg. 1 step 7 with the batched-matmul shapes of Sec. 4.3:
 *            s[b,j,n] = agg_g <q_hat[b, j*G+g], K[b,j,n]>.
 *   top-k    Sec. 4.3 item (2): the C highest-scoring tokens per KV head.
 *   attend   softmax(q K_S^T * scale) V_S over the selected set S (Sec. 4.1;
 *            Appendix B counts exactly this work, 4*q*h*C flops).
 * Around them (data movement and set arithmetic, no floating point beyond one quotient):
 *   overlap  Sec. 3 Eq. 1, the overlap ratio of two selections;
 *   append / push   the cache rank's per-step state update (Sec. 4.1 workflow);
 *   gather   KV re-organisation for the filtered tokens (Sec. 4.3, cache-rank item (3)).
 *
 * Pins (tests/test_oracle_*.py): closed forms of the predictor on hand-built
 * windows, numpy.linalg.solve, brute-force argsort, numpy GEMV, dense attention
 * from torch's CPU SDPA, and softmax special cases.  Three readings are free
 * parameters that the paper does not fix and therefore stay "parity unpinned":
 * the sign beta inside softmax(beta*omega), the value of epsilon, and how the
 * per-query-head logits of a GQA group are aggregated into one per-KV-head
 * score (max or sum).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ASO_AGG_MAX 0
#define ASO_AGG_SUM 1
/* 2 = softmax-normalised sum: aso_score_keys_softmax_sum */

static double bf16_to_f64(uint16_t h) {
  uint32_t u = ((uint32_t)h) << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

/* One rounding, double -> bf16 (8 significant bits), ties to even. */
static uint16_t f64_to_bf16(double d) {
  if (isnan(d)) return 0x7fc0;
  if (isinf(d)) return d > 0 ? 0x7f80 : 0xff80;
  if (d == 0.0) return signbit(d) ? 0x8000 : 0;
  int e;
  (void)frexp(fabs(d), &e);                 /* |d| = m * 2^e, m in [0.5,1) */
  int lsb = e - 8;                          /* exponent of the last kept bit */
  if (lsb < -133) lsb = -133;               /* bf16 subnormal spacing */
  double q = nearbyint(ldexp(fabs(d), -lsb)); /* default mode = ties to even */
  double r = ldexp(q, lsb);
  float f = (float)(d < 0 ? -r : r);        /* exact unless overflow -> inf */
  uint32_t u;
  memcpy(&u, &f, 4);
  return (uint16_t)(u >> 16);
}

int aso_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
  return omp_get_max_threads();
#else
  (void)n;
  return 1;
#endif
}

/* Solve A x = rhs (n x n, row-major, both destroyed) by Gaussian elimination
 * with partial pivoting.  Returns 0, or -1 if a pivot vanishes. */
static int solve_dense(int n, double* A, double* rhs, double* x) {
  for (int c = 0; c < n; ++c) {
    int p = c;
    for (int r = c + 1; r < n; ++r)
      if (fabs(A[r * n + c]) > fabs(A[p * n + c])) p = r;
    if (A[p * n + c] == 0.0) return -1;
    if (p != c) {
      for (int k = 0; k < n; ++k) { double t = A[c * n + k]; A[c * n + k] = A[p * n + k]; A[p * n + k] = t; }
      double t = rhs[c]; rhs[c] = rhs[p]; rhs[p] = t;
    }
    for (int r = c + 1; r < n; ++r) {
      double f = A[r * n + c] / A[c * n + c];
      for (int k = c; k < n; ++k) A[r * n + k] -= f * A[c * n + k];
      rhs[r] -= f * rhs[c];
    }
  }
  for (int r = n - 1; r >= 0; --r) {
    double s = rhs[r];
    for (int k = r + 1; k < n; ++k) s -= A[r * n + k] * x[k];
    x[r] = s / A[r * n + r];
  }
  return 0;
}

/*
 * Ridge weights for one window size (Eq. 2 read as the linear problem that
 * Alg. 1 step 3 solves): omega = (R R^T + eps I)^-1 R T, with R the k newest
 * predecessors (row i-1 = Q_{t-i}) and T = Q_t.
 *   R [k][D], T [D] fp64; omega [k] out.
 */
int aso_ridge_weights(int k, int D, const double* R, const double* T, double eps, double* omega) {
  double* G = (double*)malloc(sizeof(double) * k * k);
  double* b = (double*)malloc(sizeof(double) * k);
  if (!G || !b) { free(G); free(b); return -2; }
  for (int i = 0; i < k; ++i) {
    for (int j = 0; j < k; ++j) {
      double s = 0.0;
      for (int d = 0; d < D; ++d) s += R[i * D + d] * R[j * D + d];
      G[i * k + j] = s + (i == j ? eps : 0.0);
    }
    double s = 0.0;
    for (int d = 0; d < D; ++d) s += R[i * D + d] * T[d];
    b[i] = s;
  }
  int rc = solve_dense(k, G, b, omega);
  free(G); free(b);
  return rc;
}

/*
 * Predictor, Sec. 4.2 (Eq. 4, Eq. 5) for every (b, h).
 *   q_win  bf16 [B][Hq][W][D], oldest first (Q_{t-W} .. Q_{t-1})
 *   q_cur  bf16 [B][Hq][D]      (Q_t)
 *   q_hat  fp32 [B][Hq][D] out  (prediction of Q_{t+1})
 *   weights_out  nullable fp64 [B][Hq][W][W]; entry [k-1][i-1] = w^{(k)}_{t-i}
 *                for i <= k, 0 above.
 * Returns 0, -1 on bad arguments or a singular system.
 */
int aso_predict_query(int B, int Hq, int W, int D, const uint16_t* q_win, const uint16_t* q_cur,
                      double eps, double beta, float* q_hat, double* weights_out) {
  if (B < 0 || Hq <= 0 || W < 1 || D <= 0 || !(eps > 0.0)) return -1;
  int fail = 0;
#pragma omp parallel for schedule(static)
  for (int bh = 0; bh < B * Hq; ++bh) {
    double* R = (double*)malloc(sizeof(double) * W * D);   /* R[i-1] = Q_{t-i}        */
    double* S = (double*)malloc(sizeof(double) * W * D);   /* S[i-1] = Q_{t+1-i}      */
    double* T = (double*)malloc(sizeof(double) * D);
    double* om = (double*)malloc(sizeof(double) * W);
    double* w = (double*)malloc(sizeof(double) * W);
    double* acc = (double*)calloc(D, sizeof(double));
    if (!R || !S || !T || !om || !w || !acc) {     /* out of memory: report, do not dereference */
#pragma omp atomic write
      fail = 1;
      free(R); free(S); free(T); free(om); free(w); free(acc);
      continue;
    }
    const uint16_t* win = q_win + (size_t)bh * W * D;
    const uint16_t* cur = q_cur + (size_t)bh * D;
    for (int d = 0; d < D; ++d) T[d] = bf16_to_f64(cur[d]);
    for (int i = 1; i <= W; ++i)
      for (int d = 0; d < D; ++d) R[(i - 1) * D + d] = bf16_to_f64(win[(size_t)(W - i) * D + d]);
    /* shifted window: Q_{t+1-i}; i = 1 is Q_t itself, i >= 2 is R_{i-1} */
    for (int d = 0; d < D; ++d) S[d] = T[d];
    for (int i = 2; i <= W; ++i)
      for (int d = 0; d < D; ++d) S[(i - 1) * D + d] = R[(i - 2) * D + d];

    for (int k = 1; k <= W; ++k) {
      if (aso_ridge_weights(k, D, R, T, eps, om) != 0) {
#pragma omp atomic write
        fail = 1;
        continue;
      }
      /* softmax normalisation, Eq. 3 */
      double mx = beta * om[0];
      for (int i = 1; i < k; ++i) if (beta * om[i] > mx) mx = beta * om[i];
      double z = 0.0;
      for (int i = 0; i < k; ++i) { w[i] = exp(beta * om[i] - mx); z += w[i]; }
      for (int i = 0; i < k; ++i) w[i] /= z;
      if (weights_out) {
        double* wo = weights_out + ((size_t)bh * W + (k - 1)) * W;
        for (int i = 0; i < W; ++i) wo[i] = i < k ? w[i] : 0.0;
      }
      /* candidate for window size k applied to the shifted window (Eq. 4),
         accumulated into the mean of Eq. 5 */
      for (int d = 0; d < D; ++d) {
        double c = 0.0;
        for (int i = 0; i < k; ++i) c += w[i] * S[i * D + d];
        acc[d] += c;
      }
    }
    for (int d = 0; d < D; ++d) q_hat[(size_t)bh * D + d] = (float)(acc[d] / (double)W);
    free(R); free(S); free(T); free(om); free(w); free(acc);
  }
  return fail ? -1 : 0;
}

/*
 * Predictor with a single ridge solve (Appendix C, Alg. 1 steps 3-5, on the window bookkeeping of
 * Sec. 4.2): omega = (R R^T + eps I)^-1 R Q_t is solved once over all W predecessors; the weights
 * of window size k are the softmax of beta * omega truncated to its k newest entries
 * (truncate and renormalise), applied to the shifted window as in Eq. 4; mean over k (Eq. 5).
 * Same arguments as aso_predict_query.
 */
int aso_predict_query_single_solve(int B, int Hq, int W, int D, const uint16_t* q_win, const uint16_t* q_cur,
                                   double eps, double beta, float* q_hat, double* weights_out) {
  if (B < 0 || Hq <= 0 || W < 1 || D <= 0 || !(eps > 0.0)) return -1;
  int fail = 0;
#pragma omp parallel for schedule(static)
  for (int bh = 0; bh < B * Hq; ++bh) {
    double* R = (double*)malloc(sizeof(double) * W * D);   /* R[i-1] = Q_{t-i}   */
    double* S = (double*)malloc(sizeof(double) * W * D);   /* S[i-1] = Q_{t+1-i} */
    double* T = (double*)malloc(sizeof(double) * D);
    double* om = (double*)malloc(sizeof(double) * W);
    double* w = (double*)malloc(sizeof(double) * W);
    double* acc = (double*)calloc(D, sizeof(double));
    if (!R || !S || !T || !om || !w || !acc) {     /* out of memory: report, do not dereference */
#pragma omp atomic write
      fail = 1;
      free(R); free(S); free(T); free(om); free(w); free(acc);
      continue;
    }
    const uint16_t* win = q_win + (size_t)bh * W * D;
    const uint16_t* cur = q_cur + (size_t)bh * D;
    for (int d = 0; d < D; ++d) T[d] = bf16_to_f64(cur[d]);
    for (int i = 1; i <= W; ++i)
      for (int d = 0; d < D; ++d) R[(i - 1) * D + d] = bf16_to_f64(win[(size_t)(W - i) * D + d]);
    for (int d = 0; d < D; ++d) S[d] = T[d];
    for (int i = 2; i <= W; ++i)
      for (int d = 0; d < D; ++d) S[(i - 1) * D + d] = R[(i - 2) * D + d];
    if (aso_ridge_weights(W, D, R, T, eps, om) != 0) {
#pragma omp atomic write
      fail = 1;
    } else {
      for (int k = 1; k <= W; ++k) {
        double mx = beta * om[0];
        for (int i = 1; i < k; ++i) if (beta * om[i] > mx) mx = beta * om[i];
        double z = 0.0;
        for (int i = 0; i < k; ++i) { w[i] = exp(beta * om[i] - mx); z += w[i]; }
        for (int i = 0; i < k; ++i) w[i] /= z;
        if (weights_out) {
          double* wo = weights_out + ((size_t)bh * W + (k - 1)) * W;
          for (int i = 0; i < W; ++i) wo[i] = i < k ? w[i] : 0.0;
        }
        for (int d = 0; d < D; ++d) {
          double c = 0.0;
          for (int i = 0; i < k; ++i) c += w[i] * S[i * D + d];
          acc[d] += c;
        }
      }
      for (int d = 0; d < D; ++d) q_hat[(size_t)bh * D + d] = (float)(acc[d] / (double)W);
    }
    free(R); free(S); free(T); free(om); free(w); free(acc);
  }
  return fail ? -1 : 0;
}

static const uint16_t* token_ptr(const uint16_t* pool, const int32_t* block_table, int max_pages,
                                 int Hkv, int P, int D, int b, int j, int n) {
  int64_t page = block_table[(int64_t)b * max_pages + n / P];
  int slot = n % P;
  return pool + ((page * Hkv + j) * P + slot) * (int64_t)D;
}

/*
 * Criticality scores (Alg. 1 step 7; shapes of Sec. 4.3).
 *   k_pool bf16 [num_pages][Hkv][P][D]; block_table [B][max_pages]; ctx_lens [B]
 *   q_hat fp32 [B][Hq][D]; scores fp32 [B][Hkv][stride]; entries n >= ctx_lens[b]
 *   are left untouched.  agg: 0 = max over the group, 1 = sum.
 */
int aso_score_keys(int B, int Hq, int Hkv, int D, int P, const uint16_t* k_pool,
                   const int32_t* block_table, int max_pages, const int32_t* ctx_lens,
                   const float* q_hat, int agg, float* scores, int64_t stride) {
  if (Hkv <= 0 || Hq % Hkv != 0) return -1;
  int G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b)
    for (int j = 0; j < Hkv; ++j) {
      int N = ctx_lens[b];
      for (int n = 0; n < N; ++n) {
        const uint16_t* kr = token_ptr(k_pool, block_table, max_pages, Hkv, P, D, b, j, n);
        double best = 0.0;
        for (int g = 0; g < G; ++g) {
          const float* q = q_hat + ((size_t)b * Hq + (size_t)j * G + g) * D;
          double s = 0.0;
          for (int d = 0; d < D; ++d) s += (double)q[d] * bf16_to_f64(kr[d]);
          if (g == 0) best = s;
          else if (agg == ASO_AGG_SUM) best += s;
          else if (s > best) best = s;
        }
        float f = (float)best;
        f = f + 0.0f;                     /* -0 -> +0 */
        scores[((size_t)b * Hkv + j) * stride + n] = f;
      }
    }
  return 0;
}

/*
 * Criticality scores with softmax-normalised group aggregation (a reading of the point the paper
 * leaves open, how the per-query-head logits of Alg. 1 step 7 become one score per KV head):
 * every head's logits are turned into the attention distribution that head would have,
 *   p[g][n] = exp(scale * l[g][n] - LSE_g),  LSE_g = log sum_{n < N_b} exp(scale * l[g][n]),
 * and the score of token n is the probability mass the group gives it, s[n] = sum_g p[g][n].
 * Two passes per row, all in fp64; same layout and conventions as aso_score_keys.
 */
int aso_score_keys_softmax_sum(int B, int Hq, int Hkv, int D, int P, const uint16_t* k_pool,
                               const int32_t* block_table, int max_pages, const int32_t* ctx_lens,
                               const float* q_hat, double scale, float* scores, int64_t stride) {
  if (Hkv <= 0 || Hq % Hkv != 0) return -1;
  int G = Hq / Hkv;
  int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b)
    for (int j = 0; j < Hkv; ++j) {
      int N = ctx_lens[b];
      if (N <= 0) continue;
      double* logit = (double*)malloc(sizeof(double) * (size_t)N * G);
      double* lse = (double*)malloc(sizeof(double) * G);
      if (!logit || !lse) {               /* out of memory: report, do not dereference */
#pragma omp atomic write
        fail = 1;
        free(logit); free(lse);
        continue;
      }
      for (int g = 0; g < G; ++g) {
        const float* q = q_hat + ((size_t)b * Hq + (size_t)j * G + g) * D;
        double m = -INFINITY;
        for (int n = 0; n < N; ++n) {
          const uint16_t* kr = token_ptr(k_pool, block_table, max_pages, Hkv, P, D, b, j, n);
          double s = 0.0;
          for (int d = 0; d < D; ++d) s += (double)q[d] * bf16_to_f64(kr[d]);
          logit[(size_t)g * N + n] = scale * s;
          if (scale * s > m) m = scale * s;
        }
        double z = 0.0;
        for (int n = 0; n < N; ++n) z += exp(logit[(size_t)g * N + n] - m);
        lse[g] = m + log(z);
      }
      for (int n = 0; n < N; ++n) {
        double s = 0.0;
        for (int g = 0; g < G; ++g) s += exp(logit[(size_t)g * N + n] - lse[g]);
        scores[((size_t)b * Hkv + j) * stride + n] = (float)s;
      }
      free(logit); free(lse);
    }
  return fail ? -2 : 0;
}

typedef struct { float s; int32_t n; } aso_cand;

/* order: score descending (NaN below everything), then index ascending */
static int cand_cmp(const void* pa, const void* pb) {
  const aso_cand* a = (const aso_cand*)pa;
  const aso_cand* b = (const aso_cand*)pb;
  int an = isnan(a->s), bn = isnan(b->s);
  if (an != bn) return an ? 1 : -1;
  if (!an) {
    if (a->s > b->s) return -1;
    if (a->s < b->s) return 1;
  }
  return (a->n > b->n) - (a->n < b->n);
}
static int int_cmp(const void* pa, const void* pb) {
  int32_t a = *(const int32_t*)pa, b = *(const int32_t*)pb;
  return (a > b) - (a < b);
}

/*
 * Top-k per (b, kv head): full sort, keep min(C, N_b), emit ascending, pad -1.
 *   scores fp32 [B][Hkv][stride]; sel_idx int32 [B][Hkv][C]; sel_cnt int32 [B][Hkv]
 */
int aso_topk_select(int B, int Hkv, int C, const float* scores, int64_t stride,
                    const int32_t* ctx_lens, int32_t* sel_idx, int32_t* sel_cnt) {
  if (C < 1) return -1;
  int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b)
    for (int j = 0; j < Hkv; ++j) {
      int N = ctx_lens[b];
      const float* s = scores + ((size_t)b * Hkv + j) * stride;
      int32_t* out = sel_idx + ((size_t)b * Hkv + j) * C;
      aso_cand* c = (aso_cand*)malloc(sizeof(aso_cand) * (N > 0 ? N : 1));
      if (!c) {                           /* out of memory: report, do not dereference */
#pragma omp atomic write
        fail = 1;
        continue;
      }
      for (int n = 0; n < N; ++n) { c[n].s = s[n]; c[n].n = n; }
      qsort(c, N, sizeof(aso_cand), cand_cmp);
      int keep = N < C ? N : C;
      for (int i = 0; i < keep; ++i) out[i] = c[i].n;
      qsort(out, keep, sizeof(int32_t), int_cmp);
      for (int i = keep; i < C; ++i) out[i] = -1;
      sel_cnt[(size_t)b * Hkv + j] = keep;
      free(c);
    }
  return fail ? -2 : 0;
}

/*
 * Sparse decode attention with the real query over S = selected tokens plus
 * the dense tail [sel_ctx_lens[b], ctx_lens[b]) (tail empty when sel_ctx_lens
 * is NULL).
 *   q bf16 [B][Hq][D]; out bf16 [B][Hq][D]; lse nullable fp32 [B][Hq] (natural log)
 *   Empty S gives out = 0 and lse = -inf.
 */
int aso_sparse_decode_attn(int B, int Hq, int Hkv, int D, int P, int C, const uint16_t* k_pool,
                           const uint16_t* v_pool, const int32_t* block_table, int max_pages,
                           const int32_t* ctx_lens, const uint16_t* q, const int32_t* sel_idx,
                           const int32_t* sel_cnt, const int32_t* sel_ctx_lens, double sm_scale,
                           uint16_t* out, float* lse) {
  if (Hkv <= 0 || Hq % Hkv != 0) return -1;
  int G = Hq / Hkv;
  int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < Hq; ++h) {
      int j = h / G;
      int N = ctx_lens[b];
      int cnt = sel_cnt[(size_t)b * Hkv + j];
      int tail0 = sel_ctx_lens ? sel_ctx_lens[b] : N;
      if (tail0 > N) tail0 = N;
      if (tail0 < 0) tail0 = 0;
      int L = cnt + (N - tail0);
      uint16_t* o = out + ((size_t)b * Hq + h) * D;
      if (L <= 0) {
        for (int d = 0; d < D; ++d) o[d] = 0;
        if (lse) lse[(size_t)b * Hq + h] = -INFINITY;
        continue;
      }
      int32_t* toks = (int32_t*)malloc(sizeof(int32_t) * L);
      double* logit = (double*)malloc(sizeof(double) * L);
      double* acc = (double*)calloc(D, sizeof(double));
      if (!toks || !logit || !acc) {      /* out of memory: report, do not dereference */
#pragma omp atomic write
        fail = 1;
        free(toks); free(logit); free(acc);
        continue;
      }
      for (int i = 0; i < cnt; ++i) toks[i] = sel_idx[((size_t)b * Hkv + j) * C + i];
      for (int n = tail0; n < N; ++n) toks[cnt + (n - tail0)] = n;
      const uint16_t* qr = q + ((size_t)b * Hq + h) * D;
      double m = -INFINITY;
      for (int i = 0; i < L; ++i) {
        const uint16_t* kr = token_ptr(k_pool, block_table, max_pages, Hkv, P, D, b, j, toks[i]);
        double s = 0.0;
        for (int d = 0; d < D; ++d) s += bf16_to_f64(qr[d]) * bf16_to_f64(kr[d]);
        logit[i] = s * sm_scale;
        if (logit[i] > m) m = logit[i];
      }
      double z = 0.0;
      for (int i = 0; i < L; ++i) {
        double p = exp(logit[i] - m);
        z += p;
        const uint16_t* vr = token_ptr(v_pool, block_table, max_pages, Hkv, P, D, b, j, toks[i]);
        for (int d = 0; d < D; ++d) acc[d] += p * bf16_to_f64(vr[d]);
      }
      for (int d = 0; d < D; ++d) o[d] = f64_to_bf16(acc[d] / z);
      if (lse) lse[(size_t)b * Hq + h] = (float)(m + log(z));
      free(toks); free(logit); free(acc);
    }
  return fail ? -2 : 0;
}

/*
 * Overlap ratio of two selections (Sec. 3, Eq. 1): O = |S_a intersect S_b| / |S|, with |S| the
 * common size of the two sets (the larger one if they differ; 0 / 0 is reported as 0).
 * Plain double loop over both index lists; entries are token indices, order irrelevant.
 *   idx_a, idx_b int32 [B][Hkv][C]; cnt_a, cnt_b int32 [B][Hkv]
 *   inter int32 [B][Hkv] out; ratio fp32 [B][Hkv] out (the fp32 quotient of the two integers)
 */
int aso_overlap_ratio(int B, int Hkv, int C, const int32_t* idx_a, const int32_t* cnt_a,
                      const int32_t* idx_b, const int32_t* cnt_b, int32_t* inter, float* ratio) {
  for (int r = 0; r < B * Hkv; ++r) {
    const int32_t* a = idx_a + (size_t)r * C;
    const int32_t* b = idx_b + (size_t)r * C;
    int na = cnt_a[r], nb = cnt_b[r], common = 0;
    for (int i = 0; i < na; ++i) {
      int hit = 0;
      for (int k = 0; k < nb; ++k) if (b[k] == a[i]) hit = 1;
      common += hit;
    }
    int den = na > nb ? na : nb;
    inter[r] = common;
    ratio[r] = den > 0 ? (float)common / (float)den : 0.0f;
  }
  return 0;
}

/*
 * Cache-side state updates of one decode step (Sec. 4.1, workflow: the cache rank appends the
 * step's key / value states to the KV cache and enqueues its query state to the sliding window).
 *
 * aso_kv_append: for every sequence with room (ctx_lens[b] < P * max_pages) the new token's
 * K and V rows are stored at position n = ctx_lens[b] and ctx_lens[b] becomes n + 1; a
 * sequence without room is left as it is.
 *   k_new, v_new bf16 [B][Hkv][D]
 */
int aso_kv_append(int B, int Hkv, int D, int P, uint16_t* k_pool, uint16_t* v_pool,
                  const int32_t* block_table, int max_pages, int32_t* ctx_lens,
                  const uint16_t* k_new, const uint16_t* v_new) {
  for (int b = 0; b < B; ++b) {
    int n = ctx_lens[b];
    if (n < 0 || n >= P * max_pages) continue;
    int64_t page = block_table[(int64_t)b * max_pages + n / P];
    for (int j = 0; j < Hkv; ++j) {
      int64_t off = ((page * Hkv + j) * P + n % P) * (int64_t)D;
      for (int d = 0; d < D; ++d) {
        k_pool[off + d] = k_new[((size_t)b * Hkv + j) * D + d];
        v_pool[off + d] = v_new[((size_t)b * Hkv + j) * D + d];
      }
    }
    ctx_lens[b] = n + 1;
  }
  return 0;
}

/*
 * aso_window_push: the window slides by one token: the oldest query leaves, the previous
 * current query becomes the newest window entry and q_new becomes the current query.
 *   q_win bf16 [B][Hq][W][D] oldest first (in place); q_cur bf16 [B][Hq][D] (in place);
 *   q_new bf16 [B][Hq][D]
 */
int aso_window_push(int B, int Hq, int W, int D, uint16_t* q_win, uint16_t* q_cur, const uint16_t* q_new) {
  for (int bh = 0; bh < B * Hq; ++bh) {
    uint16_t* win = q_win + (size_t)bh * W * D;
    uint16_t* cur = q_cur + (size_t)bh * D;
    for (int i = 0; i + 1 < W; ++i)
      for (int d = 0; d < D; ++d) win[(size_t)i * D + d] = win[(size_t)(i + 1) * D + d];
    for (int d = 0; d < D; ++d) win[(size_t)(W - 1) * D + d] = cur[d];
    for (int d = 0; d < D; ++d) cur[d] = q_new[(size_t)bh * D + d];
  }
  return 0;
}

/*
 * KV re-organisation for the filtered tokens (Sec. 4.3, cache-rank item (3)): the selected
 * rows are copied, in selection order, into a compact paged pool of Cp = ceil(C / P) pages per
 * sequence: token i of (b, j) goes to page b * Cp + i / P, slot i % P.
 *   k_out, v_out bf16 [B * Cp][Hkv][P][D]; slots at and beyond sel_cnt are left untouched
 *   out_table int32 [B][Cp] = b * Cp + i;  out_lens int32 [B] = sel_cnt[b][0]
 */
int aso_gather_kv(int B, int Hkv, int D, int P, int C, const uint16_t* k_pool, const uint16_t* v_pool,
                  const int32_t* block_table, int max_pages, const int32_t* sel_idx,
                  const int32_t* sel_cnt, uint16_t* k_out, uint16_t* v_out, int32_t* out_table,
                  int32_t* out_lens) {
  int Cp = (C + P - 1) / P;
  for (int b = 0; b < B; ++b) {
    for (int i = 0; i < Cp; ++i) out_table[(size_t)b * Cp + i] = b * Cp + i;
    out_lens[b] = sel_cnt[(size_t)b * Hkv];
    for (int j = 0; j < Hkv; ++j) {
      int cnt = sel_cnt[(size_t)b * Hkv + j];
      for (int i = 0; i < cnt; ++i) {
        int n = sel_idx[((size_t)b * Hkv + j) * C + i];
        const uint16_t* kr = token_ptr(k_pool, block_table, max_pages, Hkv, P, D, b, j, n);
        const uint16_t* vr = token_ptr(v_pool, block_table, max_pages, Hkv, P, D, b, j, n);
        int64_t off = ((((int64_t)b * Cp + i / P) * Hkv + j) * P + i % P) * (int64_t)D;
        for (int d = 0; d < D; ++d) { k_out[off + d] = kr[d]; v_out[off + d] = vr[d]; }
      }
    }
  }
  return 0;
}

/* exposed for tests of the rounding helper */
uint16_t aso_f64_to_bf16(double d) { return f64_to_bf16(d); }
