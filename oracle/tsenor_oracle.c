/*
 * CPU oracle for transposable N:M mask finding (TSENOR).  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain, double-precision statement of what the method
 * computes.  It exists so that the GPU library can be checked against it and so
 * that the benchmark can quote a host-CPU baseline.  It shares no code, header,
 * table or helper with the HIP path, and nothing in the product path may call
 * it: only tests, the smoke check and the benchmark's cpu_baseline leg do.
 *
 * What it follows, step by step and in the paper's notation:
 *   - Sec. 3.1, Eq. (2): the problem separates over the MxM blocks of the matrix.
 *   - Sec. 3.2, Eq. (4) and Algorithm 1: entropy-regularised capacitated
 *     transport solved by Dykstra's alternating KL projections onto the row-sum
 *     set C1, the column-sum set C2 and the box C3, with one dual variable Q for
 *     the box; carried out in the log domain as App. A.2 prescribes
 *     (log-sum-exp normalisation, log_Q additive).
 *   - Sec. 3.3, Algorithm 2 and Eq. (5): greedy selection over the descending
 *     order of the fractional plan, then swap-based local search.
 *
 * Readings taken where the paper leaves a choice (each is also a parameter or
 * a comment at the place it is used):
 *   - Projection order: rows first (sum over j within row i), then columns,
 *     as in Algorithm 1; cols_first=1 gives the other order.
 *   - Exactly T iterations, no convergence test; log_Q starts at 0 (Q = 1).
 *   - Greedy sort key is log S^(T); equal keys are taken in ascending flat
 *     index i*M+j.
 *   - Local search picks the lowest-index deficient row i and column j; the
 *     arg-max of Eq. (5) breaks ties towards the lowest flat index i'*M+j'.
 *   - Default local search runs until every row and column holds N ones and
 *     applies the best finite swap even if its score is <= 0 (the algorithm is
 *     stated to return a feasible mask).  strict_paper=1 gives Algorithm 2 as
 *     printed: at most L rounds, a swap applied only when its score is > 0.
 *   - tau: mode ABSOLUTE takes log-kernel tau*imp (Algorithm 1 line 1);
 *     mode REL_MATRIX_MAX takes imp / (tau * max imp), i.e. the entropy weight
 *     1/tau_eff is tau times the largest importance of the matrix (App. B.1
 *     parameter choice, read so that it is dimensionally consistent with Eq. 4).
 *
 * Pins (tests/test_oracle_pins.py): the worked 4x4 example of Fig. 2, brute
 * force over all feasible 2:4 masks, the LP optimum of Eq. (3), Sinkhorn
 * scaling when the cap cannot bind, closed forms, KKT conditions of Eq. (4)
 * at convergence, equivariances.  The iterates at finite T with an active cap
 * and the tie-break readings above are fixed by this file's readings only.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_TAU_ABSOLUTE 0
#define ORACLE_TAU_REL_MATRIX_MAX 1

int tsenor_oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void tsenor_oracle_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/* Importance of every weight: |w| or |w| * col_scale[j], one float multiply
 * (Sec. 4, Wanda integration: weights scaled per input feature before Eq. 1). */
int tsenor_oracle_importance(const float* W, int64_t rows, int64_t cols, int64_t ld,
                             const float* col_scale, float* imp) {
  if (!W || !imp || rows <= 0 || cols <= 0 || ld < cols) return -1;
  for (int64_t i = 0; i < rows; ++i)
    for (int64_t j = 0; j < cols; ++j) {
      float a = fabsf(W[i * ld + j]);
      imp[i * cols + j] = col_scale ? a * col_scale[j] : a;
    }
  return 0;
}

/* The multiplier applied to the importance to form the log-kernel. */
double tsenor_oracle_tau_eff(const float* imp, int64_t rows, int64_t cols, double tau, int tau_mode) {
  if (tau_mode == ORACLE_TAU_ABSOLUTE) return tau;
  float mx = 0.0f;
  for (int64_t k = 0; k < rows * cols; ++k)
    if (imp[k] > mx) mx = imp[k];
  if (!(mx > 0.0f)) return 0.0; /* all-zero matrix: flat kernel */
  return 1.0 / (tau * (double)mx);
}

static double lse(const double* x, int n, int stride) {
  double m = x[0];
  for (int k = 1; k < n; ++k)
    if (x[k * stride] > m) m = x[k * stride];
  double s = 0.0;
  for (int k = 0; k < n; ++k) s += exp(x[k * stride] - m);
  return m + log(s);
}

/* Algorithm 1 on one block in the log domain.  log_S, log_Q: M*M doubles, row-major. */
static void dykstra_block(const float* imp, int64_t ld, int N, int M, double tau_eff, int T,
                          int cols_first, double* log_S, double* log_Q) {
  const double logN = log((double)N);
  for (int i = 0; i < M; ++i)
    for (int j = 0; j < M; ++j) {
      log_S[i * M + j] = tau_eff * (double)imp[i * ld + j]; /* S^(0) = exp(tau |W|) */
      log_Q[i * M + j] = 0.0;                               /* Q^(0) = 1 */
    }
  for (int t = 0; t < T; ++t) {
    for (int pass = 0; pass < 2; ++pass) {
      int do_rows = (pass == 0) != (cols_first != 0);
      if (do_rows) { /* projection onto C1: every row sums to N */
        for (int i = 0; i < M; ++i) {
          double shift = lse(log_S + i * M, M, 1) - logN;
          for (int j = 0; j < M; ++j) log_S[i * M + j] -= shift;
        }
      } else { /* projection onto C2: every column sums to N */
        for (int j = 0; j < M; ++j) {
          double shift = lse(log_S + j, M, M) - logN;
          for (int i = 0; i < M; ++i) log_S[i * M + j] -= shift;
        }
      }
    }
    /* projection onto C3 with its dual: S <- min(S*Q, 1), Q <- Q * S_old / S_new */
    for (int k = 0; k < M * M; ++k) {
      double tmp = log_S[k] + log_Q[k];
      double capped = tmp < 0.0 ? tmp : 0.0;
      log_Q[k] = tmp - capped;
      log_S[k] = capped;
    }
  }
}

/* Algorithm 1 with an early exit ("maximum iterations T" read as a bound): after every `check_every`-th
 * iteration the block stops if every scaling factor that iteration applied - N / (row sum) in the projection
 * onto C1, N / (column sum) in the projection onto C2 - lies within `tol` of 1.  Returns the number of
 * iterations done.  tol <= 0 never stops early. */
static int dykstra_block_adaptive(const float* imp, int64_t ld, int N, int M, double tau_eff, int T,
                                  int cols_first, double tol, int check_every, double* log_S, double* log_Q) {
  const double logN = log((double)N);
  for (int i = 0; i < M; ++i)
    for (int j = 0; j < M; ++j) {
      log_S[i * M + j] = tau_eff * (double)imp[i * ld + j];
      log_Q[i * M + j] = 0.0;
    }
  for (int t = 0; t < T; ++t) {
    double worst = 0.0; /* largest |factor - 1| of this iteration */
    for (int pass = 0; pass < 2; ++pass) {
      int do_rows = (pass == 0) != (cols_first != 0);
      for (int k = 0; k < M; ++k) {
        double shift = (do_rows ? lse(log_S + k * M, M, 1) : lse(log_S + k, M, M)) - logN;
        double dev = fabs(exp(-shift) - 1.0); /* the factor is N / sum = exp(-shift) */
        if (dev > worst) worst = dev;
        for (int l = 0; l < M; ++l) {
          if (do_rows)
            log_S[k * M + l] -= shift;
          else
            log_S[l * M + k] -= shift;
        }
      }
    }
    for (int k = 0; k < M * M; ++k) {
      double tmp = log_S[k] + log_Q[k];
      double capped = tmp < 0.0 ? tmp : 0.0;
      log_Q[k] = tmp - capped;
      log_S[k] = capped;
    }
    if (tol > 0.0 && (t + 1) % check_every == 0 && worst <= tol) return t + 1;
  }
  return T;
}

/* The early-exit variant over every block.  iters_done (optional): one int per block, block-row major. */
int tsenor_oracle_dykstra_adaptive(const float* imp, int64_t rows, int64_t cols, int N, int M, double tau_eff,
                                   int T, int cols_first, double tol, int check_every, double* log_S,
                                   int32_t* iters_done) {
  if (!imp || !log_S || M <= 0 || rows <= 0 || cols <= 0 || rows % M || cols % M || N < 1 || N > M || T < 0 ||
      check_every < 1)
    return -1;
  const int64_t bc = cols / M, nb = (rows / M) * bc;
  int err = 0;
#pragma omp parallel
  {
    double* s = (double*)malloc(sizeof(double) * M * M);
    double* q = (double*)malloc(sizeof(double) * M * M);
    if (!s || !q) {
#pragma omp atomic write
      err = 1;
    } else {
#pragma omp for schedule(dynamic, 16)
      for (int64_t b = 0; b < nb; ++b) {
        int64_t r0 = (b / bc) * M, c0 = (b % bc) * M;
        int done = dykstra_block_adaptive(imp + r0 * cols + c0, cols, N, M, tau_eff, T, cols_first, tol,
                                          check_every, s, q);
        if (iters_done) iters_done[b] = done;
        for (int i = 0; i < M; ++i)
          for (int j = 0; j < M; ++j) log_S[(r0 + i) * cols + c0 + j] = s[i * M + j];
      }
    }
    free(s);
    free(q);
  }
  return err ? -2 : 0;
}

/* Algorithm 1 over every block.  imp: rows x cols floats (row-major, dense).
 * log_S: rows x cols doubles in the matrix's own layout; log_Q may be NULL. */
int tsenor_oracle_dykstra(const float* imp, int64_t rows, int64_t cols, int N, int M,
                          double tau_eff, int T, int cols_first, double* log_S, double* log_Q) {
  if (!imp || !log_S || M <= 0 || rows <= 0 || cols <= 0 || rows % M || cols % M || N < 1 || N > M || T < 0)
    return -1;
  const int64_t bc = cols / M, nb = (rows / M) * bc;
  int err = 0;
#pragma omp parallel
  {
    double* s = (double*)malloc(sizeof(double) * M * M);
    double* q = (double*)malloc(sizeof(double) * M * M);
    if (!s || !q) {
#pragma omp atomic write
      err = 1;
    } else {
#pragma omp for schedule(dynamic, 16)
      for (int64_t b = 0; b < nb; ++b) {
        int64_t r0 = (b / bc) * M, c0 = (b % bc) * M;
        dykstra_block(imp + r0 * cols + c0, cols, N, M, tau_eff, T, cols_first, s, q);
        for (int i = 0; i < M; ++i)
          for (int j = 0; j < M; ++j) {
            log_S[(r0 + i) * cols + c0 + j] = s[i * M + j];
            if (log_Q) log_Q[(r0 + i) * cols + c0 + j] = q[i * M + j];
          }
      }
    }
    free(s);
    free(q);
  }
  return err ? -2 : 0;
}

typedef struct {
  double key;
  int idx;
} keyed;

static int by_key_desc_then_index(const void* a, const void* b) {
  const keyed* x = (const keyed*)a;
  const keyed* y = (const keyed*)b;
  if (x->key > y->key) return -1;
  if (x->key < y->key) return 1;
  return (x->idx > y->idx) - (x->idx < y->idx);
}

/* Algorithm 2 on one block.  key: M*M doubles (row-major, stride ldk); imp: floats, stride ldi.
 * S: M*M bytes out.  Returns the number of swaps applied; counters go to st[0..3]:
 * st[0] += units still missing after greedy, st[1] += swaps applied with score <= 0,
 * st[2] += 1 if the block needed more than L rounds (default mode), st[3] += units
 * still missing at return (strict mode only). */
static void round_block(const double* key, int64_t ldk, const float* imp, int64_t ldi, int N, int M,
                        int L, int strict_paper, uint8_t* S, keyed* order, int* R, int* C, int64_t* st) {
  const int MM = M * M;
  for (int i = 0; i < M; ++i)
    for (int j = 0; j < M; ++j) {
      order[i * M + j].key = key[i * ldk + j];
      order[i * M + j].idx = i * M + j;
    }
  qsort(order, MM, sizeof(keyed), by_key_desc_then_index);
  memset(S, 0, MM);
  for (int i = 0; i < M; ++i) R[i] = C[i] = 0;
  /* greedy selection, Algorithm 2 lines 3-6 */
  int placed = 0;
  for (int t = 0; t < MM; ++t) {
    int i = order[t].idx / M, j = order[t].idx % M;
    if (R[i] < N && C[j] < N) {
      S[i * M + j] = 1;
      ++R[i];
      ++C[j];
      ++placed;
    }
  }
  int deficit = N * M - placed;
  st[0] += deficit;
  /* local search, Algorithm 2 lines 7-13 */
  int rounds = 0;
  while (deficit > 0) {
    if (strict_paper && rounds >= L) break;
    int i = -1, j = -1;
    for (int k = 0; k < M && i < 0; ++k)
      if (R[k] < N) i = k;
    for (int k = 0; k < M && j < 0; ++k)
      if (C[k] < N) j = k;
    /* Eq. (5): Swap(i',j') = imp[i][j'] + imp[i'][j] - imp[i'][j'] over S[i'][j']=1, S[i][j']=0, S[i'][j]=0 */
    int have = 0, bi = -1, bj = -1;
    double best = 0.0;
    for (int ip = 0; ip < M; ++ip)
      for (int jp = 0; jp < M; ++jp) {
        if (!S[ip * M + jp] || S[i * M + jp] || S[ip * M + j]) continue;
        double sc = (double)imp[i * ldi + jp] + (double)imp[ip * ldi + j] - (double)imp[ip * ldi + jp];
        if (!have || sc > best) {
          have = 1;
          best = sc;
          bi = ip;
          bj = jp;
        }
      }
    ++rounds;
    if (!have) break;
    if (strict_paper && !(best > 0.0)) break; /* nothing changes, so later rounds repeat this one */
    if (!(best > 0.0)) st[1] += 1;
    S[bi * M + bj] = 0;
    S[bi * M + j] = 1;
    S[i * M + bj] = 1;
    ++R[i];
    ++C[j];
    --deficit;
  }
  if (!strict_paper && rounds > L) st[2] += 1;
  st[3] += deficit;
}

/* Algorithm 2 over every block.  key: rows x cols doubles (the fractional plan or
 * any score to round); imp: rows x cols floats; mask: rows x cols bytes out.
 * stats: 4 int64 counters (see round_block), may be NULL. */
int tsenor_oracle_round(const double* key, const float* imp, int64_t rows, int64_t cols, int N, int M,
                        int L, int strict_paper, uint8_t* mask, int64_t* stats) {
  if (!key || !imp || !mask || M <= 0 || rows <= 0 || cols <= 0 || rows % M || cols % M || N < 0 || N > M)
    return -1;
  const int64_t bc = cols / M, nb = (rows / M) * bc;
  int64_t tot[4] = {0, 0, 0, 0};
  int err = 0;
#pragma omp parallel
  {
    uint8_t* S = (uint8_t*)malloc(M * M);
    keyed* order = (keyed*)malloc(sizeof(keyed) * M * M);
    int* R = (int*)malloc(sizeof(int) * 2 * M);
    int64_t st[4] = {0, 0, 0, 0};
    if (!S || !order || !R) {
#pragma omp atomic write
      err = 1;
    } else {
#pragma omp for schedule(dynamic, 16)
      for (int64_t b = 0; b < nb; ++b) {
        int64_t r0 = (b / bc) * M, c0 = (b % bc) * M;
        round_block(key + r0 * cols + c0, cols, imp + r0 * cols + c0, cols, N, M, L, strict_paper, S, order,
                    R, R + M, st);
        for (int i = 0; i < M; ++i) memcpy(mask + (r0 + i) * cols + c0, S + i * M, M);
      }
#pragma omp critical
      for (int k = 0; k < 4; ++k) tot[k] += st[k];
    }
    free(S);
    free(order);
    free(R);
  }
  if (stats)
    for (int k = 0; k < 4; ++k) stats[k] = tot[k];
  return err ? -2 : 0;
}

/* Swap scores of Eq. (5) for one block and a given (i, j); -inf where the triple is invalid.
 * Exposed so that the printed score matrix of the worked example can be checked. */
int tsenor_oracle_swap_scores(const float* imp, const uint8_t* S, int M, int i, int j, double* score) {
  if (!imp || !S || !score || i < 0 || j < 0 || i >= M || j >= M) return -1;
  for (int ip = 0; ip < M; ++ip)
    for (int jp = 0; jp < M; ++jp) {
      if (!S[ip * M + jp] || S[i * M + jp] || S[ip * M + j])
        score[ip * M + jp] = -INFINITY;
      else
        score[ip * M + jp] = (double)imp[i * M + jp] + (double)imp[ip * M + j] - (double)imp[ip * M + jp];
    }
  return 0;
}

/* The whole path: importance -> tau_eff -> Algorithm 1 -> Algorithm 2.
 * W: rows x cols floats with leading dimension ld (bf16 inputs are widened by the caller, exactly).
 * plan_log (optional): rows x cols doubles, log S^(T).  tau_eff_out (optional). */
int tsenor_oracle_mask(const float* W, int64_t rows, int64_t cols, int64_t ld, const float* col_scale, int N,
                       int M, double tau, int tau_mode, int T, int L, int strict_paper, int cols_first,
                       uint8_t* mask, double* plan_log, double* tau_eff_out, int64_t* stats) {
  if (!W || !mask || M <= 0 || rows <= 0 || cols <= 0 || rows % M || cols % M || N < 0 || N > M || T < 0)
    return -1;
  if (N == 0 || N == M) { /* nothing to decide */
    memset(mask, N == 0 ? 0 : 1, (size_t)(rows * cols));
    if (stats) memset(stats, 0, 4 * sizeof(int64_t));
    return 0;
  }
  float* imp = (float*)malloc(sizeof(float) * rows * cols);
  double* ls = plan_log ? plan_log : (double*)malloc(sizeof(double) * rows * cols);
  int rc = -2;
  if (imp && ls) {
    rc = tsenor_oracle_importance(W, rows, cols, ld, col_scale, imp);
    if (!rc) {
      double te = tsenor_oracle_tau_eff(imp, rows, cols, tau, tau_mode);
      if (tau_eff_out) *tau_eff_out = te;
      rc = tsenor_oracle_dykstra(imp, rows, cols, N, M, te, T, cols_first, ls, NULL);
    }
    if (!rc) rc = tsenor_oracle_round(ls, imp, rows, cols, N, M, L, strict_paper, mask, stats);
  }
  free(imp);
  if (!plan_log) free(ls);
  return rc;
}

/* Importance with the transforms of Sec. 4 / Proposition 1, every step one float operation in this order:
 * x = W + add_scale * add;  a = |x|;  a = a * col_scale[j];  importance = a or a * a.
 * value (optional) receives x, the number a kept entry carries. */
int tsenor_oracle_importance_ex(const float* W, const float* add, float add_scale, int64_t rows, int64_t cols,
                                int64_t ld, const float* col_scale, int square, float* imp, float* value) {
  if (!W || !imp || rows <= 0 || cols <= 0 || ld < cols) return -1;
  for (int64_t i = 0; i < rows; ++i)
    for (int64_t j = 0; j < cols; ++j) {
      float x = W[i * ld + j];
      if (add) {
        volatile float t = add_scale * add[i * ld + j]; /* rounded product, then rounded sum: no fused multiply-add */
        x = x + t;
      }
      if (value) value[i * cols + j] = x;
      volatile float a = fabsf(x);
      if (col_scale) a = a * col_scale[j];
      if (square) a = a * a;
      imp[i * cols + j] = a;
    }
  return 0;
}

/* Objective of Eq. (1): sum of the importance the mask keeps, accumulated in double block by block. */
double tsenor_oracle_objective(const uint8_t* mask, const float* imp, int64_t rows, int64_t cols, int M) {
  double total = 0.0;
  for (int64_t r0 = 0; r0 < rows; r0 += M)
    for (int64_t c0 = 0; c0 < cols; c0 += M) {
      double blk = 0.0;
      for (int i = 0; i < M; ++i)
        for (int j = 0; j < M; ++j)
          if (mask[(r0 + i) * cols + c0 + j]) blk += (double)imp[(r0 + i) * cols + c0 + j];
      total += blk;
    }
  return total;
}
