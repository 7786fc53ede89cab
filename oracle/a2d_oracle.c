/*
 * fp64 CPU oracle for the per-device compute of Attention2D (arXiv 2503.15758).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * GPU library must compute.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it; the product path never does.  It shares no code
 * with the HIP kernels.
 *
 * Every function is the paper's definition written out element by element:
 *   - attention_fwd / attention_bwd : Sec. 2.1, Eq. (1)-(2) (+ the 1/sqrt(H)
 *     scale the paper's footnote in Sec. 2.1 leaves out, passed explicitly) and
 *     the textbook gradient of that expression,
 *   - partial_fwd                   : Sec. 3.1, Eq. (3),
 *   - partial_fwd_pos / _bwd_pos    : the same tile computations when the keys of the tile
 *                                     carry arbitrary global positions (the gathered K_g, V_g
 *                                     of Alg. GatherComputeScatter line "Compute", whose
 *                                     sub-blocks come from different devices; Sec. 4.1 names the
 *                                     resulting step-like mask),
 *   - attnfix_pair                  : Alg. 2 (AttnFix),
 *   - fix                           : Alg. 2 folded over k partials followed by
 *                                     O = Diag(D^-1) N (Alg. 1, line 6) and
 *                                     L = M + log D (footnote in Sec. 3.2),
 *   - partial_bwd                   : the per-tile gradient call of Alg. 3, line 3,
 *   - fix_bwd                       : the summing reductions of Alg. 3, lines 4-5.
 *
 * Layout of every matrix argument: [heads][rows][H], H contiguous, fp64.
 * Per-row vectors: [heads][rows].  Heads are independent (the paper works per
 * head).  The causal mask is x_{i,r} = -inf iff (q_off+i) < (kv_off+r), with
 * q_off / kv_off the global index of row 0 / key 0 of the tile (Sec. 2.1).
 *
 * Conventions where the paper is silent:
 *   - a row that sees no key in a tile has m = -inf, d = 0, n = 0;
 *   - AttnFix gives weight 0 to a partial whose m is -inf (never forms
 *     -inf - (-inf)); if every partial is empty the merged row is O = 0,
 *     lse = -inf.
 *
 * Pins: tests/test_oracle_*.py check these functions against closed forms,
 * brute force in pure Python, torch's fp64 CPU attention + autograd, finite
 * differences and the partition identities of Sec. 3.1.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int a2d_oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* s_{i,r} = scale * sum_h q_{i,h} k_{r,h} + x_{i,r}   (Sec. 2.1, element form) */
static double score(const double* q, const double* k, int H, double scale,
                    int causal, int64_t gi, int64_t gr) {
  if (causal && gi < gr) return -INFINITY;
  double s = 0.0;
  for (int h = 0; h < H; ++h) s += q[h] * k[h];
  return scale * s;
}

/* ------------------------------------------------------------------------- */
/* Sec. 2.1, Eq. (1)-(2): full attention of one sequence of n tokens.         */
/* O [heads][n][H], lse [heads][n] (= m_i + log d_i), P optional [heads][n][n] */
void a2d_oracle_attention_fwd(int heads, int n, int H, const double* Q,
                              const double* K, const double* V, double scale,
                              int causal, double* O, double* lse, double* P) {
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
  for (int b = 0; b < heads; ++b) {
    for (int i = 0; i < n; ++i) {
      const double* q = Q + ((size_t)b * n + i) * H;
      double* s = (double*)malloc(sizeof(double) * (size_t)n);
      double m = -INFINITY;
      for (int r = 0; r < n; ++r) {
        s[r] = score(q, K + ((size_t)b * n + r) * H, H, scale, causal, i, r);
        if (s[r] > m) m = s[r];
      }
      double d = 0.0;
      for (int r = 0; r < n; ++r) {
        s[r] = (s[r] == -INFINITY) ? 0.0 : exp(s[r] - m);
        d += s[r];
      }
      double* o = O + ((size_t)b * n + i) * H;
      for (int j = 0; j < H; ++j) o[j] = 0.0;
      for (int r = 0; r < n; ++r) {
        const double* v = V + ((size_t)b * n + r) * H;
        double p = s[r] / d;
        if (P) P[((size_t)b * n + i) * n + r] = p;
        for (int j = 0; j < H; ++j) o[j] += p * v[j];
      }
      lse[(size_t)b * n + i] = m + log(d);
      free(s);
    }
  }
}

/* ------------------------------------------------------------------------- */
/* Gradient of Eq. (1)-(2) with respect to Q, K, V given dO (textbook form):   */
/*   P = Softmax(S), dV = P^T dO, dP = dO V^T,                                 */
/*   dS_{i,r} = P_{i,r} (dP_{i,r} - sum_t P_{i,t} dP_{i,t}),                   */
/*   dQ = scale dS K, dK = scale dS^T Q.                                        */
/* Pass A walks query rows (dQ and the per-row sums), pass B walks key rows    */
/* (dK, dV), so every output element is written by exactly one loop iteration. */
void a2d_oracle_attention_bwd(int heads, int n, int H, const double* Q,
                              const double* K, const double* V,
                              const double* dO, double scale, int causal,
                              double* dQ, double* dK, double* dV) {
  size_t rows = (size_t)heads * n;
  double* rm = (double*)malloc(sizeof(double) * rows);   /* m_i           */
  double* rd = (double*)malloc(sizeof(double) * rows);   /* d_i           */
  double* rc = (double*)malloc(sizeof(double) * rows);   /* sum_t P dP    */
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
  for (int b = 0; b < heads; ++b) {
    for (int i = 0; i < n; ++i) {
      size_t row = (size_t)b * n + i;
      const double* q = Q + row * H;
      const double* go = dO + row * H;
      double* p = (double*)malloc(sizeof(double) * (size_t)n);
      double* dp = (double*)malloc(sizeof(double) * (size_t)n);
      double m = -INFINITY;
      for (int r = 0; r < n; ++r) {
        p[r] = score(q, K + ((size_t)b * n + r) * H, H, scale, causal, i, r);
        if (p[r] > m) m = p[r];
      }
      double d = 0.0;
      for (int r = 0; r < n; ++r) {
        p[r] = (p[r] == -INFINITY) ? 0.0 : exp(p[r] - m);
        d += p[r];
      }
      double c = 0.0;
      for (int r = 0; r < n; ++r) {
        const double* v = V + ((size_t)b * n + r) * H;
        p[r] /= d;
        double t = 0.0;
        for (int j = 0; j < H; ++j) t += go[j] * v[j];
        dp[r] = t;
        c += p[r] * t;
      }
      double* gq = dQ + row * H;
      for (int h = 0; h < H; ++h) gq[h] = 0.0;
      for (int r = 0; r < n; ++r) {
        const double* k = K + ((size_t)b * n + r) * H;
        double ds = p[r] * (dp[r] - c);
        for (int h = 0; h < H; ++h) gq[h] += scale * ds * k[h];
      }
      rm[row] = m; rd[row] = d; rc[row] = c;
      free(p); free(dp);
    }
  }
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
  for (int b = 0; b < heads; ++b) {
    for (int r = 0; r < n; ++r) {
      size_t krow = (size_t)b * n + r;
      const double* k = K + krow * H;
      const double* v = V + krow * H;
      double* gk = dK + krow * H;
      double* gv = dV + krow * H;
      for (int h = 0; h < H; ++h) { gk[h] = 0.0; gv[h] = 0.0; }
      for (int i = 0; i < n; ++i) {
        size_t row = (size_t)b * n + i;
        const double* q = Q + row * H;
        const double* go = dO + row * H;
        double s = score(q, k, H, scale, causal, i, r);
        if (s == -INFINITY) continue;
        double p = exp(s - rm[row]) / rd[row];
        double dp = 0.0;
        for (int j = 0; j < H; ++j) dp += go[j] * v[j];
        double ds = p * (dp - rc[row]);
        for (int h = 0; h < H; ++h) {
          gv[h] += p * go[h];
          gk[h] += scale * ds * q[h];
        }
      }
    }
  }
  free(rm); free(rd); free(rc);
}

/* ------------------------------------------------------------------------- */
/* Sec. 3.1, Eq. (3): attention of a block of queries restricted to the keys   */
/* R_x of one tile.  N [heads][nq][H] unnormalised, m, d [heads][nq].          */
/* kpos[r] is the global index of key r of the tile: key r is hidden from      */
/* query i iff causal and q_off + i < kpos[r] (Sec. 2.1).                      */
void a2d_oracle_partial_fwd_pos(int heads, int nq, int nkv, int H, const double* Q,
                                const double* K, const double* V, int64_t q_off,
                                const int64_t* kpos, int causal, double scale,
                                double* N, double* m_out, double* d_out) {
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
  for (int b = 0; b < heads; ++b) {
    for (int i = 0; i < nq; ++i) {
      size_t row = (size_t)b * nq + i;
      const double* q = Q + row * H;
      double* s = (double*)malloc(sizeof(double) * (size_t)(nkv > 0 ? nkv : 1));
      double m = -INFINITY;
      for (int r = 0; r < nkv; ++r) {
        s[r] = score(q, K + ((size_t)b * nkv + r) * H, H, scale, causal,
                     q_off + i, kpos[r]);
        if (s[r] > m) m = s[r];
      }
      double* nrow = N + row * H;
      for (int j = 0; j < H; ++j) nrow[j] = 0.0;
      double d = 0.0;
      if (m != -INFINITY) {
        for (int r = 0; r < nkv; ++r) {
          if (s[r] == -INFINITY) continue;
          const double* v = V + ((size_t)b * nkv + r) * H;
          double e = exp(s[r] - m);
          d += e;
          for (int j = 0; j < H; ++j) nrow[j] += e * v[j];
        }
      }
      m_out[row] = m;
      d_out[row] = d;
      free(s);
    }
  }
}

/* global key indices of a tile whose keys are consecutive tokens from kv_off */
static int64_t* consecutive_positions(int nkv, int64_t kv_off) {
  int64_t* kpos = (int64_t*)malloc(sizeof(int64_t) * (size_t)(nkv > 0 ? nkv : 1));
  for (int r = 0; r < nkv; ++r) kpos[r] = kv_off + r;
  return kpos;
}

/* The tile of consecutive tokens: key r is token kv_off + r. */
void a2d_oracle_partial_fwd(int heads, int nq, int nkv, int H, const double* Q,
                            const double* K, const double* V, int64_t q_off,
                            int64_t kv_off, int causal, double scale,
                            double* N, double* m_out, double* d_out) {
  int64_t* kpos = consecutive_positions(nkv, kv_off);
  a2d_oracle_partial_fwd_pos(heads, nq, nkv, H, Q, K, V, q_off, kpos, causal, scale, N, m_out, d_out);
  free(kpos);
}

/* ------------------------------------------------------------------------- */
/* Alg. 2 (AttnFix): combine two partial outputs, row by row.                   */
void a2d_oracle_attnfix_pair(int64_t rows, int H, const double* M1,
                             const double* N1, const double* D1,
                             const double* M2, const double* N2,
                             const double* D2, double* M, double* N,
                             double* D) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < rows; ++i) {
    double m = M1[i] > M2[i] ? M1[i] : M2[i];
    double e1 = (M1[i] == -INFINITY) ? 0.0 : exp(M1[i] - m);
    double e2 = (M2[i] == -INFINITY) ? 0.0 : exp(M2[i] - m);
    for (int j = 0; j < H; ++j)
      N[i * H + j] = e1 * N1[i * H + j] + e2 * N2[i * H + j];
    D[i] = e1 * D1[i] + e2 * D2[i];
    M[i] = m;
  }
}

/* Alg. 2 over k partials in ONE pass (M = max over all partials, each weighted  */
/* exp(M_x - M), sums in index order; by the associativity of Sec. 3.1 this is  */
/* the pairwise fold of Alg. 2, which a pin checks), then Alg. 1 line 6 and the */
/* log-sum-exp statistic.  parts are arrays of k pointers.                      */
void a2d_oracle_fix(int k, int64_t rows, int H, const double* const* Nparts,
                    const double* const* Mparts, const double* const* Dparts,
                    double* O, double* lse) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < rows; ++i) {
    double m = -INFINITY;
    for (int x = 0; x < k; ++x)
      if (Mparts[x][i] > m) m = Mparts[x][i];
    double d = 0.0;
    double* o = O + i * H;
    for (int j = 0; j < H; ++j) o[j] = 0.0;
    for (int x = 0; x < k; ++x) {
      if (Mparts[x][i] == -INFINITY) continue;
      double e = exp(Mparts[x][i] - m);
      d += e * Dparts[x][i];
      for (int j = 0; j < H; ++j) o[j] += e * Nparts[x][i * H + j];
    }
    if (d > 0.0) {
      for (int j = 0; j < H; ++j) o[j] /= d;
      lse[i] = m + log(d);
    } else {
      lse[i] = -INFINITY;
    }
  }
}

/* ------------------------------------------------------------------------- */
/* Alg. 3 line 3 for one tile: gradients of the tile's share of the scores,    */
/* using the FINAL merged O and lse of the query block (the saved set of       */
/* Alg. 1 line 7):  P_{i,r} = exp(s_{i,r} - lse_i),  delta_i = sum_j dO O,     */
/* dV = P^T dO, dP = dO V^T, dS = P o (dP - delta), dQ = scale dS K,           */
/* dK = scale dS^T Q.                                                           */
/* kpos[r]: global index of key r, as in partial_fwd_pos.                       */
void a2d_oracle_partial_bwd_pos(int heads, int nq, int nkv, int H, const double* Q,
                                const double* K, const double* V, const double* O,
                                const double* dO, const double* lse, int64_t q_off,
                                const int64_t* kpos, int causal, double scale,
                                double* dQ, double* dK, double* dV) {
  size_t rows = (size_t)heads * nq;
  double* delta = (double*)malloc(sizeof(double) * (rows ? rows : 1));
#pragma omp parallel for schedule(static)
  for (int64_t row = 0; row < (int64_t)rows; ++row) {
    double t = 0.0;
    for (int j = 0; j < H; ++j) t += dO[row * H + j] * O[row * H + j];
    delta[row] = t;
  }
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
  for (int b = 0; b < heads; ++b) {
    for (int i = 0; i < nq; ++i) {
      size_t row = (size_t)b * nq + i;
      const double* q = Q + row * H;
      const double* go = dO + row * H;
      double* gq = dQ + row * H;
      for (int h = 0; h < H; ++h) gq[h] = 0.0;
      if (lse[row] == -INFINITY) continue;
      for (int r = 0; r < nkv; ++r) {
        const double* k = K + ((size_t)b * nkv + r) * H;
        const double* v = V + ((size_t)b * nkv + r) * H;
        double s = score(q, k, H, scale, causal, q_off + i, kpos[r]);
        if (s == -INFINITY) continue;
        double p = exp(s - lse[row]);
        double dp = 0.0;
        for (int j = 0; j < H; ++j) dp += go[j] * v[j];
        double ds = p * (dp - delta[row]);
        for (int h = 0; h < H; ++h) gq[h] += scale * ds * k[h];
      }
    }
  }
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
  for (int b = 0; b < heads; ++b) {
    for (int r = 0; r < nkv; ++r) {
      size_t krow = (size_t)b * nkv + r;
      const double* k = K + krow * H;
      const double* v = V + krow * H;
      double* gk = dK + krow * H;
      double* gv = dV + krow * H;
      for (int h = 0; h < H; ++h) { gk[h] = 0.0; gv[h] = 0.0; }
      for (int i = 0; i < nq; ++i) {
        size_t row = (size_t)b * nq + i;
        if (lse[row] == -INFINITY) continue;
        const double* q = Q + row * H;
        const double* go = dO + row * H;
        double s = score(q, k, H, scale, causal, q_off + i, kpos[r]);
        if (s == -INFINITY) continue;
        double p = exp(s - lse[row]);
        double dp = 0.0;
        for (int j = 0; j < H; ++j) dp += go[j] * v[j];
        double ds = p * (dp - delta[row]);
        for (int h = 0; h < H; ++h) {
          gv[h] += p * go[h];
          gk[h] += scale * ds * q[h];
        }
      }
    }
  }
  free(delta);
}

/* The tile of consecutive tokens: key r is token kv_off + r. */
void a2d_oracle_partial_bwd(int heads, int nq, int nkv, int H, const double* Q,
                            const double* K, const double* V, const double* O,
                            const double* dO, const double* lse, int64_t q_off,
                            int64_t kv_off, int causal, double scale,
                            double* dQ, double* dK, double* dV) {
  int64_t* kpos = consecutive_positions(nkv, kv_off);
  a2d_oracle_partial_bwd_pos(heads, nq, nkv, H, Q, K, V, O, dO, lse, q_off, kpos, causal, scale,
                             dQ, dK, dV);
  free(kpos);
}

/* Alg. 3 lines 4-5: the gradient partials of a grid row / column are summed.  */
void a2d_oracle_fix_bwd(int k, int64_t n, const double* const* parts,
                        double* out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    double t = 0.0;
    for (int x = 0; x < k; ++x) t += parts[x][i];
    out[i] = t;
  }
}
