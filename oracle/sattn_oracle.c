/*
 * CPU oracle for sigmoid self-attention (and the softmax attention it is compared with).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of what the
 * GPU library must compute.  It shares no code, header, table or helper with the HIP
 * path, and the product never calls it: only the tests, the smoke check and the
 * cpu_baseline leg of the benchmark do.
 *
 * What is computed (paper: Section 2, the boxed sigmoid-attention equation; Appendix F.1,
 * the forward/backward table, right half for sigmoid and left half for softmax):
 *
 *   S = Q K^T / sqrt(d)                         scaled logits
 *   T = S + b - m_h * |i - j|                   bias b added after the scale; optional ALiBi
 *   P = sigmoid(T), P_ij = 0 where causal and j > i   (diagonal kept, Appendix G.1 mask)
 *   O = P V
 *   dV = P^T dO,  dP = dO V^T,  dS = P (1-P) dP (0 where masked)
 *   dQ = dS K / sqrt(d),  dK = dS^T Q / sqrt(d)
 *   db_i = sum_j dS_ij                          gradient of a bias added to row i of T; a
 *                                               scalar learnable b (Section 5.4, Appendix G.4:
 *                                               one per layer) gets the sum over its rows
 *
 * The table in Appendix F.1 and Algorithm 2 print the last two with a factor sqrt(d);
 * since S = Q K^T / sqrt(d) the chain rule gives 1/sqrt(d), which the finite-difference
 * pins confirm.  Algorithm 2's "dV_i += P_ij^T dO_j" and "dP_ij = dO_i V_i^T" are read
 * with the indices of the table: dV_j += P_ij^T dO_i and dP_ij = dO_i V_j^T.
 *
 * Softmax (comparison system): same S and ALiBi term, no b (a constant shift cancels),
 * masked logits are -inf, P = rowwise softmax, dS = P (dP - rowsum(dO o O)).
 *
 * Layout: every tensor is a contiguous [B, H, N, d] array of double.  Loops are over
 * (b,h), then rows i, then keys j, exactly as the definition reads; nothing is tiled.
 * OpenMP only spreads independent (b,h) heads, or independent requested rows, over cores.
 *
 * Parity pins (tests/test_oracle_*.py): closed forms for zero logits, the N=1 scalar case,
 * the exp(s)/(exp(s)+n) form of Section 2 (sequence equation), sigma(-x)=1-sigma(x)
 * symmetry, the Heaviside limit of Appendix C, additivity over key halves, central finite
 * differences (also in b, for the bias gradient), and PyTorch's fp64 CPU sigmoid/softmax/scaled_dot_product_attention with
 * autograd.  No function here is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double sigmoid_stable(double t) {
  if (t >= 0.0) return 1.0 / (1.0 + exp(-t));
  double e = exp(t);
  return e / (1.0 + e);
}

static double dot(const double* a, const double* b, int d) {
  double s = 0.0;
  for (int t = 0; t < d; ++t) s += a[t] * b[t];
  return s;
}

/* logit T_ij of one head (without masking) */
static double logit(const double* qi, const double* kj, int d, double bias, double slope, int i, int j) {
  double s = dot(qi, kj, d) / sqrt((double)d);
  return s + bias - slope * fabs((double)(i - j));
}

/* ---------------- sigmoid attention, one head ---------------- */

static void sig_row_probs(const double* q, const double* k, int N, int d, double bias, int causal, double slope,
                          int i, double* p) {
  for (int j = 0; j < N; ++j) {
    if (causal && j > i) { p[j] = 0.0; continue; }
    p[j] = sigmoid_stable(logit(q + (size_t)i * d, k + (size_t)j * d, d, bias, slope, i, j));
  }
}

static void sig_head_fwd(const double* q, const double* k, const double* v, double* o, int N, int d, double bias,
                         int causal, double slope) {
  double* p = (double*)malloc(sizeof(double) * (size_t)N);
  for (int i = 0; i < N; ++i) {
    sig_row_probs(q, k, N, d, bias, causal, slope, i, p);
    double* oi = o + (size_t)i * d;
    for (int t = 0; t < d; ++t) oi[t] = 0.0;
    for (int j = 0; j < N; ++j)
      for (int t = 0; t < d; ++t) oi[t] += p[j] * v[(size_t)j * d + t];
  }
  free(p);
}

static void sig_head_bwd(const double* q, const double* k, const double* v, const double* dout, double* dq,
                         double* dk, double* dv, int N, int d, double bias, int causal, double slope) {
  const double inv = 1.0 / sqrt((double)d);
  double* p = (double*)malloc(sizeof(double) * (size_t)N);
  memset(dq, 0, sizeof(double) * (size_t)N * d);
  memset(dk, 0, sizeof(double) * (size_t)N * d);
  memset(dv, 0, sizeof(double) * (size_t)N * d);
  for (int i = 0; i < N; ++i) {
    sig_row_probs(q, k, N, d, bias, causal, slope, i, p);
    const double* doi = dout + (size_t)i * d;
    const double* qi = q + (size_t)i * d;
    for (int j = 0; j < N; ++j) {
      if (causal && j > i) continue;
      double dp = dot(doi, v + (size_t)j * d, d);
      double ds = p[j] * (1.0 - p[j]) * dp;
      for (int t = 0; t < d; ++t) {
        dv[(size_t)j * d + t] += p[j] * doi[t];
        dq[(size_t)i * d + t] += inv * ds * k[(size_t)j * d + t];
        dk[(size_t)j * d + t] += inv * ds * qi[t];
      }
    }
  }
  free(p);
}

void oracle_sigmoid_attn_fwd(const double* q, const double* k, const double* v, double* o, int B, int H, int N,
                             int d, double bias, int causal, const double* alibi_slopes) {
  const size_t hs = (size_t)N * d;
#pragma omp parallel for schedule(dynamic, 1)
  for (int bh = 0; bh < B * H; ++bh) {
    double slope = alibi_slopes ? alibi_slopes[bh % H] : 0.0;
    sig_head_fwd(q + bh * hs, k + bh * hs, v + bh * hs, o + bh * hs, N, d, bias, causal, slope);
  }
}

void oracle_sigmoid_attn_bwd(const double* q, const double* k, const double* v, const double* dout, double* dq,
                             double* dk, double* dv, int B, int H, int N, int d, double bias, int causal,
                             const double* alibi_slopes) {
  const size_t hs = (size_t)N * d;
#pragma omp parallel for schedule(dynamic, 1)
  for (int bh = 0; bh < B * H; ++bh) {
    double slope = alibi_slopes ? alibi_slopes[bh % H] : 0.0;
    sig_head_bwd(q + bh * hs, k + bh * hs, v + bh * hs, dout + bh * hs, dq + bh * hs, dk + bh * hs, dv + bh * hs,
                 N, d, bias, causal, slope);
  }
}

/* Row sums of dS: T_ij = S_ij + b, so dL/db collects dL/dT_ij = dS_ij over every unmasked
 * pair the bias enters; db_rows[bh][i] = sum_j dS_ij keeps the rows apart. */
void oracle_sigmoid_attn_bias_grad(const double* q, const double* k, const double* v, const double* dout,
                                   double* db_rows, int B, int H, int N, int d, double bias, int causal,
                                   const double* alibi_slopes) {
  const size_t hs = (size_t)N * d;
#pragma omp parallel for schedule(dynamic, 1)
  for (int bh = 0; bh < B * H; ++bh) {
    double slope = alibi_slopes ? alibi_slopes[bh % H] : 0.0;
    double* p = (double*)malloc(sizeof(double) * (size_t)N);
    for (int i = 0; i < N; ++i) {
      sig_row_probs(q + bh * hs, k + bh * hs, N, d, bias, causal, slope, i, p);
      double acc = 0.0;
      for (int j = 0; j < N; ++j) {
        if (causal && j > i) continue;
        double dp = dot(dout + bh * hs + (size_t)i * d, v + bh * hs + (size_t)j * d, d);
        acc += p[j] * (1.0 - p[j]) * dp;
      }
      db_rows[(size_t)bh * N + i] = acc;
    }
    free(p);
  }
}

/* ---------------- sampled rows of one head (for sizes where a full pass is too slow) --------
 * q,k,v,dout point at one head's [N,d] slice.  rows[] lists query indices (fwd, dq) or key
 * indices (dk, dv).  Each requested row is recomputed from the definition independently. */

void oracle_sigmoid_attn_fwd_rows(const double* q, const double* k, const double* v, int N, int d, double bias,
                                  int causal, double slope, const int* rows, int nrows, double* o_rows) {
#pragma omp parallel for schedule(dynamic, 1)
  for (int r = 0; r < nrows; ++r) {
    int i = rows[r];
    double* p = (double*)malloc(sizeof(double) * (size_t)N);
    sig_row_probs(q, k, N, d, bias, causal, slope, i, p);
    double* oi = o_rows + (size_t)r * d;
    for (int t = 0; t < d; ++t) oi[t] = 0.0;
    for (int j = 0; j < N; ++j)
      for (int t = 0; t < d; ++t) oi[t] += p[j] * v[(size_t)j * d + t];
    free(p);
  }
}

void oracle_sigmoid_attn_dq_rows(const double* q, const double* k, const double* v, const double* dout, int N,
                                 int d, double bias, int causal, double slope, const int* rows, int nrows,
                                 double* dq_rows) {
  const double inv = 1.0 / sqrt((double)d);
#pragma omp parallel for schedule(dynamic, 1)
  for (int r = 0; r < nrows; ++r) {
    int i = rows[r];
    double* p = (double*)malloc(sizeof(double) * (size_t)N);
    sig_row_probs(q, k, N, d, bias, causal, slope, i, p);
    double* out = dq_rows + (size_t)r * d;
    for (int t = 0; t < d; ++t) out[t] = 0.0;
    for (int j = 0; j < N; ++j) {
      if (causal && j > i) continue;
      double dp = dot(dout + (size_t)i * d, v + (size_t)j * d, d);
      double ds = p[j] * (1.0 - p[j]) * dp;
      for (int t = 0; t < d; ++t) out[t] += inv * ds * k[(size_t)j * d + t];
    }
    free(p);
  }
}

void oracle_sigmoid_attn_dkdv_rows(const double* q, const double* k, const double* v, const double* dout, int N,
                                   int d, double bias, int causal, double slope, const int* rows, int nrows,
                                   double* dk_rows, double* dv_rows) {
  const double inv = 1.0 / sqrt((double)d);
#pragma omp parallel for schedule(dynamic, 1)
  for (int r = 0; r < nrows; ++r) {
    int j = rows[r];
    double* ok = dk_rows + (size_t)r * d;
    double* ov = dv_rows + (size_t)r * d;
    for (int t = 0; t < d; ++t) { ok[t] = 0.0; ov[t] = 0.0; }
    for (int i = 0; i < N; ++i) {
      if (causal && j > i) continue;
      double p = sigmoid_stable(logit(q + (size_t)i * d, k + (size_t)j * d, d, bias, slope, i, j));
      double dp = dot(dout + (size_t)i * d, v + (size_t)j * d, d);
      double ds = p * (1.0 - p) * dp;
      for (int t = 0; t < d; ++t) {
        ov[t] += p * dout[(size_t)i * d + t];
        ok[t] += inv * ds * q[(size_t)i * d + t];
      }
    }
  }
}

/* ---------------- softmax attention (comparison system), one head ---------------- */

/* p[j] = softmax_j of row i; returns the row's log-sum-exp (natural log) */
static double soft_row_probs(const double* q, const double* k, int N, int d, int causal, double slope, int i,
                             double* p) {
  double mx = -INFINITY;
  for (int j = 0; j < N; ++j) {
    if (causal && j > i) { p[j] = -INFINITY; continue; }
    p[j] = logit(q + (size_t)i * d, k + (size_t)j * d, d, 0.0, slope, i, j);
    if (p[j] > mx) mx = p[j];
  }
  double sum = 0.0;
  for (int j = 0; j < N; ++j) {
    p[j] = (p[j] == -INFINITY) ? 0.0 : exp(p[j] - mx);
    sum += p[j];
  }
  for (int j = 0; j < N; ++j) p[j] /= sum;
  return mx + log(sum);
}

static void soft_head_fwd(const double* q, const double* k, const double* v, double* o, double* lse, int N, int d,
                          int causal, double slope) {
  double* p = (double*)malloc(sizeof(double) * (size_t)N);
  for (int i = 0; i < N; ++i) {
    double l = soft_row_probs(q, k, N, d, causal, slope, i, p);
    if (lse) lse[i] = l;
    double* oi = o + (size_t)i * d;
    for (int t = 0; t < d; ++t) oi[t] = 0.0;
    for (int j = 0; j < N; ++j)
      for (int t = 0; t < d; ++t) oi[t] += p[j] * v[(size_t)j * d + t];
  }
  free(p);
}

static void soft_head_bwd(const double* q, const double* k, const double* v, const double* dout, double* dq,
                          double* dk, double* dv, int N, int d, int causal, double slope) {
  const double inv = 1.0 / sqrt((double)d);
  double* p = (double*)malloc(sizeof(double) * (size_t)N);
  double* oi = (double*)malloc(sizeof(double) * (size_t)d);
  memset(dq, 0, sizeof(double) * (size_t)N * d);
  memset(dk, 0, sizeof(double) * (size_t)N * d);
  memset(dv, 0, sizeof(double) * (size_t)N * d);
  for (int i = 0; i < N; ++i) {
    soft_row_probs(q, k, N, d, causal, slope, i, p);
    const double* doi = dout + (size_t)i * d;
    const double* qi = q + (size_t)i * d;
    /* O_i and rowsum(dO o O)_i */
    for (int t = 0; t < d; ++t) oi[t] = 0.0;
    for (int j = 0; j < N; ++j)
      for (int t = 0; t < d; ++t) oi[t] += p[j] * v[(size_t)j * d + t];
    double D = dot(doi, oi, d);
    for (int j = 0; j < N; ++j) {
      if (causal && j > i) continue;
      double dp = dot(doi, v + (size_t)j * d, d);
      double ds = p[j] * (dp - D);
      for (int t = 0; t < d; ++t) {
        dv[(size_t)j * d + t] += p[j] * doi[t];
        dq[(size_t)i * d + t] += inv * ds * k[(size_t)j * d + t];
        dk[(size_t)j * d + t] += inv * ds * qi[t];
      }
    }
  }
  free(p);
  free(oi);
}

void oracle_softmax_attn_fwd(const double* q, const double* k, const double* v, double* o, double* lse, int B,
                             int H, int N, int d, int causal, const double* alibi_slopes) {
  const size_t hs = (size_t)N * d;
#pragma omp parallel for schedule(dynamic, 1)
  for (int bh = 0; bh < B * H; ++bh) {
    double slope = alibi_slopes ? alibi_slopes[bh % H] : 0.0;
    soft_head_fwd(q + bh * hs, k + bh * hs, v + bh * hs, o + bh * hs, lse ? lse + (size_t)bh * N : NULL, N, d,
                  causal, slope);
  }
}

void oracle_softmax_attn_bwd(const double* q, const double* k, const double* v, const double* dout, double* dq,
                             double* dk, double* dv, int B, int H, int N, int d, int causal,
                             const double* alibi_slopes) {
  const size_t hs = (size_t)N * d;
#pragma omp parallel for schedule(dynamic, 1)
  for (int bh = 0; bh < B * H; ++bh) {
    double slope = alibi_slopes ? alibi_slopes[bh % H] : 0.0;
    soft_head_bwd(q + bh * hs, k + bh * hs, v + bh * hs, dout + bh * hs, dq + bh * hs, dk + bh * hs, dv + bh * hs,
                  N, d, causal, slope);
  }
}

void oracle_softmax_attn_fwd_rows(const double* q, const double* k, const double* v, int N, int d, int causal,
                                  double slope, const int* rows, int nrows, double* o_rows, double* lse_rows) {
#pragma omp parallel for schedule(dynamic, 1)
  for (int r = 0; r < nrows; ++r) {
    int i = rows[r];
    double* p = (double*)malloc(sizeof(double) * (size_t)N);
    double l = soft_row_probs(q, k, N, d, causal, slope, i, p);
    if (lse_rows) lse_rows[r] = l;
    double* oi = o_rows + (size_t)r * d;
    for (int t = 0; t < d; ++t) oi[t] = 0.0;
    for (int j = 0; j < N; ++j)
      for (int t = 0; t < d; ++t) oi[t] += p[j] * v[(size_t)j * d + t];
    free(p);
  }
}

int oracle_num_threads(void) {
  int n = 1;
#ifdef _OPENMP
#pragma omp parallel
  {
#pragma omp master
    n = omp_get_num_threads();
  }
#endif
  return n;
}
