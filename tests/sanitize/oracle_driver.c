/* Calls every entry point of the CPU oracle on small, ragged problems with exactly sized heap
 * buffers, for a build with -fsanitize=address,undefined: an index slip in the oracle shows up
 * as a sanitizer report.  Test infrastructure; prints one checksum per call. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

void oracle_sigmoid_attn_fwd(const double*, const double*, const double*, double*, int, int, int, int, double, int, const double*);
void oracle_sigmoid_attn_bwd(const double*, const double*, const double*, const double*, double*, double*, double*, int, int, int, int, double, int, const double*);
void oracle_sigmoid_attn_bias_grad(const double*, const double*, const double*, const double*, double*, int, int, int, int, double, int, const double*);
void oracle_sigmoid_attn_fwd_rows(const double*, const double*, const double*, int, int, double, int, double, const int*, int, double*);
void oracle_sigmoid_attn_dq_rows(const double*, const double*, const double*, const double*, int, int, double, int, double, const int*, int, double*);
void oracle_sigmoid_attn_dkdv_rows(const double*, const double*, const double*, const double*, int, int, double, int, double, const int*, int, double*, double*);
void oracle_softmax_attn_fwd(const double*, const double*, const double*, double*, double*, int, int, int, int, int, const double*);
void oracle_softmax_attn_bwd(const double*, const double*, const double*, const double*, double*, double*, double*, int, int, int, int, int, const double*);
void oracle_softmax_attn_fwd_rows(const double*, const double*, const double*, int, int, int, double, const int*, int, double*, double*);
int oracle_num_threads(void);

static double* rnd(size_t n, unsigned* seed) {
  double* p = (double*)malloc(n * sizeof(double));
  for (size_t i = 0; i < n; ++i) {
    *seed = *seed * 1664525u + 1013904223u;
    p[i] = ((double)(*seed >> 8) / (double)(1u << 24)) * 2.0 - 1.0;
  }
  return p;
}
static double sum(const double* p, size_t n) {
  double s = 0;
  for (size_t i = 0; i < n; ++i) s += p[i];
  return s;
}

int main(void) {
  unsigned seed = 12345u;
  const int shapes[4][4] = {{1, 1, 1, 1}, {2, 3, 37, 8}, {1, 2, 5, 3}, {1, 1, 64, 16}};
  for (int s = 0; s < 4; ++s) {
    const int B = shapes[s][0], H = shapes[s][1], N = shapes[s][2], d = shapes[s][3];
    const size_t n = (size_t)B * H * N * d, hs = (size_t)N * d;
    double *q = rnd(n, &seed), *k = rnd(n, &seed), *v = rnd(n, &seed), *g = rnd(n, &seed), *sl = rnd(H, &seed);
    double *o = malloc(n * 8), *dq = malloc(n * 8), *dk = malloc(n * 8), *dv = malloc(n * 8);
    double *lse = malloc((size_t)B * H * N * 8), *db = malloc((size_t)B * H * N * 8);
    for (int h = 0; h < H; ++h) sl[h] = fabs(sl[h]);
    for (int causal = 0; causal < 2; ++causal)
      for (int alibi = 0; alibi < 2; ++alibi) {
        const double* slp = alibi ? sl : NULL;
        oracle_sigmoid_attn_fwd(q, k, v, o, B, H, N, d, -log(N + 1.0), causal, slp);
        oracle_sigmoid_attn_bwd(q, k, v, g, dq, dk, dv, B, H, N, d, -0.3, causal, slp);
        oracle_sigmoid_attn_bias_grad(q, k, v, g, db, B, H, N, d, -0.3, causal, slp);
        printf("sig %d %d %d: %.6g %.6g %.6g %.6g %.6g\n", s, causal, alibi, sum(o, n), sum(dq, n), sum(dk, n), sum(dv, n),
               sum(db, (size_t)B * H * N));
        oracle_softmax_attn_fwd(q, k, v, o, lse, B, H, N, d, causal, slp);
        oracle_softmax_attn_bwd(q, k, v, g, dq, dk, dv, B, H, N, d, causal, slp);
        printf("soft %d %d %d: %.6g %.6g %.6g %.6g %.6g\n", s, causal, alibi, sum(o, n), sum(lse, (size_t)B * H * N),
               sum(dq, n), sum(dk, n), sum(dv, n));
        /* sampled rows of the last head: first, middle, last row (and a repeated one) */
        int rows[4] = {0, N / 2, N - 1, 0};
        double *ro = malloc(4 * d * 8), *rk = malloc(4 * d * 8), *rv = malloc(4 * d * 8), *rl = malloc(4 * 8);
        const size_t off = ((size_t)B * H - 1) * hs;
        const double slope = alibi ? sl[H - 1] : 0.0;
        oracle_sigmoid_attn_fwd_rows(q + off, k + off, v + off, N, d, -0.3, causal, slope, rows, 4, ro);
        oracle_sigmoid_attn_dq_rows(q + off, k + off, v + off, g + off, N, d, -0.3, causal, slope, rows, 4, rk);
        oracle_sigmoid_attn_dkdv_rows(q + off, k + off, v + off, g + off, N, d, -0.3, causal, slope, rows, 4, rk, rv);
        oracle_softmax_attn_fwd_rows(q + off, k + off, v + off, N, d, causal, slope, rows, 4, ro, rl);
        printf("rows %d %d %d: %.6g %.6g %.6g %.6g\n", s, causal, alibi, sum(ro, 4 * d), sum(rk, 4 * d), sum(rv, 4 * d), sum(rl, 4));
        free(ro); free(rk); free(rv); free(rl);
      }
    free(q); free(k); free(v); free(g); free(sl); free(o); free(dq); free(dk); free(dv); free(lse); free(db);
  }
  printf("threads %d\nok\n", oracle_num_threads());
  return 0;
}
