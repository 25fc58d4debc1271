/* Runs the C oracle under AddressSanitizer / UndefinedBehaviorSanitizer on small inputs that
 * reach every code path: both set definitions (Eq. 11-12, Eq. 13), overlap, a short last
 * chunk, both stabilisers, a row subset, the feature map, the state and the chunk plan,
 * and the argument checks.  Prints "oracle sanitize ok" when every call returned what it
 * should. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int rehyat_oracle_chunk_plan(int T, int HW, int chunk, int overlap, int64_t *table, int *n_chunks);
int rehyat_oracle_phi(const double *x, int64_t n, int d, const double *w1, const double *b1, const double *w2,
                      const double *b2, int hidden, int dprime, int degree, double *out);
int rehyat_oracle_forward(const double *q, const double *k, const double *v, const double *w1_q,
                          const double *b1_q, const double *w2_q, const double *b2_q, const double *w1_k,
                          const double *b1_k, const double *w2_k, const double *b2_k, int hidden, int dprime,
                          int degree, int B, int H, int T, int HW, int d, int chunk, int overlap, int causal,
                          int stab, const int64_t *rows, int64_t n_rows, double *out, double *m, double *nS,
                          double *aS, double *nL, double *aL);
int rehyat_oracle_state(const double *k, const double *v, int64_t upto, int d, const double *w1,
                        const double *b1, const double *w2, const double *b2, int hidden, int dprime,
                        int degree, double *S, double *z);

static uint64_t rng = 88172645463325252ULL;
static double rnd(void) {
  rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17;
  return (double)(rng % 20001) / 10000.0 - 1.0;
}
static double *alloc_rnd(size_t n, double scale) {
  double *p = (double *)malloc(n * sizeof(double));
  for (size_t i = 0; i < n; ++i) p[i] = rnd() * scale;
  return p;
}
#define CHECK(c) do { if (!(c)) { printf("FAILED line %d: %s\n", __LINE__, #c); return 1; } } while (0)

int main(void) {
  const int B = 1, H = 2, T = 5, HW = 7, d = 8, hidden = 12, dp = 6;
  const int64_t N = (int64_t)T * HW;
  double *q = alloc_rnd((size_t)B * H * N * d, 1.0), *k = alloc_rnd((size_t)B * H * N * d, 1.0);
  double *v = alloc_rnd((size_t)B * H * N * d, 1.0);
  double *w1q = alloc_rnd((size_t)H * hidden * d, 0.5), *b1q = alloc_rnd((size_t)H * hidden, 0.5);
  double *w2q = alloc_rnd((size_t)H * dp * hidden, 0.5), *b2q = alloc_rnd((size_t)H * dp, 0.5);
  double *w1k = alloc_rnd((size_t)H * hidden * d, 0.5), *b1k = alloc_rnd((size_t)H * hidden, 0.5);
  double *w2k = alloc_rnd((size_t)H * dp * hidden, 0.5), *b2k = alloc_rnd((size_t)H * dp, 0.5);
  double *out = (double *)malloc((size_t)B * H * N * d * sizeof(double));
  double *m = (double *)malloc((size_t)B * H * N * sizeof(double)), *nS = (double *)malloc((size_t)B * H * N * sizeof(double));
  double *nL = (double *)malloc((size_t)B * H * N * sizeof(double));
  double *aS = (double *)malloc((size_t)B * H * N * d * sizeof(double)), *aL = (double *)malloc((size_t)B * H * N * d * sizeof(double));
  for (int causal = 0; causal < 2; ++causal)
    for (int stab = 0; stab < 2; ++stab)
      for (int chunk = 1; chunk <= 6; chunk += 1)
        for (int overlap = 0; overlap < 3; ++overlap) {
          int rc = rehyat_oracle_forward(q, k, v, w1q, b1q, w2q, b2q, w1k, b1k, w2k, b2k, hidden, dp, 2, B, H, T, HW,
                                         d, chunk, overlap, causal, stab, NULL, 0, out, m, nS, aS, nL, aL);
          CHECK(rc == 0);
          for (int64_t i = 0; i < B * H * N * d; ++i) CHECK(isfinite(out[i]));
          for (int64_t i = 0; i < B * H * N; ++i) CHECK(nL[i] >= 0.0 && nS[i] > 0.0);
        }
  /* a row subset (first, middle, last row), degree 3 features */
  {
    const int64_t rows[3] = {0, N / 2, N - 1};
    int rc = rehyat_oracle_forward(q, k, v, w1q, b1q, w2q, b2q, w1k, b1k, w2k, b2k, hidden, dp, 3, B, H, T, HW, d, 2,
                                   1, 1, 0, rows, 3, out, m, nS, aS, nL, aL);
    CHECK(rc == 0);
  }
  /* argument checks return errors and touch nothing */
  CHECK(rehyat_oracle_forward(q, k, v, w1q, b1q, w2q, b2q, w1k, b1k, w2k, b2k, hidden, dp, 4, B, H, T, HW, d, 1, 0,
                              1, 0, NULL, 0, out, m, nS, aS, nL, aL) != 0); /* dprime % degree != 0 */
  CHECK(rehyat_oracle_forward(q, k, v, w1q, b1q, w2q, b2q, w1k, b1k, w2k, b2k, hidden, dp, 2, B, H, 0, HW, d, 1, 0,
                              1, 0, NULL, 0, out, m, nS, aS, nL, aL) != 0);
  {
    double *phi = (double *)malloc((size_t)N * dp * sizeof(double));
    CHECK(rehyat_oracle_phi(k, N, d, w1k, b1k, w2k, b2k, hidden, dp, 2, phi) == 0);
    for (int64_t i = 0; i < N * dp; ++i) CHECK(phi[i] >= 0.0);
    free(phi);
  }
  {
    double *S = (double *)malloc((size_t)dp * d * sizeof(double)), *z = (double *)malloc((size_t)dp * sizeof(double));
    for (int64_t upto = 0; upto <= N; upto += HW) CHECK(rehyat_oracle_state(k, v, upto, d, w1k, b1k, w2k, b2k, hidden, dp, 2, S, z) == 0);
    free(S); free(z);
  }
  {
    int n = 0;
    int64_t table[5 * 64];
    CHECK(rehyat_oracle_chunk_plan(21, 1560, 2, 1, NULL, &n) == 0 && n == 11);
    CHECK(rehyat_oracle_chunk_plan(21, 1560, 2, 1, table, &n) == 0 && table[5 * 10 + 1] == 32760);
    CHECK(rehyat_oracle_chunk_plan(0, 1, 1, 0, NULL, &n) != 0);
  }
  free(q); free(k); free(v); free(w1q); free(b1q); free(w2q); free(b2q); free(w1k); free(b1k); free(w2k); free(b2k);
  free(out); free(m); free(nS); free(nL); free(aS); free(aL);
  printf("oracle sanitize ok\n");
  return 0;
}
