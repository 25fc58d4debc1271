/*
 * TEST INFRASTRUCTURE -- fp64 CPU oracle for the Recurrent Hybrid Attention
 * operator (ReHyAt).  Plain, slow, written from the paper's definitions; it is
 * independent of the GPU library (no shared code, headers, tables or helpers)
 * and may be called only from tests, the smoke check and the cpu_baseline leg
 * of the benchmark.
 *
 * What it evaluates (paper section 3.2 "Hybrid Attention Formulation" and
 * section 3.3 "Recurrent HyAt"):
 *
 *   y_i = (a^S_i + a^L_i) / (n^S_i + n^L_i)                       (Eq. 5)
 *   a^S_i = sum_{j in T^S_t} exp(q_i.k_j/sqrt(d) - c_i) v_j        (Eq. 6)
 *   a^L_i = phi_q(q_i) . sum_{j in T^L_t} phi_k(k_j) v_j^T         (Eq. 7)
 *   n^S_i = sum_{j in T^S_t} exp(q_i.k_j/sqrt(d) - c_i)            (Eq. 8)
 *   n^L_i = phi_q(q_i) . sum_{j in T^L_t} phi_k(k_j)               (Eq. 9)
 *
 * with t the chunk of token i, T^S_t the overlapping softmax window of Eq. 12
 * and T^L_t either every earlier token (Eq. 13, causal) or every token outside
 * the window (Eq. 11/12, bidirectional).  The causal form is evaluated as the
 * chunk-wise RNN of Eq. 14-18: a running state S (D' x d) and z (D') that
 * absorbs tokens as they leave the softmax window.
 *
 * Readings of points the paper leaves open (all switchable or stated):
 *   - c_i is per query row: the largest exponent of that row (stab = 0), or
 *     zero (stab = 1).  The output depends on this choice because the linear
 *     terms are not rescaled.                     [parity unpinned by the paper]
 *   - 1/sqrt(D) uses the per-head width d.        [parity unpinned by the paper]
 *   - phi: u = relu(W1 x + b1), psi = relu(W2 u + b2), psi split into `degree`
 *     equal parts, part p (1-based) raised element-wise to the power p
 *     ("Characterization of phi").  ReLU is one non-negative choice; the paper
 *     does not name the activation.              [parity unpinned by the paper]
 *   - Eq. 17-18 as printed would re-add what s_t already holds; the reading
 *     used is s_t = sum over T^L_t, i.e. s_{t+1} = s_t + the tokens that enter
 *     T^L between chunk t and chunk t+1.  Pinned by "recurrent == causal
 *     parallel form" (section 3.3, point 2) against the brute-force evaluator.
 *   - T not divisible by the chunk size: the last chunk is short.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC rehyat_oracle.c -o librehyat_oracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_E_ARG (-1)
#define ORACLE_E_MEM (-2)

/* ---------------------------------------------------------------------------
 * Chunk bookkeeping (section 3.2 token layout, Eq. 12, Eq. 13).
 * Tokens are frame-major: token = frame * HW + position.  Chunk t owns frames
 * [t*chunk, min((t+1)*chunk, T)).  Row t of `table` holds
 *   q_lo, q_hi : query token range of chunk t
 *   s_lo, s_hi : softmax window  [max(q_lo - overlap*HW, 0), q_hi)
 *   l_hi       : causal linear set is [0, l_hi) with l_hi = s_lo
 * `table` may be NULL to query only the chunk count.
 * ------------------------------------------------------------------------- */
int rehyat_oracle_chunk_plan(int T, int HW, int chunk, int overlap,
                             int64_t *table, int *n_chunks) {
  if (T < 1 || HW < 1 || chunk < 1 || overlap < 0 || !n_chunks) return ORACLE_E_ARG;
  int nc = 0;
  for (int f0 = 0; f0 < T; f0 += chunk) {
    int f1 = f0 + chunk;
    if (f1 > T) f1 = T;
    int64_t q_lo = (int64_t)f0 * HW;
    int64_t q_hi = (int64_t)f1 * HW;
    int64_t s_lo = q_lo - (int64_t)overlap * HW;
    if (s_lo < 0) s_lo = 0;
    if (table) {
      int64_t *row = table + 5 * (int64_t)nc;
      row[0] = q_lo;
      row[1] = q_hi;
      row[2] = s_lo;
      row[3] = q_hi;
      row[4] = s_lo;
    }
    ++nc;
  }
  *n_chunks = nc;
  return ORACLE_OK;
}

/* ---------------------------------------------------------------------------
 * Feature map phi for n rows of x [n, d] -> out [n, dprime]
 * ("Characterization of phi"; appendix "Training Details": two-layer MLP,
 * polynomial degree 2).  w1 [hidden, d], b1 [hidden], w2 [dprime, hidden],
 * b2 [dprime], all row-major.
 * ------------------------------------------------------------------------- */
static void phi_one(const double *x, int d, const double *w1, const double *b1,
                    const double *w2, const double *b2, int hidden, int dprime,
                    int degree, double *u, double *out) {
  for (int a = 0; a < hidden; ++a) {
    double s = b1[a];
    for (int c = 0; c < d; ++c) s += w1[(int64_t)a * d + c] * x[c];
    u[a] = s > 0.0 ? s : 0.0;
  }
  int part = dprime / degree;
  for (int e = 0; e < dprime; ++e) {
    double s = b2[e];
    for (int a = 0; a < hidden; ++a) s += w2[(int64_t)e * hidden + a] * u[a];
    double psi = s > 0.0 ? s : 0.0;
    int p = e / part + 1; /* part index, 1-based: the power it is raised to */
    double r = psi;
    for (int rep = 1; rep < p; ++rep) r *= psi;
    out[e] = r;
  }
}

int rehyat_oracle_phi(const double *x, int64_t n, int d, const double *w1,
                      const double *b1, const double *w2, const double *b2,
                      int hidden, int dprime, int degree, double *out) {
  if (!x || !w1 || !b1 || !w2 || !b2 || !out) return ORACLE_E_ARG;
  if (n < 0 || d < 1 || hidden < 1 || dprime < 1 || degree < 1 || dprime % degree)
    return ORACLE_E_ARG;
  int bad = 0;
#pragma omp parallel
  {
    double *u = (double *)malloc(sizeof(double) * (size_t)hidden);
    if (!u) {
#pragma omp atomic write
      bad = 1;
    }
#pragma omp for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
      if (u)
        phi_one(x + i * d, d, w1, b1, w2, b2, hidden, dprime, degree, u,
                out + i * dprime);
    }
    free(u);
  }
  return bad ? ORACLE_E_MEM : ORACLE_OK;
}

/* S += phi_k(k_j) v_j^T and z += phi_k(k_j) for j in [lo, hi)   (Eq. 17-18) */
static int absorb(const double *k, const double *v, int64_t lo, int64_t hi, int d,
                  const double *w1, const double *b1, const double *w2,
                  const double *b2, int hidden, int dprime, int degree, double *S,
                  double *z) {
  if (hi <= lo) return ORACLE_OK;
  int64_t n = hi - lo;
  double *pk = (double *)malloc(sizeof(double) * (size_t)n * (size_t)dprime);
  if (!pk) return ORACLE_E_MEM;
  int rc = rehyat_oracle_phi(k + lo * d, n, d, w1, b1, w2, b2, hidden, dprime,
                             degree, pk);
  if (rc == ORACLE_OK) {
#pragma omp parallel for schedule(static)
    for (int e = 0; e < dprime; ++e) {
      double *Srow = S + (int64_t)e * d;
      double zacc = z[e];
      for (int64_t j = 0; j < n; ++j) {
        double f = pk[j * dprime + e];
        const double *vj = v + (lo + j) * d;
        for (int c = 0; c < d; ++c) Srow[c] += f * vj[c];
        zacc += f;
      }
      z[e] = zacc;
    }
  }
  free(pk);
  return rc;
}

/* ---------------------------------------------------------------------------
 * Hybrid attention, chunk-recurrent evaluation.
 *
 * q, k, v : [B, H, N, d] row-major fp64, N = T*HW.
 * w1_q .. b2_k : phi_q and phi_k parameters, each with a leading H axis
 *                (w1 [H, hidden, d], b1 [H, hidden], w2 [H, dprime, hidden],
 *                b2 [H, dprime]).
 * causal  : 1 -> T^L_t = tokens before the window (Eq. 13);
 *           0 -> T^L_t = all tokens outside the window (Eq. 11-12).
 * stab    : 0 -> c_i = row maximum of the exponents; 1 -> c_i = 0.
 * rows    : optional sorted list of `nrows` query token indices in [0, N);
 *           NULL means all N tokens (then nrows is ignored).  Outputs hold one
 *           entry per listed row, in list order, for every (b, h).
 * out     : [B, H, R, d] with R = nrows or N.
 * m, nS, nL : optional [B, H, R];  aS, aL : optional [B, H, R, d].
 *           m is the row maximum of the softmax exponents (whatever `stab`).
 * ------------------------------------------------------------------------- */
int rehyat_oracle_forward(const double *q, const double *k, const double *v,
                          const double *w1_q, const double *b1_q,
                          const double *w2_q, const double *b2_q,
                          const double *w1_k, const double *b1_k,
                          const double *w2_k, const double *b2_k, int hidden,
                          int dprime, int degree, int B, int H, int T, int HW,
                          int d, int chunk, int overlap, int causal, int stab,
                          const int64_t *rows, int64_t nrows, double *out,
                          double *m, double *nS, double *aS, double *nL,
                          double *aL) {
  if (!q || !k || !v || !out) return ORACLE_E_ARG;
  if (!w1_q || !b1_q || !w2_q || !b2_q || !w1_k || !b1_k || !w2_k || !b2_k)
    return ORACLE_E_ARG;
  if (B < 1 || H < 1 || d < 1 || hidden < 1 || dprime < 1 || degree < 1 ||
      dprime % degree)
    return ORACLE_E_ARG;
  if (stab != 0 && stab != 1) return ORACLE_E_ARG;
  int nc = 0;
  if (rehyat_oracle_chunk_plan(T, HW, chunk, overlap, NULL, &nc) != ORACLE_OK)
    return ORACLE_E_ARG;
  const int64_t N = (int64_t)T * HW;
  const int64_t R = rows ? nrows : N;
  if (rows) {
    for (int64_t r = 0; r < nrows; ++r) {
      if (rows[r] < 0 || rows[r] >= N) return ORACLE_E_ARG;
      if (r > 0 && rows[r] <= rows[r - 1]) return ORACLE_E_ARG;
    }
  }
  int64_t *plan = (int64_t *)malloc(sizeof(int64_t) * 5 * (size_t)nc);
  double *S = (double *)malloc(sizeof(double) * (size_t)dprime * (size_t)d);
  double *z = (double *)malloc(sizeof(double) * (size_t)dprime);
  /* bidirectional mode only: totals over all tokens, and what has been
     absorbed up to the end of the current window */
  double *Sall = (double *)calloc((size_t)dprime * (size_t)d, sizeof(double));
  double *zall = (double *)calloc((size_t)dprime, sizeof(double));
  double *Sthru = (double *)malloc(sizeof(double) * (size_t)dprime * (size_t)d);
  double *zthru = (double *)malloc(sizeof(double) * (size_t)dprime);
  double *Slin = (double *)malloc(sizeof(double) * (size_t)dprime * (size_t)d);
  double *zlin = (double *)malloc(sizeof(double) * (size_t)dprime);
  int rc = ORACLE_OK;
  if (!plan || !S || !z || !Sall || !zall || !Sthru || !zthru || !Slin || !zlin)
    rc = ORACLE_E_MEM;
  if (rc == ORACLE_OK)
    rehyat_oracle_chunk_plan(T, HW, chunk, overlap, plan, &nc);
  const double scale = 1.0 / sqrt((double)d);

  for (int b = 0; b < B && rc == ORACLE_OK; ++b) {
    for (int hd = 0; hd < H && rc == ORACLE_OK; ++hd) {
      const int64_t bh = (int64_t)b * H + hd;
      const double *qh = q + bh * N * d;
      const double *kh = k + bh * N * d;
      const double *vh = v + bh * N * d;
      const double *W1q = w1_q + (int64_t)hd * hidden * d;
      const double *B1q = b1_q + (int64_t)hd * hidden;
      const double *W2q = w2_q + (int64_t)hd * dprime * hidden;
      const double *B2q = b2_q + (int64_t)hd * dprime;
      const double *W1k = w1_k + (int64_t)hd * hidden * d;
      const double *B1k = b1_k + (int64_t)hd * hidden;
      const double *W2k = w2_k + (int64_t)hd * dprime * hidden;
      const double *B2k = b2_k + (int64_t)hd * dprime;

      /* s_0 = 0, z_0 = 0                                          (Eq. 14-15) */
      memset(S, 0, sizeof(double) * (size_t)dprime * (size_t)d);
      memset(z, 0, sizeof(double) * (size_t)dprime);
      int64_t absorbed = 0; /* tokens [0, absorbed) are in S, z */
      int64_t absorbed_thru = 0;
      if (!causal) {
        memset(Sall, 0, sizeof(double) * (size_t)dprime * (size_t)d);
        memset(zall, 0, sizeof(double) * (size_t)dprime);
        rc = absorb(kh, vh, 0, N, d, W1k, B1k, W2k, B2k, hidden, dprime, degree,
                    Sall, zall);
        memset(Sthru, 0, sizeof(double) * (size_t)dprime * (size_t)d);
        memset(zthru, 0, sizeof(double) * (size_t)dprime);
      }
      int64_t rcur = 0; /* cursor into `rows` */

      for (int t = 0; t < nc && rc == ORACLE_OK; ++t) {
        const int64_t q_lo = plan[5 * t + 0], q_hi = plan[5 * t + 1];
        const int64_t s_lo = plan[5 * t + 2], s_hi = plan[5 * t + 3];
        const int64_t l_hi = plan[5 * t + 4];
        /* state update: absorb the tokens that left the softmax window */
        rc = absorb(kh, vh, absorbed, l_hi, d, W1k, B1k, W2k, B2k, hidden, dprime,
                    degree, S, z);
        if (rc != ORACLE_OK) break;
        if (l_hi > absorbed) absorbed = l_hi;
        const double *Suse = S;
        const double *zuse = z;
        if (!causal) {
          rc = absorb(kh, vh, absorbed_thru, s_hi, d, W1k, B1k, W2k, B2k, hidden,
                      dprime, degree, Sthru, zthru);
          if (rc != ORACLE_OK) break;
          absorbed_thru = s_hi;
          /* tokens before the window + tokens after it */
          for (int64_t e = 0; e < (int64_t)dprime * d; ++e)
            Slin[e] = S[e] + (Sall[e] - Sthru[e]);
          for (int e = 0; e < dprime; ++e) zlin[e] = z[e] + (zall[e] - zthru[e]);
          Suse = Slin;
          zuse = zlin;
        }

        /* which query rows of this chunk are wanted */
        int64_t first, count;
        if (rows) {
          while (rcur < nrows && rows[rcur] < q_lo) ++rcur;
          first = rcur;
          while (rcur < nrows && rows[rcur] < q_hi) ++rcur;
          count = rcur - first;
        } else {
          first = q_lo;
          count = q_hi - q_lo;
        }
        int bad = 0;
#pragma omp parallel
        {
          const int64_t W = s_hi - s_lo;
          double *sc = (double *)malloc(sizeof(double) * (size_t)W);
          double *u = (double *)malloc(sizeof(double) * (size_t)hidden);
          double *fq = (double *)malloc(sizeof(double) * (size_t)dprime);
          double *accS = (double *)malloc(sizeof(double) * (size_t)d);
          double *accL = (double *)malloc(sizeof(double) * (size_t)d);
          if (!sc || !u || !fq || !accS || !accL) {
#pragma omp atomic write
            bad = 1;
          }
#pragma omp for schedule(dynamic, 8)
          for (int64_t rr = 0; rr < count; ++rr) {
            if (!sc || !u || !fq || !accS || !accL) continue;
            const int64_t slot = first + rr;          /* index into outputs */
            const int64_t i = rows ? rows[slot] : slot; /* query token */
            const double *qi = qh + i * d;
            /* softmax part: exponents, their maximum, then Eq. 6 and 8 */
            double mx = -INFINITY;
            for (int64_t j = 0; j < W; ++j) {
              const double *kj = kh + (s_lo + j) * d;
              double s = 0.0;
              for (int c = 0; c < d; ++c) s += qi[c] * kj[c];
              s *= scale;
              sc[j] = s;
              if (s > mx) mx = s;
            }
            const double c_i = (stab == 0) ? mx : 0.0;
            double ns = 0.0;
            for (int c = 0; c < d; ++c) accS[c] = 0.0;
            for (int64_t j = 0; j < W; ++j) {
              double w = exp(sc[j] - c_i);
              const double *vj = vh + (s_lo + j) * d;
              ns += w;
              for (int c = 0; c < d; ++c) accS[c] += w * vj[c];
            }
            /* linear part: Eq. 7 and 9 through the state (Eq. 16) */
            phi_one(qi, d, W1q, B1q, W2q, B2q, hidden, dprime, degree, u, fq);
            double nl = 0.0;
            for (int c = 0; c < d; ++c) accL[c] = 0.0;
            for (int e = 0; e < dprime; ++e) {
              const double f = fq[e];
              const double *Srow = Suse + (int64_t)e * d;
              nl += f * zuse[e];
              for (int c = 0; c < d; ++c) accL[c] += f * Srow[c];
            }
            /* joint normalisation, Eq. 5 */
            const double den = ns + nl;
            const int64_t o = bh * R + slot;
            for (int c = 0; c < d; ++c) out[o * d + c] = (accS[c] + accL[c]) / den;
            if (m) m[o] = mx;
            if (nS) nS[o] = ns;
            if (nL) nL[o] = nl;
            if (aS)
              for (int c = 0; c < d; ++c) aS[o * d + c] = accS[c];
            if (aL)
              for (int c = 0; c < d; ++c) aL[o * d + c] = accL[c];
          }
          free(sc);
          free(u);
          free(fq);
          free(accS);
          free(accL);
        }
        if (bad) rc = ORACLE_E_MEM;
      }
    }
  }
  free(plan);
  free(S);
  free(z);
  free(Sall);
  free(zall);
  free(Sthru);
  free(zthru);
  free(Slin);
  free(zlin);
  return rc;
}

/* ---------------------------------------------------------------------------
 * State of the chunk-wise RNN after absorbing tokens [0, upto) of one head
 * (Eq. 14-15, 17-18): S [dprime, d] and z [dprime].  Used by tests of the
 * state kernels and of prefix consistency.
 * k, v : [N, d] of one (b, h);  phi_k parameters of that head.
 * ------------------------------------------------------------------------- */
int rehyat_oracle_state(const double *k, const double *v, int64_t upto, int d,
                        const double *w1, const double *b1, const double *w2,
                        const double *b2, int hidden, int dprime, int degree,
                        double *S, double *z) {
  if (!k || !v || !w1 || !b1 || !w2 || !b2 || !S || !z) return ORACLE_E_ARG;
  if (upto < 0 || d < 1 || hidden < 1 || dprime < 1 || degree < 1 || dprime % degree)
    return ORACLE_E_ARG;
  memset(S, 0, sizeof(double) * (size_t)dprime * (size_t)d);
  memset(z, 0, sizeof(double) * (size_t)dprime);
  return absorb(k, v, 0, upto, d, w1, b1, w2, b2, hidden, dprime, degree, S, z);
}
