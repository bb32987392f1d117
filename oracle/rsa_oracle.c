/* fp64 CPU oracle for Ring Self-Attention; see rsa_oracle.h.  Test infrastructure only. */
#include "rsa_oracle.h"
#include <math.h>
#include <omp.h>
#include <stdlib.h>
#include <string.h>

static int bad_problem(const rsa_oracle_problem *p) {
  if (!p) return 1;
  if (p->B < 1 || p->Z < 1 || p->L < 1 || p->A < 1 || p->Lq < 1) return 1;
  /* query rows are tokens q0 .. q0+Lq-1 of the sequence only under the causal mask; without
     it the row index never enters the arithmetic and the keys may be any set (Table 3's
     projected keys are fewer than the queries) */
  if (p->q0 < 0 || (p->causal && p->q0 + p->Lq > p->L)) return 1;
  return 0;
}

/* Number of keys query row (global index i) may look at. */
static int64_t visible(const rsa_oracle_problem *p, int64_t i) {
  return p->causal ? i + 1 : p->L;
}

/* Steps 1-2 for one query row q (A values): fills S[0..L) (masked = -inf) and
 * P[0..L) (masked = 0), returns m and l through pointers. */
static void score_row(const rsa_oracle_problem *p, const double *q,
                      const double *Kh, int64_t i_global, double *S, double *P,
                      double *m_out, double *l_out) {
  const int64_t L = p->L, A = p->A, nvis = visible(p, i_global);
  double m = -INFINITY;
  for (int64_t j = 0; j < L; ++j) {
    if (j < nvis) {
      const double *k = Kh + j * A;
      double acc = 0.0;
#pragma omp simd reduction(+ : acc)
      for (int64_t a = 0; a < A; ++a) acc += q[a] * k[a];
      S[j] = p->scale * acc;
      if (S[j] > m) m = S[j];
    } else {
      S[j] = -INFINITY;
    }
  }
  double l = 0.0;
  for (int64_t j = 0; j < nvis; ++j) l += exp(S[j] - m);
  for (int64_t j = 0; j < L; ++j) P[j] = (j < nvis) ? exp(S[j] - m) / l : 0.0;
  *m_out = m;
  *l_out = l;
}

int rsa_oracle_forward(const rsa_oracle_problem *p, const double *Q,
                       const double *K, const double *V, double *O,
                       double *LSE, double *S_out, double *P_out) {
  if (bad_problem(p) || !Q || !K || !V || !O || !LSE) return -1;
  const int64_t L = p->L, A = p->A, Lq = p->Lq, heads = p->B * p->Z;
  int failed = 0;
#pragma omp parallel
  {
    double *S = (double *)malloc(sizeof(double) * (size_t)L);
    double *P = (double *)malloc(sizeof(double) * (size_t)L);
    if (!S || !P) {
#pragma omp atomic write
      failed = 1;
    }
#pragma omp barrier
    if (!failed) {
#pragma omp for collapse(2) schedule(dynamic, 8)
      for (int64_t h = 0; h < heads; ++h) {
        for (int64_t r = 0; r < Lq; ++r) {
          const double *q = Q + (h * Lq + r) * A;
          const double *Kh = K + h * L * A;
          const double *Vh = V + h * L * A;
          double m, l;
          score_row(p, q, Kh, p->q0 + r, S, P, &m, &l);
          LSE[h * Lq + r] = m + log(l);
          double *o = O + (h * Lq + r) * A;
          for (int64_t a = 0; a < A; ++a) o[a] = 0.0;
          for (int64_t j = 0; j < L; ++j) {
            const double pj = P[j];
            if (pj == 0.0) continue;
            const double *v = Vh + j * A;
#pragma omp simd
            for (int64_t a = 0; a < A; ++a) o[a] += pj * v[a];
          }
          if (S_out) memcpy(S_out + (h * Lq + r) * L, S, sizeof(double) * (size_t)L);
          if (P_out) memcpy(P_out + (h * Lq + r) * L, P, sizeof(double) * (size_t)L);
        }
      }
    }
    free(S);
    free(P);
  }
  return failed ? -1 : 0;
}

int rsa_oracle_backward(const rsa_oracle_problem *p, const double *Q,
                        const double *K, const double *V, const double *dO,
                        double *dQ, double *dK, double *dV,
                        const int64_t *cols, int64_t ncols, double *dP_out,
                        double *dS_out) {
  if (bad_problem(p) || !Q || !K || !V || !dO || !dQ || !dK || !dV) return -1;
  const int64_t L = p->L, A = p->A, Lq = p->Lq, heads = p->B * p->Z;
  if (cols) {
    if (ncols < 1) return -1;
    for (int64_t c = 0; c < ncols; ++c)
      if (cols[c] < 0 || cols[c] >= L) return -1;
  } else {
    ncols = L;
  }
  /* row statistics of step 2 and D of step 6, kept for the column pass */
  double *row_m = (double *)malloc(sizeof(double) * (size_t)(heads * Lq));
  double *row_l = (double *)malloc(sizeof(double) * (size_t)(heads * Lq));
  double *row_D = (double *)malloc(sizeof(double) * (size_t)(heads * Lq));
  int failed = (!row_m || !row_l || !row_D);

  /* Row pass: steps 1, 2, 5, 6, 7, 8 for every query row. */
#pragma omp parallel
  {
    double *S = (double *)malloc(sizeof(double) * (size_t)L);
    double *P = (double *)malloc(sizeof(double) * (size_t)L);
    double *dP = (double *)malloc(sizeof(double) * (size_t)L);
    if (!S || !P || !dP) {
#pragma omp atomic write
      failed = 1;
    }
#pragma omp barrier
    if (!failed) {
#pragma omp for collapse(2) schedule(dynamic, 8)
      for (int64_t h = 0; h < heads; ++h) {
        for (int64_t r = 0; r < Lq; ++r) {
          const double *q = Q + (h * Lq + r) * A;
          const double *go = dO + (h * Lq + r) * A;
          const double *Kh = K + h * L * A;
          const double *Vh = V + h * L * A;
          double m, l;
          score_row(p, q, Kh, p->q0 + r, S, P, &m, &l);
          double D = 0.0;
          for (int64_t j = 0; j < L; ++j) { /* steps 5, 6 */
            const double *v = Vh + j * A;
            double acc = 0.0;
#pragma omp simd reduction(+ : acc)
            for (int64_t a = 0; a < A; ++a) acc += go[a] * v[a];
            dP[j] = acc;
            D += P[j] * acc;
          }
          double *gq = dQ + (h * Lq + r) * A;
          for (int64_t a = 0; a < A; ++a) gq[a] = 0.0;
          for (int64_t j = 0; j < L; ++j) { /* steps 7, 8 */
            const double dS = P[j] * (dP[j] - D);
            if (dS_out) dS_out[(h * Lq + r) * L + j] = dS;
            const double *k = Kh + j * A;
            const double w = p->scale * dS;
#pragma omp simd
            for (int64_t a = 0; a < A; ++a) gq[a] += w * k[a];
          }
          if (dP_out) memcpy(dP_out + (h * Lq + r) * L, dP, sizeof(double) * (size_t)L);
          row_m[h * Lq + r] = m;
          row_l[h * Lq + r] = l;
          row_D[h * Lq + r] = D;
        }
      }
    }
    free(S);
    free(P);
    free(dP);
  }

  /* Column pass: steps 4 and 9 for every requested key column (the sums over
   * query rows; on the ring these are what the two all-reduces add up). */
  if (!failed) {
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
    for (int64_t h = 0; h < heads; ++h) {
      for (int64_t c = 0; c < ncols; ++c) {
        const int64_t j = cols ? cols[c] : c;
        const double *k = K + (h * L + j) * A;
        const double *v = V + (h * L + j) * A;
        double *gk = dK + (h * ncols + c) * A;
        double *gv = dV + (h * ncols + c) * A;
        for (int64_t a = 0; a < A; ++a) gk[a] = gv[a] = 0.0;
        for (int64_t r = 0; r < Lq; ++r) {
          if (j >= visible(p, p->q0 + r)) continue; /* masked: P = dS = 0 */
          const double *q = Q + (h * Lq + r) * A;
          const double *go = dO + (h * Lq + r) * A;
          double s_acc = 0.0, dp_acc = 0.0;
#pragma omp simd reduction(+ : s_acc, dp_acc)
          for (int64_t a = 0; a < A; ++a) {
            s_acc += q[a] * k[a];
            dp_acc += go[a] * v[a];
          }
          const double S = p->scale * s_acc;
          const double P = exp(S - row_m[h * Lq + r]) / row_l[h * Lq + r];
          const double dS = P * (dp_acc - row_D[h * Lq + r]);
          const double w = p->scale * dS;
#pragma omp simd
          for (int64_t a = 0; a < A; ++a) {
            gv[a] += P * go[a];
            gk[a] += w * q[a];
          }
        }
      }
    }
  }
  free(row_m);
  free(row_l);
  free(row_D);
  return failed ? -1 : 0;
}

int rsa_oracle_threads(void) { return omp_get_max_threads(); }
