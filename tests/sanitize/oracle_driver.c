/* Host sanitizer job for the fp64 oracle: built with -fsanitize=address,undefined by
 * tests/test_sanitizers.py and run on seeded shapes (ragged row ranges, causal and not, column
 * subsets, the optional score outputs).  It checks what holds for any input -- rows of P sum to 1,
 * rows of dS sum to 0, outputs finite -- so that every buffer is both written and read under the
 * sanitizer; the numerical pins of the oracle live in tests/test_oracle_pins.py. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "rsa_oracle.h"

static uint64_t state = 0x9E3779B97F4A7C15ull;
static double rnd(void) { /* xorshift64*, uniform in [-1, 1) */
  state ^= state >> 12; state ^= state << 25; state ^= state >> 27;
  return (double)((state * 0x2545F4914F6CDD1Dull) >> 11) / 4503599627370496.0 - 1.0;
}
static double *fill(size_t n) {
  double *p = (double *)malloc(n * sizeof(double));
  if (!p) { fprintf(stderr, "out of memory\n"); exit(2); }
  for (size_t i = 0; i < n; ++i) p[i] = rnd();
  return p;
}
static int finite_all(const double *p, size_t n) {
  for (size_t i = 0; i < n; ++i) if (!isfinite(p[i])) return 0;
  return 1;
}

static int run_case(int64_t B, int64_t Z, int64_t L, int64_t A, int64_t Lq, int64_t q0, int causal, int64_t ncols) {
  rsa_oracle_problem p = {B, Z, L, A, Lq, q0, causal, 1.0 / sqrt((double)A)};
  const size_t nq = (size_t)(B * Z * Lq * A), nk = (size_t)(B * Z * L * A), ns = (size_t)(B * Z * Lq * L);
  double *Q = fill(nq), *K = fill(nk), *V = fill(nk), *dO = fill(nq);
  double *O = fill(nq), *LSE = fill((size_t)(B * Z * Lq)), *S = fill(ns), *P = fill(ns);
  double *dQ = fill(nq), *dP = fill(ns), *dS = fill(ns);
  int64_t *cols = NULL;
  size_t ng = nk;
  if (ncols > 0) {
    cols = (int64_t *)malloc((size_t)ncols * sizeof(int64_t));
    for (int64_t i = 0; i < ncols; ++i) cols[i] = (int64_t)((rnd() + 1.0) * 0.5 * (double)L) % L;
    ng = (size_t)(B * Z * ncols * A);
  }
  double *dK = fill(ng), *dV = fill(ng);
  int bad = 0;
  bad |= rsa_oracle_forward(&p, Q, K, V, O, LSE, S, P) != 0;
  bad |= rsa_oracle_forward(&p, Q, K, V, O, LSE, NULL, NULL) != 0;
  bad |= rsa_oracle_backward(&p, Q, K, V, dO, dQ, dK, dV, cols, ncols, dP, dS) != 0;
  bad |= rsa_oracle_backward(&p, Q, K, V, dO, dQ, dK, dV, cols, ncols, NULL, NULL) != 0;
  bad |= !finite_all(O, nq) || !finite_all(LSE, (size_t)(B * Z * Lq)) || !finite_all(dQ, nq) ||
         !finite_all(dK, ng) || !finite_all(dV, ng);
  for (int64_t r = 0; r < B * Z * Lq && !bad; ++r) {
    double sp = 0.0, sd = 0.0;
    for (int64_t j = 0; j < L; ++j) { sp += P[r * L + j]; sd += dS[r * L + j]; }
    if (fabs(sp - 1.0) > 1e-12 || fabs(sd) > 1e-10) bad = 1;
  }
  /* bad arguments are refused, not dereferenced */
  rsa_oracle_problem q = p;
  q.Lq = 0;
  bad |= rsa_oracle_forward(&q, Q, K, V, O, LSE, NULL, NULL) != -1;
  bad |= rsa_oracle_forward(&p, NULL, K, V, O, LSE, NULL, NULL) != -1;
  if (bad) fprintf(stderr, "case B%lld Z%lld L%lld A%lld Lq%lld q0 %lld causal %d ncols %lld FAILED\n", (long long)B,
                   (long long)Z, (long long)L, (long long)A, (long long)Lq, (long long)q0, causal, (long long)ncols);
  free(Q); free(K); free(V); free(dO); free(O); free(LSE); free(S); free(P); free(dQ); free(dP); free(dS);
  free(dK); free(dV); free(cols);
  return bad;
}

int main(void) {
  int bad = 0;
  bad |= run_case(1, 1, 1, 1, 1, 0, 0, 0);
  bad |= run_case(1, 2, 7, 3, 7, 0, 1, 0);
  bad |= run_case(2, 3, 65, 8, 65, 0, 0, 5);
  bad |= run_case(1, 2, 130, 16, 33, 97, 1, 0);      /* a rank's share that ends with the sequence */
  bad |= run_case(2, 1, 96, 64, 17, 40, 1, 9);       /* a share in the middle, column subset */
  bad |= run_case(1, 3, 257, 5, 64, 0, 0, 257);      /* every column listed */
  for (int i = 0; i < 12; ++i) {
    const int64_t L = 1 + (int64_t)((rnd() + 1.0) * 60.0), Lq = 1 + (int64_t)((rnd() + 1.0) * 0.5 * (double)(L - 1));
    const int64_t q0 = (int64_t)((rnd() + 1.0) * 0.5 * (double)(L - Lq + 1)) % (L - Lq + 1);
    bad |= run_case(1 + i % 2, 1 + i % 3, L, 1 + (int64_t)((rnd() + 1.0) * 16.0), Lq, q0, i & 1, (i % 3 == 0) ? 1 + i : 0);
  }
  printf(bad ? "SANITIZE_ORACLE_FAILED\n" : "SANITIZE_ORACLE_OK threads=%d\n", rsa_oracle_threads());
  return bad;
}
