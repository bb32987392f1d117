/*
 * rsa_oracle.h -- fp64 CPU oracle for Ring Self-Attention (TEST INFRASTRUCTURE ONLY).
 *
 * This library is the slow, plain checker that the GPU path is compared with.
 * It is not part of the product: only tests, the smoke check and the CPU
 * baseline leg of the benchmark may load it.  It shares no code, header,
 * constant or table with the HIP library.
 *
 * What it computes.  Ring Self-Attention on device n produces
 * Attention^n(Q^n, K, V) (paper section 3.1): the ring of key chunks yields the
 * score strip S^n = Q^n K^T, a full-row softmax is taken, and the ring of value
 * chunks yields O^n = sum_i S^n_i V_i (Eq. 3), which is just the block form of
 * the matrix product.  The result is therefore exactly Eq. 1,
 *     Attention(Q,K,V) = softmax(Q K^T / sqrt(d_k)) V,
 * up to floating-point summation order, so the oracle is that definition
 * written out row by row with no chunking at all.  Heads are independent
 * problems (section 3.1; appendix A).
 *
 * Readings of the paper taken here (the paper is silent or garbled on these):
 *  - S^n in Eq. 3 is the post-softmax matrix; the 1/sqrt(d_k) scale and the
 *    softmax over all L columns sit between the two ring passes (Eq. 1).
 *  - "V_i = V^n" under Eq. 3 is read as V_i = V^i, the chunk held by device i.
 *  - The backward pass is not printed in the paper; it is the analytic
 *    derivative of Eq. 1 (steps 4-9 below).  Its structure matches the
 *    paper's communication count in section 3.2.2: two ring passes (V for dP,
 *    K for dQ) and two all-reduces (the sums over query rows in dK and dV).
 *  - The paper treats bidirectional attention only.  The optional causal mask
 *    is an extension: key j is visible to query i iff j <= i in global token
 *    index; a masked score is -infinity, its probability exactly 0.
 *
 * Steps, for each (batch, head) and each query row i (global index q0 + r):
 *   1. S_ij  = scale * sum_a Q_ia K_ja            (masked: -inf)
 *   2. m_i   = max_j S_ij ; l_i = sum_j exp(S_ij - m_i)
 *      P_ij  = exp(S_ij - m_i) / l_i ; LSE_i = m_i + log(l_i)
 *   3. O_ia  = sum_j P_ij V_ja
 *   4. dV_ja = sum_i P_ij dO_ia
 *   5. dP_ij = sum_a dO_ia V_ja
 *   6. D_i   = sum_j P_ij dP_ij
 *   7. dS_ij = P_ij (dP_ij - D_i)
 *   8. dQ_ia = scale * sum_j dS_ij K_ja
 *   9. dK_ja = scale * sum_i dS_ij Q_ia
 *
 * Layout: every tensor is a dense row-major double array.  K, V, dK, dV are
 * (B, Z, L, A); Q, O, dO, dQ are (B, Z, Lq, A) and cover query rows
 * [q0, q0 + Lq) of the sequence (one rank's share, or all rows when q0 = 0 and
 * Lq = L).  With a partial row range dK and dV are that range's partial sums,
 * which is what the ring's all-reduce would add up.
 *
 * Pins (tests/test_oracle_*.py): a library fp64 softmax(QK^T s)V and its
 * autograd on tiny inputs, central finite differences, closed forms (Q = 0,
 * constant V, L = 1, key shift, joint K/V permutation), row-sum and
 * column-sum invariants, the explicit block sum of Eq. 3, and the causal
 * prefix mean.
 */
#ifndef RSA_ORACLE_H
#define RSA_ORACLE_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int64_t B, Z, L, A; /* batch, heads, total sequence length, head size     */
  int64_t Lq, q0;     /* number of query rows held, global index of row 0   */
  int32_t causal;     /* 0 = bidirectional (the paper), 1 = causal extension */
  double scale;       /* 1/sqrt(d_k) of Eq. 1                               */
} rsa_oracle_problem;

/* Steps 1-3.  O: (B,Z,Lq,A).  LSE: (B,Z,Lq).  S_out and P_out, if not NULL,
 * receive the scaled (masked) scores and the probabilities, (B,Z,Lq,L).
 * Returns 0, or -1 on a bad argument. */
int rsa_oracle_forward(const rsa_oracle_problem *p, const double *Q,
                       const double *K, const double *V, double *O,
                       double *LSE, double *S_out, double *P_out);

/* Steps 4-9 (steps 1-2 are recomputed internally).  dQ: (B,Z,Lq,A).
 * If cols is NULL, dK and dV are (B,Z,L,A).  Otherwise cols lists ncols key
 * indices in [0,L) and dK, dV are (B,Z,ncols,A), holding those keys only.
 * dP_out and dS_out, if not NULL, receive steps 5 and 7, (B,Z,Lq,L).
 * Returns 0, or -1 on a bad argument. */
int rsa_oracle_backward(const rsa_oracle_problem *p, const double *Q,
                        const double *K, const double *V, const double *dO,
                        double *dQ, double *dK, double *dV,
                        const int64_t *cols, int64_t ncols, double *dP_out,
                        double *dS_out);

/* Number of OpenMP threads the two calls above will use. */
int rsa_oracle_threads(void);

#ifdef __cplusplus
}
#endif
#endif
