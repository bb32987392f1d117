"""fp64 oracle of the Linformer variant of sequence-parallel attention.  Test infrastructure only.

Table 3 of the paper (rows Projection, Ring-QK^T, Ring-AV): every rank projects its K and V chunk
along the sequence with its row block of a projection matrix,
    Projection: (B, Z, L/N, A) x (L/N, K) -> (B, Z, K, A)        (summed over the ranks),
and attends its queries to the K projected keys and values,
    Ring-QK^T:  (B, Z, L/N, A) x (B, Z, K, A) -> (B, Z, L/N, K)
    Ring-AV:    (B, Z, L/N, K) x (B, Z, K, A) -> (B, Z, L/N, A),
with the softmax of Eq. 1 over the K projected keys in between (the table, like section 3.1, does
not print it).  The paper prints no backward; the one here is the derivative of these products.
The attention itself is the attention oracle called with K, V of length K; this file adds only the
projections, written with numpy float64 products.  Nothing here is shared with the HIP path.

E and F are (L, K): row l weights token l.  `rows` = (first, count) restricts the projection to a
block of tokens (one rank's share; the shares add up to the whole).
"""
import numpy as np

from . import rsa_oracle


def project(X, E, rows=None):
    """X (B, Z, L, A), E (L, K) -> (B, Z, K, A): out[b,z,k,a] = sum_l E[l,k] X[b,z,l,a]."""
    X = np.asarray(X, dtype=np.float64)
    E = np.asarray(E, dtype=np.float64)
    if rows is not None:
        X, E = X[:, :, rows[0]:rows[0] + rows[1]], E[rows[0]:rows[0] + rows[1]]
    return np.einsum("lk,bzla->bzka", E, X)


def project_bwd(dXp, X, E, rows=None):
    """Derivative of project: dX (B, Z, L, A) = E dXp and dE (L, K) = sum_{b,z} X dXp^T
    (zero outside `rows`)."""
    X = np.asarray(X, dtype=np.float64)
    E = np.asarray(E, dtype=np.float64)
    dXp = np.asarray(dXp, dtype=np.float64)
    dX = np.zeros_like(X)
    dE = np.zeros_like(E)
    r0, n = (0, X.shape[2]) if rows is None else rows
    dX[:, :, r0:r0 + n] = np.einsum("lk,bzka->bzla", E[r0:r0 + n], dXp)
    dE[r0:r0 + n] = np.einsum("bzla,bzka->lk", X[:, :, r0:r0 + n], dXp)
    return dX, dE


def forward(Q, Kp, Vp, scale=None):
    """Attention of Q (B, Z, rows, A) to the projected Kp, Vp (B, Z, K, A): O and LSE."""
    return rsa_oracle.forward(Q, Kp, Vp, q0=0, causal=False, scale=scale)


def backward(Q, Kp, Vp, dO, scale=None):
    """dQ, dKp, dVp of the attention above."""
    return rsa_oracle.backward(Q, Kp, Vp, dO, q0=0, causal=False, scale=scale)
