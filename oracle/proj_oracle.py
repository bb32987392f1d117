"""fp64 oracle of the two linear maps around Ring Self-Attention.  Test infrastructure only.

Table 2 of the paper, sequence-parallel rows "Q/K/V" and "Linear": on the rank's rows,
    Q/K/V:  (B, rows, H) x (H, AZ)  ->  (B, Z, rows, A)      (one product for each of Q, K, V)
    Linear: (B, Z, rows, A) x (AZ, H) -> (B, rows, H)
The paper prints no bias and no backward; the backward below is the derivative of these two
products.  Everything is the definition written out with numpy float64 matrix products; nothing
here is shared with, or imported by, the HIP path.

Weight layout: Wqkv is (H, 3*Z*A), columns ordered [Q | K | V], each block head-major
(column z*A + a of a block is element a of head z); Wo is (Z*A, H), rows head-major.
"""
import numpy as np


def _split_heads(Y, Z, A):
    """(B, rows, Z*A) -> (B, Z, rows, A)."""
    B, rows, _ = Y.shape
    return np.ascontiguousarray(Y.reshape(B, rows, Z, A).transpose(0, 2, 1, 3))


def _merge_heads(T):
    """(B, Z, rows, A) -> (B, rows, Z*A)."""
    B, Z, rows, A = T.shape
    return np.ascontiguousarray(T.transpose(0, 2, 1, 3).reshape(B, rows, Z * A))


def qkv_proj(X, Wqkv, Z, A):
    """Table 2, row Q/K/V: returns Q, K, V, each (B, Z, rows, A)."""
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(Wqkv, dtype=np.float64)
    ZA = Z * A
    assert W.shape == (X.shape[2], 3 * ZA)
    return tuple(_split_heads(X @ W[:, i * ZA:(i + 1) * ZA], Z, A) for i in range(3))


def out_proj(O, Wo):
    """Table 2, row Linear: (B, Z, rows, A) x (AZ, H) -> (B, rows, H)."""
    O = np.asarray(O, dtype=np.float64)
    return _merge_heads(O) @ np.asarray(Wo, dtype=np.float64)


def out_proj_bwd(dY, O, Wo):
    """Derivative of out_proj: dO (B, Z, rows, A) and dWo (AZ, H), summed over batch and rows."""
    dY = np.asarray(dY, dtype=np.float64)
    O = np.asarray(O, dtype=np.float64)
    Wo = np.asarray(Wo, dtype=np.float64)
    B, Z, rows, A = O.shape
    dO = _split_heads(dY @ Wo.T, Z, A)
    Om = _merge_heads(O).reshape(B * rows, Z * A)
    dWo = Om.T @ dY.reshape(B * rows, -1)
    return dO, dWo


def qkv_proj_bwd(dQ, dK, dV, X, Wqkv):
    """Derivative of qkv_proj: dX (B, rows, H) and dWqkv (H, 3*Z*A)."""
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(Wqkv, dtype=np.float64)
    G = np.concatenate([_merge_heads(np.asarray(t, dtype=np.float64)) for t in (dQ, dK, dV)], axis=2)
    dX = G @ W.T
    B, rows, H = X.shape
    dW = X.reshape(B * rows, H).T @ G.reshape(B * rows, -1)
    return dX, dW
