"""CPU models of a bf16 attention pipeline, for deriving and checking tolerances (test-only).

`ideal_bf16_pipeline` is exact fp64 arithmetic with only the roundings that ANY path
with bf16 matrix-core operands and bf16 storage must make:
    P as the operand of P V and of P^T dO, dS as the operand of dS K and dS^T Q,
    the stored O (which then enters D = rowsum(dO o O)), and the stored dQ, dK, dV.
The fused HIP kernels make exactly these roundings and no others (their scores, softmax
statistics, products with the row terms and accumulations are fp32), so this model is
also the model of the kernels; the GPU tests hold the kernels to stated multiples of
its error on the same inputs.  Two details of how P is rounded in the forward:
  reference="true_max":    P = bf16(exp(S - max_j S)): a two-pass softmax.  The row's largest
                           probability is then exactly 1 and carries no rounding error.
  reference="running_max": an online softmax rounds exp(S - m) for whatever m its running
                           maximum held when the key went by, so where in its binade a
                           probability sits (which decides its rounding error) is arbitrary,
                           the largest one included.  Modelled by a seeded per-row offset
                           u in [0, 1): P = 2^u bf16(2^-u exp(S - max_j S)).
The two differ only on rows that one key dominates (a sharp softmax: that key's rounding is
most of the row's error); the fused forward is an online softmax and is compared with the second.

`strip_bf16_pipeline` is the model of the paper's two-pass layout with the score strip stored
in bf16: the normalised P is rounded once, when it is written, and both O = P V and
dS = P o (dP - D) are formed from that rounded P (dS is then rounded again as an operand).

`folded_scale_pipeline` adds the one rounding an earlier version of the backward kernels
made on top: the factor s log2(e) folded into a bf16 operand (K for dK/dV, Q for dQ).
It is kept as the planted mistake that the tolerance must reject.

Written from the step list of Eq. 1 and its derivative; shares nothing with the HIP
path or the oracle.
"""
import numpy as np

from paper_2105_13120_amd import inputs


def r(a):
    """Round to bf16 (nearest even), back in float64."""
    return inputs.round_to_bf16(np.asarray(a, dtype=np.float32)).astype(np.float64)


def _head(Q, K, V, dO, s, qtok, causal, fold=False, strip=False, rng=None):
    """One head: Q, dO (Lq, A) are the query rows of tokens qtok; K, V (L, A)."""
    L = K.shape[0]
    log2e = 1.4426950408889634
    S = s * (Q @ K.T)
    mask = None
    if causal:
        mask = np.arange(L)[None, :] > qtok[:, None]
        S[mask] = -np.inf
    m = S.max(-1, keepdims=True)
    p = np.exp(S - m)
    l = p.sum(-1, keepdims=True)
    P = p / l
    if strip:
        Pr = r(P)
        O = r(Pr @ V)
    else:
        if rng is None:
            pr = r(p)
        else:
            u = np.exp2(rng.random((Q.shape[0], 1)))
            pr = r(p / u) * u
        O = r((pr @ V) / l)
    out = [O, m[:, 0] + np.log(l[:, 0])]
    if dO is None:
        return out
    lse = m + np.log(l)
    if fold:
        # P recomputed from bf16(K s log2e) for dV, dK and from bf16(Q s log2e) for dQ
        c = s * log2e
        Sk = Q @ r(K * c).T
        Sq = r(Q * c) @ K.T
        if causal:
            Sk[mask] = -np.inf
            Sq[mask] = -np.inf
        Pk, Pq = np.exp2(Sk - lse * log2e), np.exp2(Sq - lse * log2e)
    elif strip:
        Pk = Pq = Pr
    else:
        Pk = Pq = P
    dP = dO @ V.T
    D = (dO * O).sum(-1, keepdims=True)
    dV = r(r(Pk).T @ dO)
    dK = r(s * (r(Pk * (dP - D)).T @ Q))
    dQ = r(s * (r(Pq * (dP - D)) @ K))
    return out + [dQ, dK, dV]


def _pipeline(Q, K, V, dO, scale, qtok, causal, **kw):
    B, Z, Lq, A = Q.shape
    s = 1.0 / np.sqrt(A) if scale is None else scale
    qtok = np.arange(Lq) if qtok is None else np.asarray(qtok, dtype=np.int64)
    assert qtok.shape == (Lq,)
    res = None
    for b in range(B):
        for z in range(Z):
            h = _head(Q[b, z], K[b, z], V[b, z], None if dO is None else dO[b, z], s, qtok, causal, **kw)
            if res is None:
                res = [np.empty((B, Z) + x.shape) for x in h]
            for dst, x in zip(res, h):
                dst[b, z] = x
    return tuple(res)


def ideal_bf16_pipeline(Q, K, V, dO=None, scale=None, qtok=None, causal=False, reference="true_max"):
    """(O, LSE) or (O, LSE, dQ, dK, dV) of the ideal bf16 pipeline; arrays (B, Z, rows, A) float64
    holding bf16-representable inputs.  Row i of Q, dO is token qtok[i] of the sequence (default:
    token i); dK, dV are those rows' partial sums.  reference: see the top of the file."""
    assert reference in ("true_max", "running_max")
    rng = np.random.Generator(np.random.PCG64(20210525)) if reference == "running_max" else None
    return _pipeline(Q, K, V, dO, scale, qtok, causal, rng=rng)


def strip_bf16_pipeline(Q, K, V, dO=None, scale=None, qtok=None, causal=False):
    """The same for the two-pass layout whose probability strip is stored in bf16."""
    return _pipeline(Q, K, V, dO, scale, qtok, causal, strip=True)


def folded_scale_pipeline(Q, K, V, dO, scale=None, qtok=None, causal=False):
    """The ideal pipeline with s log2(e) folded into a bf16 operand of the recomputed scores."""
    return _pipeline(Q, K, V, dO, scale, qtok, causal, fold=True)
