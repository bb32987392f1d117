"""Pins for the fp64 oracle (CPU only).

The oracle must be trusted before any GPU result is compared with it, so each
test here checks it against something that is not the oracle: a library
softmax/matmul and autograd, finite differences, closed forms, invariants, a
hand-worked two-key example, the explicit block sum of Eq. 3 and a scalar
brute-force loop.  Citations are to the paper's sections and equations.
"""
import math

import numpy as np
import pytest
import torch

import oracle


def rand(shape, seed):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape)


def torch_attention(Q, K, V, q0=0, causal=False, scale=None):
    """Library routine: softmax(Q K^T s) V in float64 (Eq. 1), explicit -inf mask."""
    q, k, v = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (Q, K, V))
    s = (1.0 / math.sqrt(Q.shape[-1])) if scale is None else scale
    S = (q @ k.transpose(-1, -2)) * s
    if causal:
        i = torch.arange(Q.shape[2])[:, None] + q0
        j = torch.arange(K.shape[2])[None, :]
        S = S.masked_fill(j > i, float("-inf"))
    P = torch.softmax(S, dim=-1)
    return q, k, v, S, P, P @ v


# ---------------------------------------------------------------- forward ----

def test_hand_worked_two_keys():
    # One query, two keys, A = 1, scale 1: S = [0, ln 2] so P = [1/3, 2/3],
    # O = (3 + 2*6)/3 = 5 and LSE = ln 3.  (Eq. 1 by hand.)
    Q = np.array([[[[1.0]]]])
    K = np.array([[[[0.0], [math.log(2.0)]]]])
    V = np.array([[[[3.0], [6.0]]]])
    Qrep = np.repeat(Q, 2, axis=2)  # Lq may not exceed L; both rows identical
    O, LSE, S, P = oracle.forward(Qrep, K, V, scale=1.0, want_scores=True)
    np.testing.assert_allclose(P[0, 0, 0], [1 / 3, 2 / 3], rtol=1e-15)
    np.testing.assert_allclose(O[0, 0, :, 0], [5.0, 5.0], rtol=1e-15)
    np.testing.assert_allclose(LSE[0, 0], [math.log(3.0)] * 2, rtol=1e-15)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", [(1, 1, 8, 4), (2, 3, 33, 8), (1, 2, 64, 64)])
def test_forward_matches_library_softmax(shape, causal):
    # N = 1 is the textbook softmax(QK^T / sqrt d) V  (Eq. 1).
    B, Z, L, A = shape
    Q, K, V = rand(shape, 1), rand(shape, 2), rand(shape, 3)
    _, _, _, S_t, P_t, O_t = torch_attention(Q, K, V, causal=causal)
    O, LSE, S, P = oracle.forward(Q, K, V, causal=causal, want_scores=True)
    np.testing.assert_allclose(O, O_t.detach().numpy(), atol=1e-13)
    np.testing.assert_allclose(P, P_t.detach().numpy(), atol=1e-14)
    np.testing.assert_array_equal(np.isinf(S), np.isinf(S_t.detach().numpy()))
    fin = np.isfinite(S)
    np.testing.assert_allclose(S[fin], S_t.detach().numpy()[fin], atol=1e-13)
    np.testing.assert_allclose(LSE, torch.logsumexp(S_t, -1).detach().numpy(), atol=1e-13)


def test_forward_brute_force_scalar_loops():
    # Pure Python loops over Eq. 1, no vector code at all.
    B, Z, L, A = 1, 2, 12, 3
    Q, K, V = rand((B, Z, L, A), 4), rand((B, Z, L, A), 5), rand((B, Z, L, A), 6)
    s = 1 / math.sqrt(A)
    for causal in (False, True):
        O, LSE = oracle.forward(Q, K, V, causal=causal)
        for z in range(Z):
            for i in range(L):
                n = i + 1 if causal else L
                sc = [s * sum(Q[0, z, i, a] * K[0, z, j, a] for a in range(A)) for j in range(n)]
                den = sum(math.exp(x) for x in sc)
                for a in range(A):
                    ref = sum(math.exp(sc[j]) / den * V[0, z, j, a] for j in range(n))
                    assert abs(O[0, z, i, a] - ref) < 1e-13
                assert abs(LSE[0, z, i] - math.log(den)) < 1e-13


def test_rows_of_P_sum_to_one_and_V_ones_gives_ones():
    shape = (2, 2, 40, 16)
    Q, K = rand(shape, 7), rand(shape, 8)
    V = np.ones(shape)
    for causal in (False, True):
        O, _, _, P = oracle.forward(Q, K, V, causal=causal, want_scores=True)
        np.testing.assert_allclose(P.sum(-1), 1.0, atol=1e-14)
        np.testing.assert_allclose(O, 1.0, atol=1e-14)
        assert (P >= 0).all()


def test_zero_queries_give_uniform_attention():
    # Q = 0 => every score is 0 => P uniform: O_i = mean_j V_j, LSE = ln L;
    # under the causal mask O_i is the prefix mean and LSE_i = ln(i + 1).
    shape = (1, 2, 24, 8)
    K, V = rand(shape, 9), rand(shape, 10)
    Q = np.zeros(shape)
    O, LSE = oracle.forward(Q, K, V)
    np.testing.assert_allclose(O, np.broadcast_to(V.mean(2, keepdims=True), shape), atol=1e-14)
    np.testing.assert_allclose(LSE, math.log(24), atol=1e-14)
    O, LSE = oracle.forward(Q, K, V, causal=True)
    prefix = np.cumsum(V, axis=2) / np.arange(1, 25)[None, None, :, None]
    np.testing.assert_allclose(O, prefix, atol=1e-14)
    np.testing.assert_allclose(LSE, np.broadcast_to(np.log(np.arange(1, 25)), LSE.shape), atol=1e-14)


def test_constant_value_rows_and_single_token():
    shape = (1, 2, 20, 8)
    Q, K = rand(shape, 11), rand(shape, 12)
    v = rand((8,), 13)
    V = np.broadcast_to(v, shape).copy()
    O, _ = oracle.forward(Q, K, V)
    np.testing.assert_allclose(O, V, atol=1e-14)
    one = (1, 1, 1, 8)
    Q1, K1, V1 = rand(one, 14), rand(one, 15), rand(one, 16)
    O1, LSE1 = oracle.forward(Q1, K1, V1)
    np.testing.assert_allclose(O1, V1, atol=0)
    np.testing.assert_allclose(LSE1[0, 0, 0], (Q1 * K1).sum() / math.sqrt(8), atol=1e-14)


def test_key_shift_and_joint_permutation_leave_output_unchanged():
    shape = (1, 2, 30, 8)
    Q, K, V = rand(shape, 17), rand(shape, 18), rand(shape, 19)
    O, _ = oracle.forward(Q, K, V)
    u = rand((8,), 20)
    O_shift, _ = oracle.forward(Q, K + u, V)          # adds q.u to a whole row
    np.testing.assert_allclose(O_shift, O, atol=1e-13)
    perm = np.random.Generator(np.random.PCG64(21)).permutation(30)
    O_perm, _ = oracle.forward(Q, K[:, :, perm], V[:, :, perm])   # ring-order freedom
    np.testing.assert_allclose(O_perm, O, atol=1e-13)


@pytest.mark.parametrize("N", [1, 2, 4, 8])
def test_block_sum_of_eq3(N):
    # Eq. 3: O^n = sum_i S^n_i V_i with S^n_i the c x c column blocks of the
    # (post-softmax) strip of device n.  Summing explicit blocks reproduces O.
    B, Z, L, A = 1, 2, 32, 8
    c = L // N
    Q, K, V = rand((B, Z, L, A), 22), rand((B, Z, L, A), 23), rand((B, Z, L, A), 24)
    O, _, _, P = oracle.forward(Q, K, V, want_scores=True)
    for n in range(N):
        strip = P[:, :, n * c:(n + 1) * c, :]
        acc = np.zeros((B, Z, c, A))
        for i in range(N):
            acc += strip[..., i * c:(i + 1) * c] @ V[:, :, i * c:(i + 1) * c]
        np.testing.assert_allclose(acc, O[:, :, n * c:(n + 1) * c], atol=1e-13)


@pytest.mark.parametrize("causal", [False, True])
def test_rank_share_equals_rows_of_the_whole(causal):
    # Device n holds Q^n and obtains Attention^n(Q^n, K, V) (section 3.1): the
    # rows of the full result.  Partial dK/dV of the ranks add up to the whole.
    B, Z, L, A, N = 1, 2, 32, 8, 4
    c = L // N
    Q, K, V, dO = (rand((B, Z, L, A), s) for s in (25, 26, 27, 28))
    O, LSE = oracle.forward(Q, K, V, causal=causal)
    dQ, dK, dV = oracle.backward(Q, K, V, dO, causal=causal)
    dK_sum, dV_sum = np.zeros_like(dK), np.zeros_like(dV)
    for n in range(N):
        rows = slice(n * c, (n + 1) * c)
        On, LSEn = oracle.forward(Q[:, :, rows], K, V, q0=n * c, causal=causal)
        np.testing.assert_allclose(On, O[:, :, rows], atol=1e-14)
        np.testing.assert_allclose(LSEn, LSE[:, :, rows], atol=1e-14)
        dQn, dKn, dVn = oracle.backward(Q[:, :, rows], K, V, dO[:, :, rows], q0=n * c, causal=causal)
        np.testing.assert_allclose(dQn, dQ[:, :, rows], atol=1e-14)
        dK_sum += dKn
        dV_sum += dVn
    np.testing.assert_allclose(dK_sum, dK, atol=1e-13)
    np.testing.assert_allclose(dV_sum, dV, atol=1e-13)


# --------------------------------------------------------------- backward ----

@pytest.mark.parametrize("causal,q0,Lq", [(False, 0, 10), (True, 0, 10), (False, 4, 3), (True, 5, 5)])
def test_backward_matches_autograd(causal, q0, Lq):
    B, Z, L, A = 2, 2, 10, 6
    Q, dO = rand((B, Z, Lq, A), 30), rand((B, Z, Lq, A), 31)
    K, V = rand((B, Z, L, A), 32), rand((B, Z, L, A), 33)
    q, k, v, S_t, P_t, O_t = torch_attention(Q, K, V, q0=q0, causal=causal)
    P_t.retain_grad()
    S_t.retain_grad()
    O_t.backward(torch.tensor(dO))
    dQ, dK, dV, dP, dS = oracle.backward(Q, K, V, dO, q0=q0, causal=causal, want_scores=True)
    np.testing.assert_allclose(dQ, q.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(dK, k.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(dV, v.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(dP, P_t.grad.numpy(), atol=1e-13)
    # autograd's dS is w.r.t. the scaled score, as is the oracle's step 7
    np.testing.assert_allclose(dS, S_t.grad.numpy(), atol=1e-13)


@pytest.mark.parametrize("causal,q0,Lq", [(False, 0, 9), (True, 0, 9), (True, 3, 4)])
def test_backward_matches_central_finite_differences(causal, q0, Lq):
    # f = sum(O * dO); df/dx by central differences in fp64.
    B, Z, L, A = 1, 2, 9, 4
    Q, dO = rand((B, Z, Lq, A), 40), rand((B, Z, Lq, A), 41)
    K, V = rand((B, Z, L, A), 42), rand((B, Z, L, A), 43)
    dQ, dK, dV = oracle.backward(Q, K, V, dO, q0=q0, causal=causal)

    def f(Qx, Kx, Vx):
        O, _ = oracle.forward(Qx, Kx, Vx, q0=q0, causal=causal)
        return float((O * dO).sum())

    h = 1e-5
    for which, grad in ((0, dQ), (1, dK), (2, dV)):
        args = [Q, K, V]
        num = np.zeros_like(args[which])
        for idx in np.ndindex(*args[which].shape):
            plus = [a.copy() for a in args]
            minus = [a.copy() for a in args]
            plus[which][idx] += h
            minus[which][idx] -= h
            num[idx] = (f(*plus) - f(*minus)) / (2 * h)
        scale = max(1.0, float(np.abs(grad).max()))
        assert np.abs(num - grad).max() / scale < 1e-8, which


@pytest.mark.parametrize("causal", [False, True])
def test_backward_invariants(causal):
    shape = (1, 2, 28, 8)
    Q, K, V, dO = (rand(shape, s) for s in (50, 51, 52, 53))
    dQ, dK, dV, dP, dS = oracle.backward(Q, K, V, dO, causal=causal, want_scores=True)
    # softmax Jacobian annihilates constants: every row of dS sums to 0
    np.testing.assert_allclose(dS.sum(-1), 0.0, atol=1e-13)
    # shifting all keys by u leaves O unchanged  =>  sum_j dK_j = 0
    np.testing.assert_allclose(dK.sum(2), 0.0, atol=1e-13)
    # rows of P sum to 1  =>  sum_j dV_j = sum_i dO_i
    np.testing.assert_allclose(dV.sum(2), dO.sum(2), atol=1e-13)
    if causal:
        i, j = np.arange(28)[:, None], np.arange(28)[None, :]
        assert (dS[..., j > i] == 0).all()


def test_backward_constant_values_kill_dQ_and_dK():
    shape = (1, 2, 16, 8)
    Q, K, dO = rand(shape, 60), rand(shape, 61), rand(shape, 62)
    V = np.broadcast_to(rand((8,), 63), shape).copy()
    dQ, dK, dV = oracle.backward(Q, K, V, dO)
    np.testing.assert_allclose(dQ, 0.0, atol=1e-14)
    np.testing.assert_allclose(dK, 0.0, atol=1e-14)


def test_zero_queries_backward_closed_form():
    # Q = 0: P = 1/L, so dV_j = mean_i dO_i ... times L/L: dV_j = (1/L) sum_i dO_i,
    # dK = 0 (dK_j = s sum_i dS_ij Q_i), dQ_i = (s/L) sum_j (dP_ij - mean_j dP_ij) K_j.
    B, Z, L, A = 1, 1, 12, 4
    K, V, dO = rand((B, Z, L, A), 64), rand((B, Z, L, A), 65), rand((B, Z, L, A), 66)
    Q = np.zeros((B, Z, L, A))
    dQ, dK, dV = oracle.backward(Q, K, V, dO)
    np.testing.assert_allclose(dK, 0.0, atol=1e-15)
    np.testing.assert_allclose(dV, np.broadcast_to(dO.sum(2, keepdims=True) / L, dV.shape), atol=1e-14)
    dP = dO @ V.transpose(0, 1, 3, 2)
    ref = (0.5 / L) * (dP - dP.mean(-1, keepdims=True)) @ K
    np.testing.assert_allclose(dQ, ref, atol=1e-14)


def test_column_subset_equals_columns_of_full_backward():
    shape = (2, 2, 24, 8)
    Q, K, V, dO = (rand(shape, s) for s in (70, 71, 72, 73))
    for causal in (False, True):
        dQ, dK, dV = oracle.backward(Q, K, V, dO, causal=causal)
        cols = [23, 0, 7, 7, 12]
        dQs, dKs, dVs = oracle.backward(Q, K, V, dO, causal=causal, cols=cols)
        np.testing.assert_array_equal(dQs, dQ)
        np.testing.assert_array_equal(dKs, dK[:, :, cols])
        np.testing.assert_array_equal(dVs, dV[:, :, cols])


def test_bad_arguments_are_rejected():
    Q = np.zeros((1, 1, 4, 2))
    K = np.zeros((1, 1, 4, 2))
    with pytest.raises(ValueError):
        oracle.forward(Q, K, K, q0=1, causal=True)   # causal rows run past L
    with pytest.raises(ValueError):
        oracle.backward(Q, K, K, Q, cols=[4])    # column out of range
    with pytest.raises(ValueError):
        oracle.forward(Q, K, np.zeros((1, 1, 5, 2)))
