"""Pins of the Linformer oracle (paper Table 3: Projection, Ring-QK^T, Ring-AV) against things
other than itself."""
import numpy as np
import torch

import oracle

LF = oracle.linformer


def rnd(shape, seed):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape)


def test_projection_against_scalar_loops_and_rank_shares_add_up():
    B, Z, L, A, K = 2, 2, 6, 3, 4
    X, E = rnd((B, Z, L, A), 1), rnd((L, K), 2)
    got = LF.project(X, E)
    for b in range(B):
        for z in range(Z):
            for k in range(K):
                for a in range(A):
                    want = sum(E[l, k] * X[b, z, l, a] for l in range(L))
                    assert abs(got[b, z, k, a] - want) < 1e-12
    parts = LF.project(X, E, rows=(0, 2)) + LF.project(X, E, rows=(2, 4))
    assert np.abs(parts - got).max() < 1e-12


def test_selection_matrix_reduces_to_plain_attention_on_the_selected_tokens():
    """E = F = columns of the identity: the projected keys are a subset of the tokens, so the
    result is ordinary attention (Eq. 1) to that subset; with K = L it is full attention."""
    B, Z, L, A = 1, 2, 8, 4
    Q, Kx, V = rnd((B, Z, L, A), 3), rnd((B, Z, L, A), 4), rnd((B, Z, L, A), 5)
    sel = [5, 0, 6]
    E = np.zeros((L, len(sel)))
    for j, t in enumerate(sel):
        E[t, j] = 1.0
    O, lse = LF.forward(Q, LF.project(Kx, E), LF.project(V, E))
    s = np.einsum("bzia,bzja->bzij", Q, Kx[:, :, sel]) / np.sqrt(A)
    p = np.exp(s - s.max(-1, keepdims=True))
    p /= p.sum(-1, keepdims=True)
    assert np.abs(O - np.einsum("bzij,bzja->bzia", p, V[:, :, sel])).max() < 1e-12
    I = np.eye(L)
    O_full, _ = LF.forward(Q, LF.project(Kx, I), LF.project(V, I))
    O_ref, _ = oracle.forward(Q, Kx, V)
    assert np.abs(O_full - O_ref).max() < 1e-12


def test_averaging_projection_of_constant_values():
    """All value rows equal v and F columns summing to one: every projected value is v, so O = v."""
    B, Z, L, A, K = 1, 1, 8, 4, 2
    v = rnd((A,), 6)
    V = np.broadcast_to(v, (B, Z, L, A)).copy()
    F = np.abs(rnd((L, K), 7)); F /= F.sum(0, keepdims=True)
    O, _ = LF.forward(rnd((B, Z, L, A), 8), LF.project(rnd((B, Z, L, A), 9), rnd((L, K), 10)), LF.project(V, F))
    assert np.abs(O - v).max() < 1e-12


def test_whole_chain_backward_against_torch_autograd_and_finite_differences():
    B, Z, L, A, K = 1, 2, 6, 4, 3
    Q, Kx, V, dO = (rnd((B, Z, L, A), s) for s in (11, 12, 13, 14))
    E, F = rnd((L, K), 15), rnd((L, K), 16)
    Kp, Vp = LF.project(Kx, E), LF.project(V, F)
    dQ, dKp, dVp = LF.backward(Q, Kp, Vp, dO)
    dK, dE = LF.project_bwd(dKp, Kx, E)
    dV, dF = LF.project_bwd(dVp, V, F)
    t = {k: torch.tensor(v, requires_grad=True) for k, v in dict(Q=Q, K=Kx, V=V, E=E, F=F).items()}
    kp = torch.einsum("lk,bzla->bzka", t["E"], t["K"])
    vp = torch.einsum("lk,bzla->bzka", t["F"], t["V"])
    p = torch.softmax(torch.einsum("bzia,bzka->bzik", t["Q"], kp) / np.sqrt(A), dim=-1)
    (torch.einsum("bzik,bzka->bzia", p, vp) * torch.tensor(dO)).sum().backward()
    for name, got in dict(Q=dQ, K=dK, V=dV, E=dE, F=dF).items():
        assert np.abs(got - t[name].grad.numpy()).max() < 1e-11, name

    def f(E_):
        O, _ = LF.forward(Q, LF.project(Kx, E_), Vp)
        return (O * dO).sum()
    eps = 1e-6
    for idx in [(0, 0), (3, 2), (5, 1)]:
        Ep, Em = E.copy(), E.copy(); Ep[idx] += eps; Em[idx] -= eps
        assert abs((f(Ep) - f(Em)) / (2 * eps) - dE[idx]) < 1e-6
    # a rank's share: gradients of E outside its rows are zero, inside they equal the whole's rows
    dK1, dE1 = LF.project_bwd(dKp, Kx, E, rows=(2, 3))
    assert np.array_equal(dE1[:2], np.zeros((2, K))) and np.abs(dE1[2:5] - dE[2:5]).max() < 1e-12
    assert np.abs(dK1[:, :, 2:5] - dK[:, :, 2:5]).max() < 1e-12 and not dK1[:, :, :2].any()
