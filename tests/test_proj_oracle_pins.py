"""Pins of the projection oracle (the Q/K/V and Linear rows of the paper's Table 2) against
things other than itself: scalar loops, layout-only special cases, finite differences and
torch.autograd in float64."""
import numpy as np
import torch

import oracle

P = oracle.proj


def rnd(shape, seed):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape)


def test_qkv_proj_against_scalar_loops():
    B, rows, H, Z, A = 2, 3, 5, 2, 4
    X, W = rnd((B, rows, H), 1), rnd((H, 3 * Z * A), 2)
    got = P.qkv_proj(X, W, Z, A)
    for which in range(3):
        for b in range(B):
            for z in range(Z):
                for r in range(rows):
                    for a in range(A):
                        want = sum(X[b, r, h] * W[h, which * Z * A + z * A + a] for h in range(H))
                        assert abs(got[which][b, z, r, a] - want) < 1e-12


def test_out_proj_against_scalar_loops():
    B, rows, H, Z, A = 2, 3, 5, 2, 4
    O, Wo = rnd((B, Z, rows, A), 3), rnd((Z * A, H), 4)
    got = P.out_proj(O, Wo)
    assert got.shape == (B, rows, H)
    for b in range(B):
        for r in range(rows):
            for h in range(H):
                want = sum(O[b, z, r, a] * Wo[z * A + a, h] for z in range(Z) for a in range(A))
                assert abs(got[b, r, h] - want) < 1e-12


def test_identity_weights_only_change_the_layout():
    """H = Z*A and identity blocks: Q = K = V = X with heads split off, and the Linear row undoes it."""
    B, rows, Z, A = 2, 6, 3, 4
    H = Z * A
    X = rnd((B, rows, H), 5)
    W = np.concatenate([np.eye(H), 2 * np.eye(H), -np.eye(H)], axis=1)
    Q, K, V = P.qkv_proj(X, W, Z, A)
    for b in range(B):
        for z in range(Z):
            assert np.array_equal(Q[b, z], X[b, :, z * A:(z + 1) * A])
    assert np.array_equal(K, 2 * Q) and np.array_equal(V, -Q)
    assert np.array_equal(P.out_proj(Q, np.eye(H)), X)


def test_one_hot_input_picks_a_weight_row():
    Z, A, H = 2, 3, 4
    W = rnd((H, 3 * Z * A), 6)
    X = np.zeros((1, 1, H)); X[0, 0, 2] = 1.0
    Q, K, V = P.qkv_proj(X, W, Z, A)
    assert np.array_equal(Q.reshape(-1), W[2, :Z * A])
    assert np.array_equal(V.reshape(-1), W[2, 2 * Z * A:])


def test_backward_against_torch_autograd_and_finite_differences():
    B, rows, H, Z, A = 2, 3, 5, 2, 4
    X, W, Wo = rnd((B, rows, H), 7), rnd((H, 3 * Z * A), 8), rnd((Z * A, H), 9)
    gQ, gK, gV = (rnd((B, Z, rows, A), s) for s in (10, 11, 12))
    gY = rnd((B, rows, H), 13)
    # library second opinion
    Xt, Wt = torch.tensor(X, requires_grad=True), torch.tensor(W, requires_grad=True)
    Yt = (Xt @ Wt).reshape(B, rows, 3, Z, A).permute(2, 0, 3, 1, 4)
    f = (Yt[0] * torch.tensor(gQ)).sum() + (Yt[1] * torch.tensor(gK)).sum() + (Yt[2] * torch.tensor(gV)).sum()
    f.backward()
    dX, dW = P.qkv_proj_bwd(gQ, gK, gV, X, W)
    assert np.abs(dX - Xt.grad.numpy()).max() < 1e-12 and np.abs(dW - Wt.grad.numpy()).max() < 1e-12
    O = rnd((B, Z, rows, A), 14)
    Ot, Wot = torch.tensor(O, requires_grad=True), torch.tensor(Wo, requires_grad=True)
    ((Ot.permute(0, 2, 1, 3).reshape(B, rows, Z * A) @ Wot) * torch.tensor(gY)).sum().backward()
    dO, dWo = P.out_proj_bwd(gY, O, Wo)
    assert np.abs(dO - Ot.grad.numpy()).max() < 1e-12 and np.abs(dWo - Wot.grad.numpy()).max() < 1e-12
    # central differences of f = sum(out_proj(O, Wo) * gY) in a few coordinates
    eps = 1e-6
    for idx in [(0, 0, 0, 0), (1, 1, 2, 3)]:
        Op, Om = O.copy(), O.copy(); Op[idx] += eps; Om[idx] -= eps
        fd = ((P.out_proj(Op, Wo) - P.out_proj(Om, Wo)) * gY).sum() / (2 * eps)
        assert abs(fd - dO[idx]) < 1e-6
    for idx in [(0, 0), (7, 4)]:
        Wp, Wm = Wo.copy(), Wo.copy(); Wp[idx] += eps; Wm[idx] -= eps
        fd = ((P.out_proj(O, Wp) - P.out_proj(O, Wm)) * gY).sum() / (2 * eps)
        assert abs(fd - dWo[idx]) < 1e-6
    for idx in [(0, 0, 0), (1, 2, 4)]:
        Xp, Xm = X.copy(), X.copy(); Xp[idx] += eps; Xm[idx] -= eps
        qp, qm = P.qkv_proj(Xp, W, Z, A), P.qkv_proj(Xm, W, Z, A)
        fd = sum(((a - b) * g).sum() for a, b, g in zip(qp, qm, (gQ, gK, gV))) / (2 * eps)
        assert abs(fd - dX[idx]) < 1e-6
    for idx in [(0, 0), (4, 23), (2, 9)]:
        Wp, Wm = W.copy(), W.copy(); Wp[idx] += eps; Wm[idx] -= eps
        qp, qm = P.qkv_proj(X, Wp, Z, A), P.qkv_proj(X, Wm, Z, A)
        fd = sum(((a - b) * g).sum() for a, b, g in zip(qp, qm, (gQ, gK, gV))) / (2 * eps)
        assert abs(fd - dW[idx]) < 1e-6


def test_weight_gradients_add_over_row_blocks():
    """The ranks' weight gradients add up (the all-reduce of replicated weights)."""
    B, rows, H, Z, A = 1, 8, 5, 2, 4
    X, W = rnd((B, rows, H), 15), rnd((H, 3 * Z * A), 16)
    g = [rnd((B, Z, rows, A), s) for s in (17, 18, 19)]
    _, dW = P.qkv_proj_bwd(*g, X, W)
    parts = sum(P.qkv_proj_bwd(*[t[:, :, r:r + 4] for t in g], X[:, r:r + 4], W)[1] for r in (0, 4))
    assert np.abs(dW - parts).max() < 1e-12
