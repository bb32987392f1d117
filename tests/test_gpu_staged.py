"""GPU parity of the staged (two-pass) kernels against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from helpers import check, compare_heads, download, gpu_forward_backward, upload
from paper_2105_13120_amd import inputs, rsa

pytestmark = pytest.mark.gpu


def small_cfg(dtype, causal=False, B=2, Z=2, L=256, N=4, rb=0, re=-1, seed=3, A=64):
    return inputs.RSAConfig("t", B=B, Z=Z, L=L, A=A, N=N, dtype=dtype, causal=causal,
                            rank_begin=rb, rank_end=re, seed=seed)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("causal", [False, True])
def test_each_step_against_the_oracle(dtype, causal):
    """Every named step of one rank's ring walk, checked on its own output."""
    cfg = small_cfg(dtype, causal, rb=1, re=3)      # ranks 1 and 2 of 4; check rank n = 2
    x = inputs.make_inputs(cfg)
    n, c, L, N = 2, cfg.c, cfg.L, cfg.N
    heads = cfg.B * cfg.Z
    rows = slice((n - 1) * c, (n - 0) * c)           # rank n's rows inside Q (which starts at rank 1)
    Q, K, V, dO = (upload(x[k], dtype) for k in ("Q", "K", "V", "dO"))
    desc = rsa.make_desc(K, N, causal=causal, rank_begin=1, rank_end=3, mode=rsa.MODE_STAGED)
    tdt = Q.dtype
    dev = Q.device
    q64 = x["Q"][:, :, rows].astype(np.float64)
    do64 = x["dO"][:, :, rows].astype(np.float64)
    k64, v64 = x["K"].astype(np.float64), x["V"].astype(np.float64)
    O_ref, LSE_ref, S_ref, P_ref = oracle.forward(q64, k64, v64, q0=n * c, causal=causal, want_scores=True)
    dQ_ref, dK_ref, dV_ref, dP_ref, dS_ref = oracle.backward(q64, k64, v64, do64, q0=n * c,
                                                            causal=causal, want_scores=True)

    # stage 1: S^n_j for every ring step
    S = torch.full((cfg.B, cfg.Z, c, L), float("nan"), dtype=torch.float32, device=dev)
    for t in range(N):
        rsa.qk_step(desc, n, (n - t) % N, Q, K, S)
    S_h = download(S)
    assert np.array_equal(np.isneginf(S_h), np.isneginf(S_ref))
    fin = np.isfinite(S_ref)
    tol = 1e-5 if dtype == "f32" else 1e-5  # inputs are exact in both; fp32 accumulate
    assert np.abs(S_h[fin] - S_ref[fin]).max() < tol * 10

    # softmax over the full row
    P = torch.empty((cfg.B, cfg.Z, c, L), dtype=tdt, device=dev)
    LSE = torch.zeros((cfg.B, cfg.Z, cfg.Lq), dtype=torch.float32, device=dev)
    rsa.row_softmax(desc, n, S, P, LSE)
    P_h = download(P)
    assert np.abs(P_h - P_ref).max() <= (1e-6 if dtype == "f32" else 2 ** -8 * P_ref.max())
    assert np.abs(download(LSE)[:, :, rows] - LSE_ref).max() < 1e-4
    assert (download(LSE)[:, :, : (n - 1) * c] == 0).all()      # other ranks' rows untouched

    # stage 2: O^n = sum_j P^n_j V^j, accumulated step by step
    Oacc = torch.empty((cfg.B, cfg.Z, c, 64), dtype=torch.float32, device=dev)
    first = True
    for t in range(N):
        j = (n - t) % N
        rsa.av_step(desc, n, j, P, V, Oacc, not first)
        first = False
    check("Oacc", download(Oacc), O_ref, dtype)
    Ost = torch.empty((cfg.B, cfg.Z, c, 64), dtype=tdt, device=dev)
    rsa.store(desc, Oacc, Ost)
    check("O", download(Ost), O_ref, dtype)

    # backward steps.  D from the oracle's O rounded to the storage dtype.
    O_full = torch.zeros_like(Q)
    O_full[:, :, rows] = torch.from_numpy(O_ref).to(tdt).cuda()
    D = torch.zeros((cfg.B, cfg.Z, cfg.Lq), dtype=torch.float32, device=dev)
    rsa.bwd_rowdot(desc, n, dO, O_full, D)
    D_ref = (do64 * download(O_full[:, :, rows])).sum(-1)
    assert np.abs(download(D)[:, :, rows] - D_ref).max() < 1e-4

    dP = torch.empty_like(S)
    for t in range(N):
        rsa.dp_step(desc, n, (n - t) % N, dO, V, dP)
    assert np.abs(download(dP) - dP_ref).max() < 1e-4

    dS = torch.empty_like(P)
    rsa.softmax_bwd(desc, n, P, dP, D, dS)
    if dtype == "f32":
        assert np.abs(download(dS) - dS_ref).max() < 1e-5
    else:
        # element by element: dS = bf16(bf16(P) (dP - D)) is two roundings of unit roundoff 2^-8
        # each, plus P times the error that the rounding of O left in D
        dD = np.abs(download(D)[:, :, rows] - (do64 * O_ref).sum(-1))[..., None]
        bound = 2.05 * 2.0 ** -8 * np.abs(dS_ref) + 1.01 * P_ref * dD + 1e-7
        assert (np.abs(download(dS) - dS_ref) <= bound).all()

    dQacc = torch.empty((cfg.B, cfg.Z, c, 64), dtype=torch.float32, device=dev)
    dKacc = torch.zeros((cfg.B, cfg.Z, L, 64), dtype=torch.float32, device=dev)
    dVacc = torch.zeros_like(dKacc)
    first = True
    for t in range(N):
        j = (n - t) % N
        rsa.dq_step(desc, n, j, dS, K, dQacc, not first)
        rsa.dk_step(desc, n, j, dS, Q, dKacc, False)     # each chunk is visited once
        rsa.dv_step(desc, n, j, P, dO, dVacc, False)
        first = False
    check("dQ", download(dQacc), dQ_ref, dtype)
    check("dK", download(dKacc), dK_ref, dtype)
    check("dV", download(dVacc), dV_ref, dtype)


def test_config_tiny_f32_forward():
    """The small fp32 workload (tiny_f32: B1 Z2 L256 N4), forward only, max abs err <= 1e-4."""
    cfg = inputs.CONFIGS["tiny_f32"]
    x = inputs.make_inputs(cfg)
    out = gpu_forward_backward(cfg, x, mode=rsa.MODE_STAGED, backward=False)
    errs = compare_heads(cfg, x, out, [0, 1], backward=False, mode=rsa.MODE_STAGED)
    assert errs["O"] <= 1e-4


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("causal,rb,re", [(False, 0, -1), (True, 0, -1), (False, 1, 3), (True, 2, 4)])
def test_staged_forward_backward(dtype, causal, rb, re):
    cfg = small_cfg(dtype, causal, B=1, Z=3, L=384, N=6, rb=rb, re=re, seed=11)
    x = inputs.make_inputs(cfg)
    out = gpu_forward_backward(cfg, x, mode=rsa.MODE_STAGED)
    compare_heads(cfg, x, out, [0, 1, 2], mode=rsa.MODE_STAGED)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("A,causal,rb,re", [(128, False, 0, -1), (128, True, 1, 3), (192, True, 0, -1)])
def test_staged_heads_wider_than_64(dtype, A, causal, rb, re):
    """The two-pass layout takes any head size that is a multiple of 64 (up to 256)."""
    cfg = small_cfg(dtype, causal, B=1, Z=2, L=384, N=3, rb=rb, re=re, seed=29, A=A)
    x = inputs.make_inputs(cfg)
    out = gpu_forward_backward(cfg, x, mode=rsa.MODE_STAGED)
    compare_heads(cfg, x, out, [0, 1], mode=rsa.MODE_STAGED)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("L,N,causal", [(5120, 5, False), (8192, 4, True)])
def test_staged_forward_with_long_rows(dtype, L, N, causal):
    """Rows of more than 4096 scores: the softmax keeps a row in the registers of one work-group."""
    cfg = small_cfg(dtype, causal, B=1, Z=1, L=L, N=N, rb=N - 1, re=N, seed=31)
    x = inputs.make_inputs(cfg)
    out = gpu_forward_backward(cfg, x, mode=rsa.MODE_STAGED, backward=False)
    compare_heads(cfg, x, out, [0], backward=False, mode=rsa.MODE_STAGED)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_staged_explicit_softmax_scale(dtype):
    """rsa_desc.scale other than 1/sqrt(A) through the two-pass kernels."""
    import dataclasses
    cfg = dataclasses.replace(small_cfg(dtype, True, B=1, Z=2, L=384, N=3, seed=73), att_scale=0.2)
    x = inputs.make_inputs(cfg)
    out = gpu_forward_backward(cfg, x, mode=rsa.MODE_STAGED)
    compare_heads(cfg, x, out, [0, 1], mode=rsa.MODE_STAGED)
