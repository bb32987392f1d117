"""GPU parity of the Linformer variant (paper Table 3) with the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
from helpers import LSE_ATOL, check, download, upload
from paper_2105_13120_amd import inputs, rsa

pytestmark = pytest.mark.gpu
LF = oracle.linformer


def draw(shape, seed, scale=1.0):
    x = np.random.Generator(np.random.PCG64(seed)).standard_normal(shape) * scale
    return inputs.round_to_bf16(x)


def check_f32(name, got, ref):
    """fp32 output of bf16 products accumulated in fp32 (see tests/test_gpu_proj.py)."""
    rms = float(np.sqrt(np.mean(np.square(ref))))
    err = float(np.abs(got - ref).max())
    assert err <= 2e-4 * rms, f"{name}: max abs err {err:.3e} vs rms {rms:.3e}"


# (B, Z, L, N, ranks, Kp, A)
CASES = [
    (1, 1, 64, 1, (0, 1), 64, 64),
    (2, 2, 256, 2, (0, 2), 64, 64),
    (1, 3, 640, 5, (0, 5), 128, 64),
    (1, 2, 1024, 4, (1, 3), 192, 64),      # two ranks' share: partial projections and gradients
    (2, 4, 4096, 8, (0, 8), 256, 64),
    (1, 2, 64, 1, (0, 1), 256, 64),        # one tile of rows: the one-kernel backward without partial sums
    (1, 1, 256, 4, (1, 2), 128, 64),
    (3, 1, 1856, 1, (0, 1), 256, 64),      # 29 tiles per head: uneven shares of the rows
    (1, 1, 64, 1, (0, 1), 64, 128),        # heads of 128 elements
    (1, 3, 640, 5, (1, 4), 128, 128),
    (2, 2, 2048, 8, (0, 8), 256, 128),
]


@pytest.mark.parametrize("B,Z,L,N,ranks,Kp,A", CASES)
def test_linformer_chain(B, Z, L, N, ranks, Kp, A):
    c = L // N
    r0, rows = ranks[0] * c, (ranks[1] - ranks[0]) * c
    K, V = draw((B, Z, L, A), 1), draw((B, Z, L, A), 2)
    E, F = draw((L, Kp), 3, L ** -0.5), draw((L, Kp), 4, L ** -0.5)
    Q, dO = draw((B, Z, rows, A), 5), draw((B, Z, rows, A), 6)
    t = {k: upload(v, "bf16") for k, v in dict(K=K, V=V, E=E, F=F, Q=Q, dO=dO).items()}
    desc = rsa.make_desc(t["K"], N, rank_begin=ranks[0], rank_end=ranks[1])

    Kp_ = rsa.linformer_project(desc, t["K"], t["E"])
    Vp_ = rsa.linformer_project(desc, t["V"], t["F"])
    torch.cuda.synchronize()
    check("Kp", download(Kp_), LF.project(K, E, rows=(r0, rows)), "bf16")
    check("Vp", download(Vp_), LF.project(V, F, rows=(r0, rows)), "bf16")

    # each later stage is checked on the GPU's own rounded inputs
    Kp_h, Vp_h = download(Kp_), download(Vp_)
    O, LSE = rsa.linformer_forward(desc, t["Q"], Kp_, Vp_)
    dQ, dKp, dVp = rsa.linformer_backward(desc, t["dO"], t["Q"], Kp_, Vp_, O, LSE)
    torch.cuda.synchronize()
    O_ref, LSE_ref = LF.forward(Q, Kp_h, Vp_h)
    check("O", download(O), O_ref, "bf16")
    assert np.abs(download(LSE) - LSE_ref).max() <= LSE_ATOL
    dQ_ref, dKp_ref, dVp_ref = LF.backward(Q, Kp_h, Vp_h, dO)
    check("dQ", download(dQ), dQ_ref, "bf16")
    check("dKp", download(dKp), dKp_ref, "bf16")
    check("dVp", download(dVp), dVp_ref, "bf16")

    dK, dE = rsa.linformer_project_bwd(desc, dKp, t["K"], t["E"])
    torch.cuda.synchronize()
    dK_ref, dE_ref = LF.project_bwd(download(dKp), K, E, rows=(r0, rows))
    sl = slice(r0, r0 + rows)
    check("dK", download(dK)[:, :, sl], dK_ref[:, :, sl], "bf16")
    check_f32("dE", download(dE)[sl], dE_ref[sl])
    # rows of other ranks are left untouched (zero in the fresh outputs)
    other = np.ones(L, dtype=bool); other[sl] = False
    assert not download(dK)[:, :, other].any() and not download(dE)[other].any()


def test_linformer_chain_at_the_benchmark_size():
    """The setting bench.py times (section 4.4's upper bound: 114688 tokens, batch 4, 12 heads of 64,
    32 ranks, 256 projected keys), every stage on the GPU's own rounded inputs; the oracle runs on
    sampled heads (and, for dE, which sums over heads, on sampled token rows over all heads)."""
    B, Z, L, N, Kp, A = 4, 12, 114688, 32, 256, 64
    heads = [0, 13, 29, 47]

    def big(seed):   # (B, Z, L, A) drawn head by head in fp32 to bound the host memory
        rng = np.random.Generator(np.random.PCG64(seed))
        out = np.empty((B * Z, L, A), dtype=np.float32)
        for h in range(B * Z):
            out[h] = inputs.round_to_bf16(rng.standard_normal((L, A), dtype=np.float32))
        return out.reshape(B, Z, L, A)

    K, V, Q, dO = big(1), big(2), big(5), big(6)
    E, F = draw((L, Kp), 3, L ** -0.5), draw((L, Kp), 4, L ** -0.5)
    t = {k: upload(v, "bf16") for k, v in dict(K=K, V=V, E=E, F=F, Q=Q, dO=dO).items()}
    desc = rsa.make_desc(t["K"], N)
    hv = lambda a: np.ascontiguousarray(a.reshape(B * Z, *a.shape[2:])[heads][None].astype(np.float64))

    Kp_ = rsa.linformer_project(desc, t["K"], t["E"])
    Vp_ = rsa.linformer_project(desc, t["V"], t["F"])
    torch.cuda.synchronize()
    check("Kp", hv(download(Kp_)), LF.project(hv(K), E), "bf16")
    check("Vp", hv(download(Vp_)), LF.project(hv(V), F), "bf16")

    O, LSE = rsa.linformer_forward(desc, t["Q"], Kp_, Vp_)
    dQ, dKp, dVp = rsa.linformer_backward(desc, t["dO"], t["Q"], Kp_, Vp_, O, LSE)
    dK, dE = rsa.linformer_project_bwd(desc, dKp, t["K"], t["E"])
    torch.cuda.synchronize()
    Kp_h, Vp_h = hv(download(Kp_)), hv(download(Vp_))
    O_ref, LSE_ref = LF.forward(hv(Q), Kp_h, Vp_h)
    check("O", hv(download(O)), O_ref, "bf16")
    assert np.abs(download(LSE).reshape(B * Z, L)[heads][None] - LSE_ref).max() <= LSE_ATOL
    dQ_ref, dKp_ref, dVp_ref = LF.backward(hv(Q), Kp_h, Vp_h, hv(dO))
    check("dQ", hv(download(dQ)), dQ_ref, "bf16")
    check("dKp", hv(download(dKp)), dKp_ref, "bf16")
    check("dVp", hv(download(dVp)), dVp_ref, "bf16")
    dKp_h = download(dKp)
    dK_ref, _ = LF.project_bwd(hv(dKp_h), hv(K), E)
    check("dK", hv(download(dK)), dK_ref, "bf16")
    # dE[l, :] = sum over all heads of X[b, z, l, :] dXp[b, z]^T, on sampled token rows
    rows = np.concatenate([[0, 63, 64, 3583, 3584, L - 1],
                           np.random.Generator(np.random.PCG64(9)).integers(0, L, 250)])
    Xr = K[:, :, rows].astype(np.float64)                       # (B, Z, rows, A)
    dE_ref = np.einsum("bzra,bzka->rk", Xr, dKp_h)
    check_f32("dE", download(dE)[rows], dE_ref)


def test_linformer_error_codes():
    K = torch.zeros((1, 2, 256, 64), dtype=torch.bfloat16, device="cuda")
    E = torch.zeros((256, 96), dtype=torch.bfloat16, device="cuda")      # Kp = 96: not a multiple of 64
    with pytest.raises(rsa.RSAError) as e:
        rsa.linformer_project(rsa.make_desc(K, 2), K, E)
    assert e.value.status == -3
    E = torch.zeros((256, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(rsa.RSAError) as e:                                # no causal Linformer
        rsa.linformer_project(rsa.make_desc(K, 2, causal=True), K, E)
    assert e.value.status == -3
    with pytest.raises(rsa.RSAError) as e:
        rsa.linformer_project(rsa.make_desc(K, 2), K, E, ws=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -4
