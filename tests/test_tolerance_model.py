"""Where the bf16 tolerance comes from (CPU only).

An otherwise exact fp64 pipeline that rounds only what any bf16 matrix-core
path must round -- P and dS as MFMA operands, O before it enters D, and the
stored outputs -- is compared with the oracle.  Its largest error exceeds
2e-2 of the RMS (the tensors are heavy-tailed and these roundings are relative
to the element), stays inside the mixed bound the GPU tests use, and its RMS
error is a few 1e-3 of the RMS.  The emulation below is test-only arithmetic
written from the oracle's step list; it is not the GPU path and not the oracle.
"""
import numpy as np

import oracle
from helpers import BF16_REL_RMS, BF16_REL_RMS_MEAN, BF16_RTOL, check, dq_extra
from paper_2105_13120_amd import inputs


def r(a):
    return inputs.round_to_bf16(np.asarray(a, dtype=np.float32)).astype(np.float64)


def ideal_bf16_pipeline(Q, K, V, dO, s):
    S = s * Q @ K.transpose(0, 1, 3, 2)
    m = S.max(-1, keepdims=True)
    p = np.exp(S - m)
    l = p.sum(-1, keepdims=True)
    O = r((r(p) @ V) / l)
    P = p / l
    dP = dO @ V.transpose(0, 1, 3, 2)
    D = (dO * O).sum(-1, keepdims=True)
    dS = r(P * (dP - D))
    dQ = r(s * dS @ K)
    dK = r(s * dS.transpose(0, 1, 3, 2) @ Q)
    dV = r(r(P).transpose(0, 1, 3, 2) @ dO)
    return O, dQ, dK, dV


def test_ideal_bf16_pipeline_breaks_max_over_rms_but_meets_the_mixed_bound():
    cfg = inputs.RSAConfig("t", B=2, Z=4, L=512, A=64, N=1, dtype="bf16", seed=0)
    x = inputs.make_inputs(cfg)
    Q, K, V, dO = (x[k].astype(np.float64) for k in ("Q", "K", "V", "dO"))
    O_ref, _ = oracle.forward(Q, K, V)
    refs = (O_ref,) + oracle.backward(Q, K, V, dO)
    got = ideal_bf16_pipeline(Q, K, V, dO, 0.125)
    over = 0
    for name, g, ref in zip(("O", "dQ", "dK", "dV"), got, refs):
        rms = np.sqrt(np.mean(ref ** 2))
        assert np.abs(ref).max() / rms > 6.0                 # heavy tails
        over += np.abs(g - ref).max() / rms > BF16_REL_RMS
        mean = np.sqrt(np.mean((g - ref) ** 2)) / rms
        assert mean < BF16_REL_RMS_MEAN / 1.5
        check(name, g, ref, "bf16")                          # the bound the GPU tests use
    assert over >= 3       # the plain max/rms reading fails for most tensors even here


def test_check_rejects_small_systematic_errors():
    ref = np.random.Generator(np.random.PCG64(1)).standard_normal((1, 1, 256, 64))
    check("ok", r(ref), ref, "bf16")
    for bad in (ref * 1.02, ref + 0.03, np.where(np.abs(ref) < 0.5, ref * 1.05, ref)):
        try:
            check("bad", bad, ref, "bf16")
        except AssertionError:
            continue
        raise AssertionError("check accepted a wrong tensor")


def test_rounding_of_the_stored_O_inside_D_needs_its_own_term_on_the_first_causal_rows():
    """Token 1 of a causal sequence sees two keys; D_1 = dO_1 . O_1 is formed from the bf16 O_1 and
    its error enters dS_10 and dS_11 with one sign.  On this input (found by the seeded random-shape
    GPU tests) the ideal pipeline is 1.3 times the mixed bound at that row and meets the bound
    widened by dq_extra; no later row comes near."""
    cfg = inputs.RSAConfig("r", B=1, Z=3, L=4096, A=64, N=8, dtype="bf16", causal=True, seed=193410553,
                           rank_begin=0, rank_end=5, zigzag=True)
    x = inputs.make_inputs(cfg)
    n = 256   # rank 0's first half-chunk: tokens 0..255, which see only themselves
    Q, K, V, dO = (x[k][:, :1, :n].astype(np.float64) for k in ("Q", "K", "V", "dO"))
    s = 0.125
    S = s * Q @ K.transpose(0, 1, 3, 2)
    S[..., np.triu(np.ones((n, n), bool), 1)] = -np.inf
    p = np.exp(S - S.max(-1, keepdims=True))
    l = p.sum(-1, keepdims=True)
    O = r((r(p) @ V) / l)
    P = p / l
    D = (dO * O).sum(-1, keepdims=True)
    dQ = r(s * r(P * (dO @ V.transpose(0, 1, 3, 2) - D)) @ K)
    O_ref, _ = oracle.forward(Q, K, V, causal=True)
    dQ_ref = oracle.backward(Q, K, V, dO, causal=True)[0]
    # the RMS that normalises the bound is that of the whole head (2560 rows, most of them late)
    Kf, Vf = (x[k][:, :1].astype(np.float64) for k in ("K", "V"))
    sq = 0.0
    for r0, t0, m in cfg.segments():
        g = oracle.backward(x["Q"][:, :1, r0:r0 + m].astype(np.float64), Kf, Vf,
                            x["dO"][:, :1, r0:r0 + m].astype(np.float64), q0=t0, causal=True)[0]
        sq += float(np.sum(g ** 2))
    rms = np.sqrt(sq / (cfg.Lq * 64))
    plain = BF16_REL_RMS * rms + BF16_RTOL * np.abs(dQ_ref).max(-1, keepdims=True)
    ratio = np.abs(dQ - dQ_ref) / plain
    assert ratio[0, 0, 1].max() > 1.2 and ratio[0, 0, 8:].max() < 0.8
    check("dQ", dQ, dQ_ref, "bf16", extra=dq_extra(Q, K, V, dO, O_ref, 0, True))
    # the term is negligible where a row sees many keys
    x_ = dq_extra(Q, K, V, dO, O_ref, 0, True)
    assert (x_[0, 0, 128:] < 0.25 * plain[0, 0, 128:]).all()
