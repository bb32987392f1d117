"""Where the bf16 tolerance comes from (CPU only).

tests/bf16_model.py holds an otherwise exact fp64 pipeline that rounds only what any bf16
matrix-core path must round -- P and dS as MFMA operands, O before it enters D, and the stored
outputs.  Here it is compared with the oracle: the stated bar read literally (largest error <=
2e-2 of the RMS) fails already for the exact result rounded once to bf16; the pipeline sits at
a stated fraction of the bounds the GPU tests use; and a pipeline with one avoidable rounding
more (the planted mistake) is rejected by the comparison with the ideal pipeline.
"""
import numpy as np
import pytest

import oracle
from bf16_model import folded_scale_pipeline, ideal_bf16_pipeline, r, strip_bf16_pipeline
from helpers import (BF16_REL_RMS, BF16_REL_RMS_MEAN, BF16_RTOL, IDEAL_RMS_RATIO, check, dq_extra)
from paper_2105_13120_amd import inputs

NAMES = ("O", "dQ", "dK", "dV")


def case(causal=False, L=512, Z=4, A=64, seed=0, qkv_scale=1.0):
    cfg = inputs.RSAConfig("t", B=1, Z=Z, L=L, A=A, N=1, dtype="bf16", seed=seed, causal=causal,
                           qkv_scale=qkv_scale)
    x = inputs.make_inputs(cfg)
    Q, K, V, dO = (x[k].astype(np.float64) for k in ("Q", "K", "V", "dO"))
    O_ref, _ = oracle.forward(Q, K, V, causal=causal)
    refs = (O_ref,) + oracle.backward(Q, K, V, dO, causal=causal)
    return Q, K, V, dO, refs


def pick(m):
    return (m[0],) + tuple(m[2:])


def test_the_exact_result_rounded_to_bf16_breaks_the_literal_bar():
    """16 heads of 512 tokens: the largest element of O is more than 6 times the RMS, and rounding
    it to bf16 (unit roundoff 2^-8) alone leaves an error above 2e-2 of the RMS."""
    Q, K, V, dO, refs = case(Z=16)
    O = refs[0]
    rms = np.sqrt(np.mean(O ** 2))
    assert np.abs(O).max() / rms > 6.0
    assert np.abs(r(O) - O).max() / rms > BF16_REL_RMS


@pytest.mark.parametrize("causal,L,A,qkv_scale", [(False, 512, 64, 1.0), (True, 512, 64, 1.0),
                                                  (False, 1024, 64, 0.5), (True, 768, 128, 1.0)])
def test_ideal_pipeline_sits_at_a_stated_fraction_of_the_bounds(causal, L, A, qkv_scale):
    Q, K, V, dO, refs = case(causal, L, A=A, qkv_scale=qkv_scale)
    got = pick(ideal_bf16_pipeline(Q, K, V, dO, causal=causal))
    extra = dq_extra(Q, K, V, dO, refs[0], 0, causal)
    for name, g, ref in zip(NAMES, got, refs):
        rms = np.sqrt(np.mean(ref ** 2))
        bound = BF16_REL_RMS * rms + BF16_RTOL * np.abs(ref).max(-1, keepdims=True)
        if name == "dQ":
            bound = bound + extra
        worst = (np.abs(g - ref) / bound).max()
        assert 0.25 <= worst <= 0.92, (name, worst)          # criterion (1): headroom between 1.1 and 4
        mean = np.sqrt(np.mean((g - ref) ** 2)) / rms
        assert 1.8e-3 <= mean <= 2.7e-3, (name, mean)        # criterion (2) allows 3e-3
        check(name, g, ref, "bf16", extra=extra if name == "dQ" else None, ideal=g)


@pytest.mark.parametrize("causal", [False, True])
def test_running_max_and_strip_variants_of_the_model(causal):
    """An online softmax rounds P relative to a running maximum (the row's largest probability is
    then rounded like the rest): the same statistics as the two-pass model except on rows one key
    dominates.  The two-pass layout with a bf16 strip rounds P before dS is formed from it: RMS error
    of dQ and dK sqrt(1.5) = 1.22 times the ideal's.  Both stay inside criteria (1) and (2)."""
    Q, K, V, dO, refs = case(causal, 768)
    base = pick(ideal_bf16_pipeline(Q, K, V, dO, causal=causal))
    online = pick(ideal_bf16_pipeline(Q, K, V, dO, causal=causal, reference="running_max"))
    strip = pick(strip_bf16_pipeline(Q, K, V, dO, causal=causal))
    extra = dq_extra(Q, K, V, dO, refs[0], 0, causal)
    rmse = lambda g, ref: np.sqrt(np.mean((g - ref) ** 2))
    for i, name in enumerate(NAMES):
        x_ = extra if name == "dQ" else None
        check(name, online[i], refs[i], "bf16", extra=x_)
        check(name, strip[i], refs[i], "bf16", extra=x_, strip=True)
        # under the causal mask the first rows see few keys and the largest probability's own
        # rounding is most of their error: O is then 1.1 to 1.15 times the two-pass model's
        assert 0.95 <= rmse(online[i], refs[i]) / rmse(base[i], refs[i]) <= (1.2 if causal else 1.08), name
    for i in (1, 2):
        assert 1.15 <= rmse(strip[i], refs[i]) / rmse(base[i], refs[i]) <= 1.3, NAMES[i]


def test_a_second_rounding_of_a_scaled_operand_is_rejected():
    """The planted mistake: scores recomputed from bf16(K s log2e) / bf16(Q s log2e).  It stays
    inside the per-element bound (1) and is thrown out by the comparison with the ideal pipeline:
    its RMS error is 1.2 to 1.3 times the ideal's (at or just over the 3e-3 of criterion (2)) and
    its largest dQ, dK errors 2 to 3 times."""
    Q, K, V, dO, refs = case(Z=2)
    good = pick(ideal_bf16_pipeline(Q, K, V, dO))
    bad = pick(folded_scale_pipeline(Q, K, V, dO))
    assert np.array_equal(good[0], bad[0])                   # the forward is the same
    for name, g, b, ref in zip(NAMES[1:], good[1:], bad[1:], refs[1:]):
        rms = np.sqrt(np.mean(ref ** 2))
        bound = BF16_REL_RMS * rms + BF16_RTOL * np.abs(ref).max(-1, keepdims=True)
        assert (np.abs(b - ref) <= bound).all()              # criterion (1) alone accepts it
        ratio = np.sqrt(np.mean((b - ref) ** 2)) / np.sqrt(np.mean((g - ref) ** 2))
        assert ratio > IDEAL_RMS_RATIO + 0.05, (name, ratio)
        with pytest.raises(AssertionError, match="times the ideal|rms err / rms"):
            check(name, b, ref, "bf16", ideal=g)
    for name, i in (("dQ", 1), ("dK", 2)):
        assert np.abs(bad[i] - refs[i]).max() > 2.0 * np.abs(good[i] - refs[i]).max(), name


def test_check_rejects_small_systematic_errors():
    ref = np.random.Generator(np.random.PCG64(1)).standard_normal((1, 1, 256, 64))
    check("ok", r(ref), ref, "bf16")
    for bad in (ref * 1.01, ref + 0.025, np.where(np.abs(ref) < 0.5, ref * 1.03, ref)):
        with pytest.raises(AssertionError):
            check("bad", bad, ref, "bf16")


def test_rounding_of_the_stored_O_inside_D_needs_its_own_term_on_the_first_causal_rows():
    """Token 1 of a causal sequence sees two keys; D_1 = dO_1 . O_1 is formed from the bf16 O_1 and
    its error enters dS_10 and dS_11 with one sign.  On this input (a seeded random shape) the ideal
    pipeline is well over the per-element bound at that row and meets the bound widened by dq_extra;
    no later row comes near."""
    cfg = inputs.RSAConfig("r", B=1, Z=3, L=4096, A=64, N=8, dtype="bf16", causal=True, seed=193410553,
                           rank_begin=0, rank_end=5, zigzag=True)
    x = inputs.make_inputs(cfg)
    n = 256   # rank 0's first half-chunk: tokens 0..255, which see only themselves
    Q, K, V, dO = (x[k][:, :1, :n].astype(np.float64) for k in ("Q", "K", "V", "dO"))
    dQ = ideal_bf16_pipeline(Q, K, V, dO, causal=True)[2]
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
    assert ratio[0, 0, 1].max() > 1.5 and ratio[0, 0, 8:].max() < 1.0
    x_ = dq_extra(Q, K, V, dO, O_ref, 0, True)
    assert (np.abs(dQ - dQ_ref) <= plain + x_).all()
    # the term is negligible where a row sees many keys
    assert (x_[0, 0, 128:] < 0.3 * plain[0, 0, 128:]).all()
