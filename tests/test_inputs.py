"""Seeded input generator: determinism, shapes, bf16 rounding (CPU only)."""
import numpy as np
import torch

from paper_2105_13120_amd import inputs


def test_bf16_rounding_matches_library_conversion():
    rng = np.random.Generator(np.random.PCG64(5))
    x = np.concatenate([rng.standard_normal(4096) * 3,
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 65504.0, 1e-20, -3.3895e38]])
    ours = inputs.round_to_bf16(x)
    lib = torch.tensor(x, dtype=torch.float32).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(ours, lib)
    bits = inputs.bf16_bits(ours)
    np.testing.assert_array_equal(inputs.bf16_bits_to_f32(bits), ours)
    lib_bits = torch.tensor(x, dtype=torch.float32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bits, lib_bits)


def test_configs_shapes_and_flops():
    c = inputs.CONFIGS
    assert c["tiny_f32"].c == 64 and c["bert_base"].c == 128 and c["bert_large"].c == 256
    assert c["long_32k"].c == 2048 and c["rank15_64k_causal"].c == 4096
    r = c["rank15_64k_causal"]
    assert (r.q0, r.Lq) == (61440, 4096)
    # 15 full chunks + the lower triangle of the diagonal chunk (with diagonal)
    assert r.visible_pairs() == 15 * 4096 * 4096 + 4096 * 4097 // 2 == 260048896
    assert c["bert_large"].flops() == 12 * 8 * 16 * 64 * 2048 * 2048
    assert c["tiny_f32"].flops() == 4 * 2 * 64 * 256 * 256


def test_inputs_are_deterministic_and_rounded():
    cfg = inputs.CONFIGS["tiny_f32"]
    a, b = inputs.make_inputs(cfg), inputs.make_inputs(cfg)
    for k in ("Q", "K", "V", "dO"):
        np.testing.assert_array_equal(a[k], b[k])
        assert a[k].dtype == np.float32 and a[k].shape == (1, 2, 256, 64)
    small = inputs.RSAConfig("s", B=2, Z=3, L=64, A=64, N=4, dtype="bf16",
                             rank_begin=1, rank_end=3, qkv_scale=0.5)
    x = inputs.make_inputs(small)
    assert x["Q"].shape == (2, 3, 32, 64) and x["K"].shape == (2, 3, 64, 64)
    for k in x:
        np.testing.assert_array_equal(inputs.round_to_bf16(x[k]), x[k])
    assert abs(x["K"].std() - 0.5) < 0.02 and abs(x["dO"].std() - 1.0) < 0.05
    h = inputs.make_inputs(small, heads=2)
    np.testing.assert_array_equal(h["K"][0, 1], x["K"][0, 1])
    assert h["Q"].shape == (1, 2, 32, 64)


def test_zigzag_segments_cover_every_token_once_and_balance_the_causal_work():
    """Rank n owns half-chunks n and 2N-1-n: the ranks' rows partition the sequence
    and every rank sees the same number of keys under the causal mask."""
    N, L = 8, 4096
    seen = np.zeros(L, dtype=int)
    work = []
    for n in range(N):
        cfg = inputs.RSAConfig("z", B=1, Z=1, L=L, A=64, N=N, dtype="bf16", causal=True,
                               rank_begin=n, rank_end=n + 1, zigzag=True)
        segs = cfg.segments()
        assert [s[0] for s in segs] == [0, cfg.c // 2] and sum(s[2] for s in segs) == cfg.Lq
        for _, t0, m in segs:
            seen[t0:t0 + m] += 1
        # brute force count of visible pairs
        toks = np.concatenate([np.arange(t0, t0 + m) for _, t0, m in segs])
        assert cfg.visible_pairs() == int((toks + 1).sum())
        work.append(cfg.visible_pairs())
    assert (seen == 1).all()
    assert max(work) == min(work)
    whole = inputs.RSAConfig("z", B=1, Z=1, L=L, A=64, N=N, dtype="bf16", causal=True, zigzag=True)
    assert whole.visible_pairs() == L * (L + 1) // 2 == sum(work)
    # contiguous ownership: the last rank has (2N - 1) times the work of the first
    first = inputs.RSAConfig("c", B=1, Z=1, L=L, A=64, N=N, dtype="bf16", causal=True, rank_begin=0, rank_end=1)
    last = inputs.RSAConfig("c", B=1, Z=1, L=L, A=64, N=N, dtype="bf16", causal=True, rank_begin=N - 1, rank_end=N)
    assert last.visible_pairs() > 14 * first.visible_pairs()
