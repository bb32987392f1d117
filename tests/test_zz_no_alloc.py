"""rsa_backward_static (the workspace in the library's static device array, for callers that cannot
allocate) against rsa_backward with a caller's workspace: two calls in a row, the second on a smaller
input, so the second call meets the first call's leftovers in the shared array."""
import numpy as np
import pytest
import torch

from helpers import compare_heads, upload
from paper_2105_13120_amd import inputs, rsa

pytestmark = pytest.mark.gpu


def run_pair(cfg, deterministic):
    x = inputs.make_inputs(cfg)
    Q, K, V, dO = (upload(x[k], "bf16") for k in ("Q", "K", "V", "dO"))
    rb, re = cfg.ranks
    desc = rsa.make_desc(K, cfg.N, causal=cfg.causal, rank_begin=rb, rank_end=re, zigzag=cfg.zigzag,
                         deterministic=deterministic)
    assert 0 < rsa.workspace_bytes(desc, True) <= rsa.STATIC_SCRATCH_BYTES
    O, LSE = rsa.forward(desc, Q, K, V)
    ref = rsa.backward(desc, dO, Q, K, V, O, LSE)
    nan = lambda t: torch.full_like(t, float("nan"))
    got = rsa.backward_static(desc, dO, Q, K, V, O, LSE, nan(Q), nan(K), nan(V))
    torch.cuda.synchronize()
    heads = list(range(cfg.B * cfg.Z))
    errs = compare_heads(cfg, x, dict(O=O, LSE=LSE, dQ=got[0], dK=got[1], dV=got[2]), heads)
    for name, a, b in zip(("dQ", "dK", "dV"), got, ref):
        assert torch.equal(a, b), name                   # same kernels, same summation order
    return errs


@pytest.mark.parametrize("deterministic", [True, False])
def test_static_workspace_backward_twice_second_call_smaller(deterministic):
    # one rank's share of a long causal ring: the key walk is split, partial sums in the workspace
    first = inputs.RSAConfig("a", B=1, Z=2, L=4096, A=64, N=4, dtype="bf16", causal=True,
                             rank_begin=3, rank_end=4, seed=61)
    # a whole small ring: fewer rows, no split
    second = inputs.RSAConfig("b", B=1, Z=3, L=384, A=64, N=3, dtype="bf16", seed=67)
    run_pair(first, deterministic)
    run_pair(second, deterministic)
