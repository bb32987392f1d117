#!/usr/bin/env python3
"""Prints the error table of the design doc (GPU machine): per workload and output tensor, the fused HIP path's
max|err|/rms and rms(err)/rms against the fp64 oracle, next to the same two figures of the ideal bf16
pipeline (tests/bf16_model.py, P relative to a running maximum) on the same inputs.

The dense workloads (bert_base, bert_large) are compared on their first heads; the long ones on one
head, with the model evaluated block by block over the query rows (dK, dV on sampled key columns, all
query rows).  Run:  python tests/tolerance_table.py > gpurun_out/tolerance_table.md
"""
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

import oracle  # noqa: E402
from bf16_model import ideal_bf16_pipeline, r  # noqa: E402
from helpers import download, gpu_forward_backward, heads_view, row_tokens  # noqa: E402
from paper_2105_13120_amd import inputs, rsa  # noqa: E402


def stats(x, ref):
    rms = np.sqrt(np.mean(ref ** 2))
    d = np.abs(x - ref)
    return d.max() / rms, np.sqrt(np.mean(d ** 2)) / rms


def row(name, tensor, gpu, ideal, note=""):
    print(f"| {name} | {tensor} | {gpu[0]:.2e} | {ideal[0]:.2e} | {gpu[1]:.2e} | {ideal[1]:.2e} | {note} |", flush=True)


def dense(name, nheads):
    cfg = inputs.CONFIGS[name]
    x = inputs.make_inputs(cfg)
    out = gpu_forward_backward(cfg, x)
    heads = list(range(nheads))
    Q, K, V, dO = (heads_view(x[k], heads) for k in ("Q", "K", "V", "dO"))
    O_ref, LSE_ref = oracle.forward(Q, K, V)
    refs = dict(zip(("dQ", "dK", "dV"), oracle.backward(Q, K, V, dO)), O=O_ref)
    m = ideal_bf16_pipeline(Q, K, V, dO, reference="running_max")
    model = dict(O=m[0], dQ=m[2], dK=m[3], dV=m[4])
    for t in ("O", "dQ", "dK", "dV"):
        row(name, t, stats(heads_view(download(out[t]), heads), refs[t]), stats(model[t], refs[t]),
            f"first {nheads} of {cfg.B * cfg.Z} heads")
    lse = download(out["LSE"]).reshape(-1, cfg.Lq)[heads][None]
    print(f"| {name} | LSE (fp32) | {np.abs(lse - LSE_ref).max():.2e} abs | | | | |", flush=True)


def long(name, head, ncols=256, block=2048):
    """One head of a long workload; the model walks the query rows in blocks."""
    cfg = inputs.CONFIGS[name]
    x = inputs.make_inputs(cfg)
    out = gpu_forward_backward(cfg, x)
    Q, K, V, dO = (heads_view(x[k], [head])[0, 0] for k in ("Q", "K", "V", "dO"))
    s = 1.0 / np.sqrt(cfg.A)
    tok = row_tokens(cfg)
    cols = np.sort(np.random.Generator(np.random.PCG64(11)).choice(cfg.L, ncols, replace=False))
    rng = np.random.Generator(np.random.PCG64(20210525))
    O_m, dQ_m = np.empty_like(Q), np.empty_like(Q)
    dK_m, dV_m = np.zeros((ncols, cfg.A)), np.zeros((ncols, cfg.A))
    for r0 in range(0, cfg.Lq, block):
        sl = slice(r0, min(cfg.Lq, r0 + block))
        S = s * (Q[sl] @ K.T)
        if cfg.causal:
            S[np.arange(cfg.L)[None, :] > tok[sl, None]] = -np.inf
        mx = S.max(-1, keepdims=True)
        p = np.exp(S - mx)
        l = p.sum(-1, keepdims=True)
        u = np.exp2(rng.random((p.shape[0], 1)))
        O_m[sl] = r(((r(p / u) * u) @ V) / l)
        P = p / l
        D = (dO[sl] * O_m[sl]).sum(-1, keepdims=True)
        dS = r(P * (dO[sl] @ V.T - D))
        dQ_m[sl] = r(s * (dS @ K))
        dK_m += dS[:, cols].T @ Q[sl]
        dV_m += r(P[:, cols]).T @ dO[sl]
    dK_m, dV_m = r(s * dK_m), r(dV_m)
    O_ref = np.empty_like(Q)
    dQ_ref = np.empty_like(Q)
    dK_ref = dV_ref = None
    f4 = lambda a: np.ascontiguousarray(a[None, None])
    for s0, t0, n in cfg.segments():
        O_ref[s0:s0 + n] = oracle.forward(f4(Q[s0:s0 + n]), f4(K), f4(V), q0=t0, causal=cfg.causal)[0][0, 0]
        g = oracle.backward(f4(Q[s0:s0 + n]), f4(K), f4(V), f4(dO[s0:s0 + n]), q0=t0, causal=cfg.causal, cols=cols)
        dQ_ref[s0:s0 + n] = g[0][0, 0]
        dK_ref = g[1][0, 0] if dK_ref is None else dK_ref + g[1][0, 0]
        dV_ref = g[2][0, 0] if dV_ref is None else dV_ref + g[2][0, 0]
    gpu = {t: download(out[t]).reshape(-1, download(out[t]).shape[2], cfg.A)[head] for t in ("O", "dQ", "dK", "dV")}
    note = f"head {head}"
    row(name, "O", stats(gpu["O"], O_ref), stats(O_m, O_ref), note + ", all rows")
    row(name, "dQ", stats(gpu["dQ"], dQ_ref), stats(dQ_m, dQ_ref), note + ", all rows")
    row(name, "dK", stats(gpu["dK"][cols], dK_ref), stats(dK_m, dK_ref), note + f", {ncols} key columns")
    row(name, "dV", stats(gpu["dV"][cols], dV_ref), stats(dV_m, dV_ref), note + f", {ncols} key columns")


def main():
    import torch
    assert torch.cuda.is_available()
    cfg = inputs.CONFIGS["tiny_f32"]
    x = inputs.make_inputs(cfg)
    out = gpu_forward_backward(cfg, x, mode=rsa.MODE_STAGED, backward=False)
    O_ref, LSE_ref = oracle.forward(*(x[k].astype(np.float64) for k in ("Q", "K", "V")))
    print(f"tiny_f32 (fp32, staged, forward only): max abs err O {np.abs(download(out['O']) - O_ref).max():.2e}, "
          f"LSE {np.abs(download(out['LSE']) - LSE_ref).max():.2e}  (bar 1e-4)\n")
    print("| workload | tensor | GPU max err / rms | ideal max err / rms | GPU rms err / rms | ideal rms err / rms | compared on |")
    print("|---|---|---|---|---|---|---|")
    dense("bert_base", 48)
    dense("bert_large", 16)
    long("long_32k", 5)
    long("rank15_64k_causal", 11)


if __name__ == "__main__":
    main()
