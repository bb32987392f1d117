"""Seeded synthetic inputs for Ring Self-Attention, shared by tests, bench and smoke.

This module holds no attention arithmetic: it draws iid normal Q, K, V, dO with
numpy's PCG64 generator (draw order Q, K, V, dO), scales them, and rounds them
to the storage dtype (bf16 round-to-nearest-even, or fp32).  The rounded values
are what both the GPU path and the CPU oracle receive.

The shapes stand in for the paper's BERT Base (Z=12, A=64) and BERT Large
(Z=16, A=64) attention blocks (section 4.1); the paper's Wikipedia data is not
needed because attention cost depends on shapes only.
"""
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class RSAConfig:
    """One workload: (B, Z, L, A) split into N ring chunks of c = L/N rows."""
    name: str
    B: int
    Z: int
    L: int
    A: int
    N: int
    dtype: str            # "f32" or "bf16"
    causal: bool = False
    rank_begin: int = 0   # simulated ranks [rank_begin, rank_end)
    rank_end: int = -1    # -1: N
    qkv_scale: float = 1.0
    backward: bool = True
    seed: int = 0
    zigzag: bool = False  # rank n owns half-chunks n and 2N-1-n instead of chunk n
    att_scale: float = 0.0  # the softmax scale handed to the library; 0 selects 1/sqrt(A)

    @property
    def c(self):
        return self.L // self.N

    @property
    def ranks(self):
        end = self.N if self.rank_end < 0 else self.rank_end
        return self.rank_begin, end

    @property
    def q0(self):
        return self.ranks[0] * self.c

    @property
    def Lq(self):
        b, e = self.ranks
        return (e - b) * self.c

    def segments(self):
        """The local query rows as runs of consecutive tokens: a list of
        (local_row, first_token, length), in local order."""
        b, e = self.ranks
        if not self.zigzag:
            return [(0, b * self.c, (e - b) * self.c)]
        h = self.c // 2
        out = []
        for n in range(b, e):
            out.append(((n - b) * self.c, n * h, h))
            out.append(((n - b) * self.c + h, (2 * self.N - 1 - n) * h, h))
        return out

    def visible_pairs(self):
        """Number of (query, key) pairs per head that are not masked."""
        if not self.causal:
            return self.Lq * self.L
        # row i (global) sees i + 1 keys
        return sum(n * t0 + n * (n + 1) // 2 for _, t0, n in self.segments())

    def flops(self, backward=None):
        """Algorithmic flops: 4 per pair per head-dim forward, 8 backward."""
        backward = self.backward if backward is None else backward
        per_pair = 4 + (8 if backward else 0)
        return per_pair * self.B * self.Z * self.A * self.visible_pairs()


CONFIGS = {
    "tiny_f32": RSAConfig("tiny_f32", B=1, Z=2, L=256, A=64, N=4, dtype="f32",
                          backward=False),
    "bert_base": RSAConfig("bert_base", B=16, Z=12, L=512, A=64, N=4, dtype="bf16"),
    "bert_large": RSAConfig("bert_large", B=8, Z=16, L=2048, A=64, N=8, dtype="bf16"),
    "long_32k": RSAConfig("long_32k", B=1, Z=16, L=32768, A=64, N=16, dtype="bf16",
                          qkv_scale=0.5),
    "rank15_64k_causal": RSAConfig("rank15_64k_causal", B=1, Z=12, L=65536, A=64,
                                   N=16, dtype="bf16", causal=True,
                                   rank_begin=15, rank_end=16),
    # The causal extension over the whole ring, and one rank's share of the 64K ring when
    # ownership is zig-zag (every rank then has the same share; rank 0 stands for all).
    "causal_ring_32k": RSAConfig("causal_ring_32k", B=1, Z=16, L=32768, A=64, N=16,
                                 dtype="bf16", causal=True, qkv_scale=0.5),
    "zigzag_rank0_64k_causal": RSAConfig("zigzag_rank0_64k_causal", B=1, Z=12, L=65536, A=64,
                                         N=16, dtype="bf16", causal=True,
                                         rank_begin=0, rank_end=1, zigzag=True),
    # Heads of 128 elements: the hidden size of BERT Large (1024) cut into 8 heads instead of 16.
    "wide_heads_8k": RSAConfig("wide_heads_8k", B=4, Z=8, L=8192, A=128, N=8, dtype="bf16"),
}


def round_to_bf16(x):
    """Round float values to the nearest bf16 (ties to even); returns float32."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x_f32):
    """uint16 bit patterns of float32 values that are exactly bf16-representable."""
    u = np.ascontiguousarray(x_f32, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits):
    """float32 values of uint16 bf16 bit patterns."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32)


def round_to_dtype(x, dtype):
    if dtype == "bf16":
        return round_to_bf16(x)
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    raise ValueError(f"unknown dtype {dtype!r}")


def make_inputs(cfg, heads=None):
    """Draw Q, K, V, dO for cfg.  Returns a dict of float32 arrays holding values
    exactly representable in cfg.dtype: Q, dO (B,Z,Lq,A); K, V (B,Z,L,A).

    heads: optional number of leading (b, z) pairs to keep, flattened as
    (1, heads, rows, A) -- a bounded sample of the same workload.
    """
    rng = np.random.Generator(np.random.PCG64(cfg.seed))
    out = {}
    for name, rows, scale in (("Q", cfg.Lq, cfg.qkv_scale), ("K", cfg.L, cfg.qkv_scale),
                              ("V", cfg.L, cfg.qkv_scale), ("dO", cfg.Lq, 1.0)):
        x = rng.standard_normal((cfg.B, cfg.Z, rows, cfg.A), dtype=np.float64)
        if scale != 1.0:
            x *= scale
        x = round_to_dtype(x, cfg.dtype)
        if heads is not None:
            x = np.ascontiguousarray(
                x.reshape(1, cfg.B * cfg.Z, rows, cfg.A)[:, :heads])
        out[name] = x
    return out
