"""The C-ABI library loads, exports every symbol the header declares, and
rejects bad arguments on the host before anything is launched (CPU only)."""
import ctypes
import os
import re

import pytest

from paper_2105_13120_amd import rsa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "rsa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rsa_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(names) == set(rsa.EXPORTS)
    L = rsa.lib()
    for n in names:
        assert hasattr(L, n), n
    assert L.rsa_version() >= 100


def desc(**kw):
    d = dict(B=1, Z=2, A=64, L=256, N=4, rank_begin=0, rank_end=4, causal=0,
             dtype=rsa.RSA_BF16, scale=0.0, flags=rsa.MODE_FUSED)
    d.update(kw)
    for k in ("q_stride", "kv_stride", "o_stride"):
        if k in d:
            d[k] = (ctypes.c_int64 * 3)(*d[k])
    return rsa.RSADesc(**d)


def fwd_status(d, ptr=0x1000, ws=0x1000, ws_bytes=1 << 40):
    p = ctypes.c_void_p(ptr)
    return rsa.lib().rsa_forward(ctypes.byref(d), p, p, p, p, p, ctypes.c_void_p(ws), ws_bytes, None)


def test_validation_happens_before_any_launch():
    # every call below must return on the host: the pointers are not device memory
    assert fwd_status(desc(N=3)) == -2                       # L % N != 0
    assert fwd_status(desc(L=0)) == -2
    assert fwd_status(desc(rank_begin=2, rank_end=2)) == -2
    assert fwd_status(desc(rank_end=5)) == -2
    assert fwd_status(desc(A=192)) == -3                     # the fused kernels: heads of 64 or 128
    assert rsa.workspace_bytes(desc(A=128), True) == 2 * (1 * 2 * 256 * 4)
    assert fwd_status(desc(A=96, flags=rsa.MODE_STAGED)) == -3
    assert fwd_status(desc(A=320, flags=rsa.MODE_STAGED)) == -3
    assert rsa.workspace_bytes(desc(A=128, flags=rsa.MODE_STAGED), False) > 0
    assert fwd_status(desc(L=128, N=4)) == -3                # c = 32 not a multiple of 64
    assert fwd_status(desc(dtype=7)) == -3
    assert fwd_status(desc(dtype=rsa.RSA_F32)) == -3         # fused mode is bf16 only
    assert fwd_status(desc(flags=9)) == -3
    assert fwd_status(desc(flags=rsa.MODE_STAGED | rsa.OWN_ZIGZAG)) == -3   # zig-zag: fused mode only
    assert fwd_status(desc(L=256, N=4, flags=rsa.OWN_ZIGZAG)) == -3          # half-chunk of 32 rows
    assert rsa.workspace_bytes(desc(L=512, N=4, flags=rsa.OWN_ZIGZAG), True) > 0
    # strides: all zero = dense; otherwise positive, row stride >= A, multiples of 8 elements
    dense = dict(q_stride=(2 * 256 * 64, 256 * 64, 64), kv_stride=(2 * 256 * 64, 256 * 64, 64))
    assert rsa.workspace_bytes(desc(**dense), True) == rsa.workspace_bytes(desc(), True)
    inter = dict(o_stride=(256 * 2 * 64, 64, 2 * 64))                   # heads interleaved (B, rows, Z, A)
    assert rsa.workspace_bytes(desc(**inter), True) > 0
    assert fwd_status(desc(kv_stride=(2 * 256 * 64, 256 * 64, 32))) == -2           # rows overlap
    assert fwd_status(desc(kv_stride=(2 * 256 * 64, 0, 64))) == -2
    assert fwd_status(desc(kv_stride=(2 * 256 * 68, 256 * 68, 68))) == -3           # not a multiple of 16 bytes
    assert fwd_status(desc(kv_stride=(1 << 40, 1 << 32, 1 << 25))) == -3            # row stride beyond 2^24
    assert fwd_status(desc(flags=rsa.MODE_STAGED, **inter)) == -3                   # the two-pass kernels are dense only
    pp = ctypes.c_void_p(0x1000)
    assert rsa.lib().rsa_qk_step(ctypes.byref(desc(**inter)), 0, 0, pp, pp, pp, None) == -3   # also step by step
    assert fwd_status(desc(), ptr=0) == -1
    assert fwd_status(desc(), ptr=0x1008) == -3              # misaligned
    staged = desc(flags=rsa.MODE_STAGED)
    assert rsa.workspace_bytes(staged, False) > 0
    assert fwd_status(staged, ws=0) == -4
    assert fwd_status(staged, ws_bytes=16) == -4
    assert rsa.lib().rsa_forward(None, None, None, None, None, None, None, 0, None) == -1
    p = ctypes.c_void_p(0x1000)
    bwd = rsa.lib().rsa_backward(ctypes.byref(desc()), p, p, p, p, p, p, p, p, p, None, 0, None)
    assert bwd == -4                                          # backward always needs D
    # the kernels of the backward on their own check their workspace on the host too
    L = rsa.lib()
    need = rsa.workspace_bytes(desc(flags=rsa.DETERMINISTIC), True)
    assert need == 2 * (1 * 2 * 256 * 4)
    assert L.rsa_bwd_dkdv(ctypes.byref(desc()), p, p, p, p, p, need - 1, p, p, None) == -4
    assert L.rsa_bwd_dkdv(ctypes.byref(desc()), p, p, p, p, None, need, p, p, None) == -4
    assert L.rsa_bwd_dq(ctypes.byref(desc()), p, p, p, p, p, need - 1, p, None) == -4
    assert L.rsa_bwd_dq(ctypes.byref(desc()), p, p, p, p, None, 1 << 30, p, None) == -4
    assert L.rsa_bwd_preprocess(ctypes.byref(desc()), p, p, p, p, need - 1, None) == -4
    split = desc(B=1, Z=2, L=4096, N=4, rank_begin=3, rank_end=4)   # split key walk: partial dQ behind the row terms
    assert L.rsa_bwd_dq(ctypes.byref(split), p, p, p, p, p, 2 * 2048 * 4, p, None) == -4
    # the variant with the static workspace rejects what does not fit, before touching the device
    big = desc(B=64, Z=16, L=65536, N=4)
    assert rsa.workspace_bytes(big, True) > rsa.STATIC_SCRATCH_BYTES
    assert L.rsa_backward_static(ctypes.byref(big), p, p, p, p, p, p, p, p, p, None) == -4
    assert L.rsa_backward_static(ctypes.byref(desc(N=3)), p, p, p, p, p, p, p, p, p, None) == -2
    assert L.rsa_backward_static(ctypes.byref(desc(flags=rsa.MODE_STAGED)), p, p, p, p, p, p, p, p, p, None) == -3
    step = rsa.lib().rsa_qk_step(ctypes.byref(staged), 4, 0, p, p, p, None)
    assert step == -2                                         # rank outside [begin, end)
    step = rsa.lib().rsa_qk_step(ctypes.byref(staged), 0, 7, p, p, p, None)
    assert step == -2


def test_workspace_sizes_follow_table2():
    # staged forward keeps the rank's strip: B*Z*(L/N)*L scores (Table 2, Ring-QK^T row)
    d = desc(B=2, Z=3, L=512, N=4, flags=rsa.MODE_STAGED)
    strip = 2 * 3 * 128 * 512
    assert rsa.workspace_bytes(d, False) >= strip * 4 + strip * 2
    assert rsa.workspace_bytes(desc(), False) == 0            # fused forward: no strip
    assert rsa.workspace_bytes(desc(), True) == 2 * (1 * 2 * 256 * 4)   # the two row terms, fp32
    assert rsa.workspace_bytes(desc(N=3), True) == 0          # invalid descriptor
    # one rank's share of a long sequence: the key walk is split, fp32 partial results per split
    d = desc(B=1, Z=2, L=4096, N=4, rank_begin=3, rank_end=4)
    rows, splits = 1 * 2 * 1024, 2          # 32 stages of 128 keys: at most 2 splits of 16
    assert rsa.workspace_bytes(d, False) == splits * rows * (64 + 2) * 4
    assert rsa.workspace_bytes(d, True) == 2 * rows * 4 + splits * rows * 64 * 4
    for s in range(-5, 1):
        assert rsa.strerror(s)


def test_split_plan_of_the_key_walk():
    """Host logic behind rsa_workspace_bytes in fused mode: how many work-groups share a row
    tile's walk over the keys (forward: (A + 2) floats per row and split; dQ: A floats)."""
    def splits(d):
        rows = d.B * d.Z * (d.rank_end - d.rank_begin) * (d.L // d.N)
        f = rsa.workspace_bytes(d, False) // (rows * (d.A + 2) * 4)
        b = (rsa.workspace_bytes(d, True) - 2 * rows * 4) // (rows * d.A * 4)
        return max(f, 1), max(b, 1)
    big = dict(B=1, Z=12, L=65536, N=16, causal=1)
    assert splits(desc(B=8, Z=16, L=2048, N=8, rank_end=8)) == (1, 1)          # whole ring: rows fill the chip
    assert splits(desc(B=8, Z=16, L=2048, N=8, rank_begin=3, rank_end=4)) == (1, 1)   # 16 stages: too short to split
    assert splits(desc(rank_begin=15, rank_end=16, **big)) == (8, 4)          # 192 x 8 and 384 x 4 = 3 full rounds
    assert splits(desc(rank_begin=0, rank_end=1, **big)) == (2, 2)            # first rank under the mask sees 32 stages: 2 x 16
    assert splits(desc(rank_begin=0, rank_end=1, flags=rsa.OWN_ZIGZAG, **big)) == (16, 8)   # half the tiles are long
    assert splits(desc(B=2, Z=16, L=16384, N=32, rank_begin=9, rank_end=10)) == (8, 4)     # 64 x 8 (256-row tiles) and 128 x 4: one round
    assert splits(desc(B=4, Z=8, A=128, L=8192, N=8, rank_begin=2, rank_end=3)) == (2, 2)


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(rsa, "_lib", None)
    monkeypatch.setattr(rsa, "LIB_PATH", "/nonexistent/librsa_hip.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        rsa.lib()
