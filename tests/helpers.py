"""Shared test helpers: device upload, oracle calls on head subsets, error measures."""
import numpy as np
import torch

import oracle
from bf16_model import ideal_bf16_pipeline, strip_bf16_pipeline
from paper_2105_13120_amd import inputs, rsa

# Tolerances of the comparison with the fp64 oracle.
#  fp32 path: max abs error <= 1e-4.  LSE (fp32 on both paths): 1e-4 absolute.
#  bf16 path.  The stated bar is "max abs err <= 2e-2 relative to the output RMS".  Read as a bound
#  on the largest error of a tensor it cannot be met by anything that stores bf16: O, dQ, dK, dV are
#  heavy-tailed on these inputs (largest element 10 to 12 times the RMS) and the store rounds
#  relative to the element (unit roundoff 2^-8), so the EXACT result rounded to bf16 is already
#  2.6e-2 of the RMS off at its largest element (bert_base and bert_large, all heads; the CPU test
#  tests/test_tolerance_model.py shows it).  What is asserted instead, per output tensor x with
#  oracle value r:
#   (1) every element:  |x_ia - r_ia| <= 2e-2 rms(r) + 2^-7 max_a |r_ia|   (+ dq_extra for dQ)
#       -- the stated bar plus two unit roundoffs of the row's largest element: one for the store,
#       one for the noise that the bf16 rounding of the matrix-core operands P and dS of that row
#       leaves (it scales with the row).  The ideal bf16 pipeline of tests/bf16_model.py reaches
#       0.33 to 0.89 of this bound on the shapes of tests/test_tolerance_model.py.
#   (2) the whole tensor:  rms(x - r) <= 3e-3 rms(r)   (the ideal pipeline: 2.0e-3 to 2.5e-3).
#   (3) against the ideal pipeline on the same inputs (wherever a test computes it: every dense
#       comparison): rms(x - r) <= 1.15 rms(ideal - r), the 99.9th percentile of |x - r| <= 1.25
#       times that of |ideal - r|, and max|x - r| <= 2.5 max|ideal - r|.
#       The ideal pipeline is exact arithmetic with only the roundings a bf16 matrix-core path
#       cannot avoid, which are also exactly the roundings the fused kernels make; (3) is what
#       rejects avoidable error: a second rounding of a scaled operand (the planted mistake of
#       tests/test_tolerance_model.py) passes (1) and fails (3) at 1.27 of the ideal RMS error.
#       The largest error of a tensor is one draw from the few elements of its top binade (their
#       store alone errs by up to half an ulp, and the P-rounding noise under it, a quarter ulp,
#       decides which way they round): two correct pipelines differ by a factor of up to about 2
#       there (the forward keeps P relative to a running maximum, the model to the true one, so
#       their rounding draws differ), hence the loose factor on the maximum and the tight ones on
#       the tail percentile and the RMS.  dK and dV, whose P both sides form from the same LSE,
#       agree with the model to the last digit of the largest error.
#  dQ carries one more term in (1).  Every bf16 backward forms D_i = sum_a dO_ia O_ia from the
#  *stored* O, whose rounding leaves an error delta_i in D_i with standard deviation
#  2^-9 / sqrt(3) * sqrt(sum_a dO_ia^2 O_ia^2).  It enters dS_ij = P_ij (dP_ij - D_i) for every key
#  of the row with the same sign, so dQ_i = s sum_j dS_ij K_j moves by s delta_i (sum_j P_ij K_j):
#  the row's attention-weighted mean key.  For rows that see many keys O_i is small and the term
#  vanishes; on the first rows of a causal mask (one or two keys, O_i of the size of a value vector)
#  it is the largest error in the tensor, so the dQ bound is widened by four standard deviations of
#  that term, computed from the oracle's own O and P (dq_extra below; the ideal pipeline reaches
#  0.8 to 0.9 of the widened bound on such rows).  The same delta_i reaches dK_j = s sum_i dS_ij Q_i
#  of the keys those rows see: the first keys of a causal sequence, or any key when a caller's
#  scale spreads the scores so wide that rows sit on few keys (dk_extra, same four standard
#  deviations; the ideal pipeline is 1.5 of the plain bound on a seeded case with scale 0.27).
F32_ATOL = 1e-4
BF16_REL_RMS = 2e-2
BF16_RTOL = 2.0 ** -7
BF16_REL_RMS_MEAN = 3e-3
IDEAL_MAX_RATIO = 2.5
IDEAL_P999_RATIO = 1.25
IDEAL_RMS_RATIO = 1.15
LSE_ATOL = 1e-4


def torch_dtype(name):
    return torch.bfloat16 if name == "bf16" else torch.float32


def upload(x, dtype):
    """float32 numpy (already rounded to dtype) -> device tensor of that dtype."""
    return torch.from_numpy(np.ascontiguousarray(x)).to(torch_dtype(dtype)).cuda().contiguous()


def download(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def heads_view(x, heads):
    """(B,Z,rows,A) -> (1,len(heads),rows,A) float64 for the listed flat head indices."""
    B, Z, rows, A = x.shape
    return np.ascontiguousarray(x.reshape(B * Z, rows, A)[heads][None].astype(np.float64))


def rel_rms_err(got, ref):
    rms = float(np.sqrt(np.mean(np.square(ref))))
    return float(np.abs(got - ref).max()) / max(rms, 1e-30)


def dq_extra(Q, K, V, dO, O_ref, q0, causal, scale=None):
    """The allowance for the rounding of the stored O inside D (see the comment on top):
    4 * 2^-9 / sqrt(3) * sqrt(sum_a dO^2 O^2) * s * |sum_j P_ij K_j|, per element of dQ."""
    s = 1.0 / np.sqrt(Q.shape[-1]) if scale is None else scale
    PK, _ = oracle.forward(Q, K, K, q0=q0, causal=causal, scale=scale)   # attention-weighted mean key
    sigma = 2.0 ** -9 / np.sqrt(3.0) * np.sqrt(np.sum(np.square(dO * O_ref), axis=-1, keepdims=True))
    return 4.0 * sigma * s * np.abs(PK)


def dk_extra(Q, K, V, dO, O_ref, q0, causal=True, scale=None, first=256):
    """The same rounding of the stored O inside D, seen from the keys: row i's error delta_i moves
    dK_j = s sum_i dS_ij Q_i by s delta_i P_ij Q_i for every key j the row sees.  It matters where a
    row's softmax is concentrated on few keys (O_i is then of the size of a value vector and P_ij
    of order one): on the first tokens of a causal sequence, whatever the inputs, and anywhere when
    the scores are spread wide (a caller's scale well above 1/sqrt(A)).  Returns 4 standard
    deviations, 4 s sqrt(sum_i sigma_i^2 P_ij^2 Q_ia^2), as (B, Z, keys, A): under the causal mask
    over the rows of tokens below `first` and for keys [0, first) (zeros if there is no such row),
    otherwise over all rows and keys."""
    s = 1.0 / np.sqrt(Q.shape[-1]) if scale is None else scale
    B, Z, n, A = Q.shape
    if causal:
        m = int(min(n, max(0, first - q0)))
        nk = min(first, K.shape[2])          # tokens below `first` see no later key
    else:
        m, nk = n, K.shape[2]
    out = np.zeros((B, Z, first if causal else nk, A))
    if m == 0:
        return out
    for b in range(B):
        for z in range(Z):
            sl = (slice(b, b + 1), slice(z, z + 1))
            Qs, dOs, Os = Q[sl][:, :, :m], dO[sl][:, :, :m], O_ref[sl][:, :, :m]
            P = oracle.forward(np.ascontiguousarray(Qs), np.ascontiguousarray(K[sl][:, :, :nk]),
                               np.ascontiguousarray(V[sl][:, :, :nk]), q0=q0, causal=causal, scale=scale,
                               want_scores=True)[3][0, 0]                            # (m, nk)
            var = (2.0 ** -9) ** 2 / 3.0 * np.sum(np.square(dOs * Os), axis=-1)[0, 0]   # sigma_i^2, (m,)
            out[b, z, :nk] = 4.0 * s * np.sqrt((P ** 2 * var[:, None]).T @ (Qs[0, 0] ** 2))
    return out


class Err(float):
    """max abs err / rms (bf16) or max abs err (f32), with the other figures as attributes:
    rms_rel = rms(err) / rms; vs_ideal_max, vs_ideal_p999, vs_ideal_rms = the ratios of criterion (3)
    or None."""
    rms_rel = None
    vs_ideal_max = None
    vs_ideal_p999 = None
    vs_ideal_rms = None

    def describe(self):
        t = f"{float(self):.2e}"
        if self.rms_rel is not None:
            t += f" (rms {self.rms_rel:.2e}"
            if self.vs_ideal_max is not None:
                t += (f"; x{self.vs_ideal_max:.2f} max, x{self.vs_ideal_p999:.2f} p99.9, "
                      f"x{self.vs_ideal_rms:.2f} rms of ideal")
            t += ")"
        return t


def check(name, got, ref, dtype, extra=None, ideal=None, both_rounded=False, strip=False):
    """Assert the tolerance for one output tensor; returns an Err.  extra: per-element addition
    to the bf16 bound; ideal: the same tensor from the ideal bf16 pipeline (criterion (3));
    both_rounded: ref is itself a bf16 result of the HIP path (two layouts or ring sizes compared
    with each other), so the difference carries both sides' noise: bounds times sqrt(2).
    strip: a result of the two-pass layout, whose bf16 probability strip rounds P once more on the
    way into dS (RMS error of dQ, dK sqrt(1.5) times the ideal pipeline's): criterion (2) times 1.25."""
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    diff = np.abs(got - ref)
    if dtype == "f32":
        err = float(diff.max())
        assert err <= F32_ATOL, f"{name}: max abs err {err:.3e} > {F32_ATOL}"
        return Err(err)
    rms = max(float(np.sqrt(np.mean(np.square(ref)))), 1e-30)
    widen = np.sqrt(2.0) if both_rounded else 1.0
    bound = widen * (BF16_REL_RMS * rms + BF16_RTOL * np.abs(ref).max(axis=-1, keepdims=True))
    if extra is not None:
        bound = bound + extra
    worst = float((diff / bound).max())
    assert worst <= 1.0, (f"{name}: error is {worst:.3f} of the bound "
                          f"(max abs err / rms = {diff.max() / rms:.3e})")
    mean = float(np.sqrt(np.mean(np.square(diff))))
    rms_bar = widen * (1.25 if strip else 1.0) * BF16_REL_RMS_MEAN
    assert mean <= rms_bar * rms, f"{name}: rms err / rms {mean / rms:.3e} > {rms_bar:.2e}"
    e = Err(float(diff.max()) / rms)
    e.rms_rel = mean / rms
    if ideal is not None:
        di = np.abs(ideal - ref)
        e.vs_ideal_max = float(diff.max()) / max(float(di.max()), 1e-30)
        e.vs_ideal_rms = mean / max(float(np.sqrt(np.mean(np.square(di)))), 1e-30)
        e.vs_ideal_p999 = float(np.quantile(diff, 0.999)) / max(float(np.quantile(di, 0.999)), 1e-30)
        assert e.vs_ideal_p999 <= IDEAL_P999_RATIO, (f"{name}: the 99.9th percentile of the error is "
                                                    f"{e.vs_ideal_p999:.2f} times the ideal bf16 pipeline's")
        assert e.vs_ideal_max <= IDEAL_MAX_RATIO, (f"{name}: max err is {e.vs_ideal_max:.2f} times the ideal "
                                                   f"bf16 pipeline's ({diff.max() / rms:.3e} of the rms)")
        assert e.vs_ideal_rms <= IDEAL_RMS_RATIO, (f"{name}: rms err is {e.vs_ideal_rms:.2f} times the ideal "
                                                   f"bf16 pipeline's ({mean / rms:.3e} of the rms)")
    return e


def gpu_forward_backward(cfg, x, mode=rsa.MODE_FUSED, backward=True, interleaved=False):
    """Run the HIP path on cfg's inputs x (dict of numpy float32).  interleaved: every tensor lives
    head-interleaved, (B, rows, Z, A) with a padded row, and reaches the library as a strided
    (B, Z, rows, A) view (fused mode); the outputs come back contiguous."""
    def place(t):
        if not interleaved:
            return t
        B, Z, rows, A = t.shape
        buf = torch.full((B, rows, Z, A + 8), float("nan"), dtype=t.dtype, device=t.device)
        v = buf[..., :A].permute(0, 2, 1, 3)
        v.copy_(t)
        return v
    Q, K, V = (place(upload(x[k], cfg.dtype)) for k in ("Q", "K", "V"))
    rb, re = cfg.ranks
    O = place(torch.empty(Q.shape, dtype=Q.dtype, device="cuda"))
    desc = rsa.make_desc(K, cfg.N, causal=cfg.causal, rank_begin=rb, rank_end=re, mode=mode,
                         zigzag=cfg.zigzag, scale=cfg.att_scale, Q=Q, O=O)
    O, LSE = rsa.forward(desc, Q, K, V, O=O)
    out = {"O": O, "LSE": LSE}
    if backward:
        dO = place(upload(x["dO"], cfg.dtype))
        assert dO.stride() == O.stride()
        dQ, dK, dV = rsa.backward(desc, dO, Q, K, V, O, LSE, dQ=place(torch.empty(Q.shape, dtype=Q.dtype, device="cuda")),
                                  dK=place(torch.empty(K.shape, dtype=K.dtype, device="cuda")),
                                  dV=place(torch.empty(K.shape, dtype=K.dtype, device="cuda")))
        out.update(dQ=dQ, dK=dK, dV=dV)
    torch.cuda.synchronize()
    return {k: v.contiguous() for k, v in out.items()}


def att_scale(cfg):
    """The softmax scale as the oracle takes it (None: 1/sqrt(A))."""
    return cfg.att_scale if cfg.att_scale > 0 else None


def row_tokens(cfg):
    """Global token index of every local query row."""
    return np.concatenate([np.arange(t0, t0 + n) for _, t0, n in cfg.segments()])


def oracle_on_segments(cfg, Qh, Kh, Vh, dOh=None):
    """The oracle on cfg's local query rows: one call per run of consecutive tokens
    (one run unless the ownership is zig-zag); O, LSE, dQ are put back in local row
    order and the partial dK, dV of the runs are added."""
    O = np.empty_like(Qh)
    LSE = np.empty(Qh.shape[:3])
    dQ = np.empty_like(Qh) if dOh is not None else None
    extra = np.empty_like(Qh) if dOh is not None else None
    dK = dV = None
    dk_var = None     # variance-like sum of the runs' dk_extra terms (independent rows)
    sc = att_scale(cfg)
    for r0, t0, n in cfg.segments():
        Qs = np.ascontiguousarray(Qh[:, :, r0:r0 + n])
        O[:, :, r0:r0 + n], LSE[:, :, r0:r0 + n] = oracle.forward(Qs, Kh, Vh, q0=t0, causal=cfg.causal, scale=sc)
        if dOh is not None:
            dOs = np.ascontiguousarray(dOh[:, :, r0:r0 + n])
            g = oracle.backward(Qs, Kh, Vh, dOs, q0=t0, causal=cfg.causal, scale=sc)
            dQ[:, :, r0:r0 + n] = g[0]
            dK = g[1] if dK is None else dK + g[1]
            dV = g[2] if dV is None else dV + g[2]
            extra[:, :, r0:r0 + n] = dq_extra(Qs, Kh, Vh, dOs, O[:, :, r0:r0 + n], t0, cfg.causal, scale=sc)
            if cfg.causal or cfg.att_scale > 0:     # where a row's softmax can sit on few keys
                x_ = dk_extra(Qs, Kh, Vh, dOs, O[:, :, r0:r0 + n], t0, causal=cfg.causal, scale=sc) ** 2
                dk_var = x_ if dk_var is None else dk_var + x_
    dk_x = None
    if dk_var is not None:
        dk_x = np.zeros_like(Kh)
        w = min(dk_var.shape[2], Kh.shape[2])
        dk_x[:, :, :w] = np.sqrt(dk_var[:, :, :w])
    return O, LSE, dQ, dK, dV, extra, dk_x


def compare_heads(cfg, x, out, heads, backward=True, ideal=True, ideal_heads=16, mode=rsa.MODE_FUSED):
    """Full comparison with the oracle on the listed flat head indices.  ideal: also hold the bf16
    outputs to the stated multiples of the error of the CPU model of their pipeline (criterion (3)
    on top), on the first `ideal_heads` of the listed heads: the ideal bf16 pipeline with P relative
    to a running maximum for the fused kernels, the bf16-strip pipeline for the two-pass layout."""
    Qh, Kh, Vh = (heads_view(x[k], heads) for k in ("Q", "K", "V"))
    dOh = heads_view(x["dO"], heads) if backward else None
    O_ref, LSE_ref, dQ_ref, dK_ref, dV_ref, dq_x, dk_x = oracle_on_segments(cfg, Qh, Kh, Vh, dOh)
    extras = dict(dQ=dq_x, dK=dk_x)
    got = {k: heads_view(download(out[k]), heads) for k in (("O", "dQ", "dK", "dV") if backward else ("O",))}
    refs = dict(O=O_ref, dQ=dQ_ref, dK=dK_ref, dV=dV_ref)
    errs = {}
    for name in got:
        errs[name] = check(name, got[name], refs[name], cfg.dtype, strip=mode == rsa.MODE_STAGED,
                           extra=extras.get(name) if cfg.dtype == "bf16" else None)
    lse = download(out["LSE"]).reshape(-1, cfg.Lq)[heads][None]
    err = float(np.abs(lse - LSE_ref).max())
    assert err <= LSE_ATOL, f"LSE: max abs err {err:.3e}"
    errs["LSE"] = Err(err)
    if ideal and cfg.dtype == "bf16":
        n = min(ideal_heads, len(heads))
        cut = lambda a: None if a is None else a[:, :n]
        if mode == rsa.MODE_STAGED:
            m = strip_bf16_pipeline(cut(Qh), cut(Kh), cut(Vh), cut(dOh), scale=att_scale(cfg),
                                    qtok=row_tokens(cfg), causal=cfg.causal)
        else:
            m = ideal_bf16_pipeline(cut(Qh), cut(Kh), cut(Vh), cut(dOh), scale=att_scale(cfg),
                                    qtok=row_tokens(cfg), causal=cfg.causal, reference="running_max")
        model = dict(O=m[0])
        if backward:
            model.update(dQ=m[2], dK=m[3], dV=m[4])
        for name in got:
            errs[name] = check(name, cut(got[name]), cut(refs[name]), cfg.dtype, ideal=model[name],
                               extra=cut(extras.get(name)), strip=mode == rsa.MODE_STAGED)
    return errs


def describe(errs):
    return ", ".join(f"{k} {v.describe()}" for k, v in errs.items())
