"""ctypes binding of the RSA C ABI (include/rsa.h): argument marshalling only.

Every step of the path runs in the HIP library.  PyTorch supplies device
memory and the current stream; nothing here computes.  If the library has not
been built the calls raise -- there is no fallback.
"""
import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "librsa_hip.so")

RSA_F32, RSA_BF16 = 0, 1
MODE_FUSED, MODE_STAGED = 0, 1
OWN_ZIGZAG = 2   # flag bit: rank n owns half-chunks n and 2N-1-n
DETERMINISTIC = 4   # flag bit: dQ from a kernel of its own (fixed summation order, no atomics)
STATIC_SCRATCH_BYTES = 32 << 20

EXPORTS = (
    "rsa_version", "rsa_strerror", "rsa_workspace_bytes", "rsa_forward", "rsa_backward",
    "rsa_qk_step", "rsa_row_softmax", "rsa_av_step", "rsa_bwd_rowdot", "rsa_dv_step",
    "rsa_dp_step", "rsa_softmax_bwd", "rsa_dq_step", "rsa_dk_step", "rsa_store",
    "rsa_bwd_preprocess", "rsa_bwd_dkdv", "rsa_bwd_dq", "rsa_backward_static",
    "rsa_proj_workspace_bytes", "rsa_qkv_proj", "rsa_out_proj", "rsa_out_proj_bwd", "rsa_qkv_proj_bwd",
    "rsa_linformer_workspace_bytes", "rsa_linformer_project", "rsa_linformer_forward",
    "rsa_linformer_backward", "rsa_linformer_project_bwd",
)


class RSADesc(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("Z", ctypes.c_int32), ("A", ctypes.c_int32),
        ("L", ctypes.c_int64), ("N", ctypes.c_int32),
        ("rank_begin", ctypes.c_int32), ("rank_end", ctypes.c_int32),
        ("causal", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("scale", ctypes.c_float), ("flags", ctypes.c_uint32),
        ("q_stride", ctypes.c_int64 * 3), ("kv_stride", ctypes.c_int64 * 3),
        ("o_stride", ctypes.c_int64 * 3),
    ]


class RSAError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"rsa status {status}: {message}")
        self.status = status


_lib = None


def lib():
    """The loaded HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                "(python -m paper_2105_13120_amd.build); there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        dp = ctypes.POINTER(RSADesc)
        L.rsa_version.restype = i
        L.rsa_strerror.restype = ctypes.c_char_p
        L.rsa_strerror.argtypes = [i]
        L.rsa_workspace_bytes.restype = sz
        L.rsa_workspace_bytes.argtypes = [dp, i]
        L.rsa_forward.argtypes = [dp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.rsa_backward.argtypes = [dp] + [vp] * 10 + [sz, vp]
        L.rsa_qk_step.argtypes = [dp, i, i, vp, vp, vp, vp]
        L.rsa_row_softmax.argtypes = [dp, i, vp, vp, vp, vp]
        L.rsa_av_step.argtypes = [dp, i, i, vp, vp, vp, i, vp]
        L.rsa_bwd_rowdot.argtypes = [dp, i, vp, vp, vp, vp]
        L.rsa_dv_step.argtypes = [dp, i, i, vp, vp, vp, i, vp]
        L.rsa_dp_step.argtypes = [dp, i, i, vp, vp, vp, vp]
        L.rsa_softmax_bwd.argtypes = [dp, i, vp, vp, vp, vp, vp]
        L.rsa_dq_step.argtypes = [dp, i, i, vp, vp, vp, i, vp]
        L.rsa_dk_step.argtypes = [dp, i, i, vp, vp, vp, i, vp]
        L.rsa_store.argtypes = [dp, vp, vp, sz, vp]
        L.rsa_bwd_preprocess.argtypes = [dp, vp, vp, vp, vp, sz, vp]
        L.rsa_bwd_dkdv.argtypes = [dp] + [vp] * 5 + [sz] + [vp] * 3
        L.rsa_bwd_dq.argtypes = [dp] + [vp] * 5 + [sz] + [vp] * 2
        L.rsa_backward_static.argtypes = [dp] + [vp] * 10
        L.rsa_proj_workspace_bytes.argtypes = [dp, i]
        L.rsa_qkv_proj.argtypes = [dp, i] + [vp] * 6
        L.rsa_out_proj.argtypes = [dp, i] + [vp] * 4
        L.rsa_out_proj_bwd.argtypes = [dp, i] + [vp] * 6 + [sz, vp]
        L.rsa_qkv_proj_bwd.argtypes = [dp, i] + [vp] * 8 + [sz, vp]
        for name in EXPORTS[3:]:
            getattr(L, name).restype = i
        L.rsa_proj_workspace_bytes.restype = sz
        L.rsa_linformer_workspace_bytes.argtypes = [dp, i]
        L.rsa_linformer_workspace_bytes.restype = sz
        L.rsa_linformer_project.argtypes = [dp, i, vp, vp, vp, vp, sz, vp]
        L.rsa_linformer_forward.argtypes = [dp, i] + [vp] * 6
        L.rsa_linformer_backward.argtypes = [dp, i] + [vp] * 10 + [sz, vp]
        L.rsa_linformer_project_bwd.argtypes = [dp, i] + [vp] * 6
        _lib = L
    return _lib


def strerror(status):
    return lib().rsa_strerror(int(status)).decode()


def _check(status):
    if status != 0:
        raise RSAError(status, strerror(status))


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _p(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _dtype_code(t):
    if t.dtype == torch.bfloat16:
        return RSA_BF16
    if t.dtype == torch.float32:
        return RSA_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _strides(t):
    """(batch, head, row) element strides of a (B, Z, rows, A) tensor whose last index is contiguous."""
    assert t.dim() == 4 and (t.shape[3] == 1 or t.stride(3) == 1), "the last index must be contiguous"
    return (ctypes.c_int64 * 3)(t.stride(0), t.stride(1), t.stride(2))


def make_desc(K, N, causal=False, rank_begin=0, rank_end=None, mode=MODE_FUSED, scale=0.0,
              zigzag=False, deterministic=False, Q=None, O=None):
    """Descriptor for K of shape (B, Z, L, A).  zigzag: rank n owns half-chunks n and 2N-1-n.
    deterministic: RSA_DETERMINISTIC.  K's strides are taken when it is not contiguous (V, dK, dV
    must then share them); Q and O, when given, supply the strides of Q/dQ and O/dO likewise."""
    B, Z, L, A = K.shape
    d = RSADesc(B, Z, A, L, N, rank_begin, N if rank_end is None else rank_end,
                int(bool(causal)), _dtype_code(K), float(scale),
                int(mode) | (OWN_ZIGZAG if zigzag else 0) | (DETERMINISTIC if deterministic else 0))
    if not K.is_contiguous():
        d.kv_stride = _strides(K)
    if Q is not None and not Q.is_contiguous():
        d.q_stride = _strides(Q)
    if O is not None and not O.is_contiguous():
        d.o_stride = _strides(O)
    return d


def workspace_bytes(desc, backward):
    return int(lib().rsa_workspace_bytes(ctypes.byref(desc), 1 if backward else 0))


def _workspace(desc, backward, device):
    n = workspace_bytes(desc, backward)
    ws = torch.empty(max(n, 16), dtype=torch.uint8, device=device)
    return ws, n


def forward(desc, Q, K, V, O=None, LSE=None, ws=None):
    """rsa_forward.  Q: (B,Z,Lq,A); K, V: (B,Z,L,A).  Returns (O, LSE)."""
    for t in (Q, K, V):
        assert t.is_cuda and t.stride(-1) == 1   # other strides travel in the descriptor
    if O is None:
        O = torch.empty_like(Q)
    if LSE is None:
        LSE = torch.empty(Q.shape[:3], dtype=torch.float32, device=Q.device)
    if ws is None:
        ws, n = _workspace(desc, False, Q.device)
    else:
        n = ws.numel()
    _check(lib().rsa_forward(ctypes.byref(desc), _p(Q), _p(K), _p(V), _p(O), _p(LSE),
                             _p(ws), n, _stream()))
    return O, LSE


def backward(desc, dO, Q, K, V, O, LSE, dQ=None, dK=None, dV=None, ws=None):
    """rsa_backward.  Returns (dQ, dK, dV)."""
    for t in (dO, Q, K, V, O, LSE):
        assert t.is_cuda and t.stride(-1) == 1
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    if ws is None:
        ws, n = _workspace(desc, True, Q.device)
    else:
        n = ws.numel()
    _check(lib().rsa_backward(ctypes.byref(desc), _p(dO), _p(Q), _p(K), _p(V), _p(O), _p(LSE),
                              _p(dQ), _p(dK), _p(dV), _p(ws), n, _stream()))
    return dQ, dK, dV


# ---- step-level calls (one ring step of one simulated rank) ----

def qk_step(desc, n, j, Q, K, S):
    _check(lib().rsa_qk_step(ctypes.byref(desc), n, j, _p(Q), _p(K), _p(S), _stream()))


def row_softmax(desc, n, S, P, LSE):
    _check(lib().rsa_row_softmax(ctypes.byref(desc), n, _p(S), _p(P), _p(LSE), _stream()))


def av_step(desc, n, j, P, V, Oacc, accumulate):
    _check(lib().rsa_av_step(ctypes.byref(desc), n, j, _p(P), _p(V), _p(Oacc), int(accumulate), _stream()))


def bwd_rowdot(desc, n, dO, O, D):
    _check(lib().rsa_bwd_rowdot(ctypes.byref(desc), n, _p(dO), _p(O), _p(D), _stream()))


def dv_step(desc, n, j, P, dO, dVacc, accumulate):
    _check(lib().rsa_dv_step(ctypes.byref(desc), n, j, _p(P), _p(dO), _p(dVacc), int(accumulate), _stream()))


def dp_step(desc, n, j, dO, V, dP):
    _check(lib().rsa_dp_step(ctypes.byref(desc), n, j, _p(dO), _p(V), _p(dP), _stream()))


def softmax_bwd(desc, n, P, dP, D, dS):
    _check(lib().rsa_softmax_bwd(ctypes.byref(desc), n, _p(P), _p(dP), _p(D), _p(dS), _stream()))


def dq_step(desc, n, j, dS, K, dQacc, accumulate):
    _check(lib().rsa_dq_step(ctypes.byref(desc), n, j, _p(dS), _p(K), _p(dQacc), int(accumulate), _stream()))


def dk_step(desc, n, j, dS, Q, dKacc, accumulate):
    _check(lib().rsa_dk_step(ctypes.byref(desc), n, j, _p(dS), _p(Q), _p(dKacc), int(accumulate), _stream()))


def store(desc, src, dst):
    _check(lib().rsa_store(ctypes.byref(desc), _p(src), _p(dst), src.numel(), _stream()))


def bwd_preprocess(desc, dO, O, LSE, ws):
    _check(lib().rsa_bwd_preprocess(ctypes.byref(desc), _p(dO), _p(O), _p(LSE), _p(ws),
                                    ws.numel(), _stream()))


def bwd_dkdv(desc, dO, Q, K, V, ws, dK, dV):
    _check(lib().rsa_bwd_dkdv(ctypes.byref(desc), _p(dO), _p(Q), _p(K), _p(V), _p(ws), ws.numel(),
                              _p(dK), _p(dV), _stream()))


def bwd_dq(desc, dO, Q, K, V, ws, dQ):
    _check(lib().rsa_bwd_dq(ctypes.byref(desc), _p(dO), _p(Q), _p(K), _p(V), _p(ws), ws.numel(),
                            _p(dQ), _stream()))


def backward_static(desc, dO, Q, K, V, O, LSE, dQ, dK, dV):
    """rsa_backward_static: the workspace is the library's static device array; every buffer,
    outputs included, is the caller's, so nothing is allocated here either."""
    _check(lib().rsa_backward_static(ctypes.byref(desc), _p(dO), _p(Q), _p(K), _p(V), _p(O), _p(LSE),
                                     _p(dQ), _p(dK), _p(dV), _stream()))
    return dQ, dK, dV


# ---- the linear maps around RSA (Table 2, rows Q/K/V and Linear) ----
def proj_workspace_bytes(desc, H):
    return int(lib().rsa_proj_workspace_bytes(ctypes.byref(desc), int(H)))


def _proj_ws(desc, H, device):
    return torch.empty(max(proj_workspace_bytes(desc, H), 16), dtype=torch.uint8, device=device)


def _head_shape(desc, X):
    rows = (desc.rank_end - desc.rank_begin) * (desc.L // desc.N)
    return (desc.B, desc.Z, rows, desc.A)


def qkv_proj(desc, X, Wqkv, Q=None, K=None, V=None):
    """X (B, Lq, H), Wqkv (H, 3*Z*A) -> Q, K, V (B, Z, Lq, A)."""
    H = X.shape[-1]
    Q, K, V = (torch.empty(_head_shape(desc, X), dtype=X.dtype, device=X.device) if t is None else t
               for t in (Q, K, V))
    _check(lib().rsa_qkv_proj(ctypes.byref(desc), H, _p(X), _p(Wqkv), _p(Q), _p(K), _p(V), _stream()))
    return Q, K, V


def out_proj(desc, O, Wo, Y=None):
    """O (B, Z, Lq, A), Wo (Z*A, H) -> Y (B, Lq, H)."""
    H = Wo.shape[-1]
    if Y is None:
        Y = torch.empty((O.shape[0], O.shape[2], H), dtype=O.dtype, device=O.device)
    _check(lib().rsa_out_proj(ctypes.byref(desc), H, _p(O), _p(Wo), _p(Y), _stream()))
    return Y


def out_proj_bwd(desc, dY, O, Wo, dO=None, dWo=None, ws=None):
    H = Wo.shape[-1]
    dO = torch.empty_like(O) if dO is None else dO
    dWo = torch.empty(Wo.shape, dtype=torch.float32, device=Wo.device) if dWo is None else dWo
    ws = _proj_ws(desc, H, O.device) if ws is None else ws
    _check(lib().rsa_out_proj_bwd(ctypes.byref(desc), H, _p(dY), _p(O), _p(Wo), _p(dO), _p(dWo), _p(ws),
                                  ws.numel(), _stream()))
    return dO, dWo


def qkv_proj_bwd(desc, dQ, dK, dV, X, Wqkv, dX=None, dW=None, ws=None):
    H = X.shape[-1]
    dX = torch.empty_like(X) if dX is None else dX
    dW = torch.empty(Wqkv.shape, dtype=torch.float32, device=X.device) if dW is None else dW
    ws = _proj_ws(desc, H, X.device) if ws is None else ws
    _check(lib().rsa_qkv_proj_bwd(ctypes.byref(desc), H, _p(dQ), _p(dK), _p(dV), _p(X), _p(Wqkv), _p(dX),
                                  _p(dW), _p(ws), ws.numel(), _stream()))
    return dX, dW


# ---- Linformer variant (Table 3): keys and values projected along the sequence ----
def linformer_workspace_bytes(desc, Kp):
    return int(lib().rsa_linformer_workspace_bytes(ctypes.byref(desc), int(Kp)))


def _linf_ws(desc, Kp, device):
    return torch.empty(max(linformer_workspace_bytes(desc, Kp), 16), dtype=torch.uint8, device=device)


def linformer_project(desc, X, E, Xp=None, ws=None):
    """X (B, Z, L, A), E (L, Kp) -> Xp (B, Z, Kp, A), over the tokens of the descriptor's ranks."""
    Kp = E.shape[1]
    if Xp is None:
        Xp = torch.empty((X.shape[0], X.shape[1], Kp, X.shape[3]), dtype=X.dtype, device=X.device)
    ws = _linf_ws(desc, Kp, X.device) if ws is None else ws
    _check(lib().rsa_linformer_project(ctypes.byref(desc), Kp, _p(X), _p(E), _p(Xp), _p(ws), ws.numel(),
                                       _stream()))
    return Xp


def linformer_forward(desc, Q, Kp_, Vp_, O=None, LSE=None):
    O = torch.empty_like(Q) if O is None else O
    LSE = torch.empty(Q.shape[:3], dtype=torch.float32, device=Q.device) if LSE is None else LSE
    _check(lib().rsa_linformer_forward(ctypes.byref(desc), Kp_.shape[2], _p(Q), _p(Kp_), _p(Vp_), _p(O),
                                       _p(LSE), _stream()))
    return O, LSE


def linformer_backward(desc, dO, Q, Kp_, Vp_, O, LSE, dQ=None, dKp=None, dVp=None, ws=None):
    Kp = Kp_.shape[2]
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dKp = torch.empty_like(Kp_) if dKp is None else dKp
    dVp = torch.empty_like(Vp_) if dVp is None else dVp
    ws = _linf_ws(desc, Kp, Q.device) if ws is None else ws
    _check(lib().rsa_linformer_backward(ctypes.byref(desc), Kp, _p(dO), _p(Q), _p(Kp_), _p(Vp_), _p(O),
                                        _p(LSE), _p(dQ), _p(dKp), _p(dVp), _p(ws), ws.numel(), _stream()))
    return dQ, dKp, dVp


def linformer_project_bwd(desc, dXp, X, E, dX=None, dE=None):
    """dX (rows of the descriptor's ranks; a new tensor is zero elsewhere) and dE (fp32, same)."""
    dX = torch.zeros_like(X) if dX is None else dX
    dE = torch.zeros(E.shape, dtype=torch.float32, device=E.device) if dE is None else dE
    _check(lib().rsa_linformer_project_bwd(ctypes.byref(desc), E.shape[1], _p(dXp), _p(X), _p(E), _p(dX),
                                           _p(dE), _stream()))
    return dX, dE
