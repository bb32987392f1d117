"""ctypes binding of the fp64 C oracle (rsa_oracle.c).  Test infrastructure only.

The arithmetic lives in the C file, which writes out Eq. 1 of the paper
(softmax(Q K^T / sqrt(d_k)) V) and its analytic derivative row by row; this
module only marshals numpy float64 arrays.  Nothing here is shared with, or
imported by, the HIP path.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rsa_oracle.c")
_LIB = os.path.join(_HERE, "librsa_oracle.so")
_lib = None


class _Problem(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int64),
        ("Z", ctypes.c_int64),
        ("L", ctypes.c_int64),
        ("A", ctypes.c_int64),
        ("Lq", ctypes.c_int64),
        ("q0", ctypes.c_int64),
        ("causal", ctypes.c_int32),
        ("scale", ctypes.c_double),
    ]


def build(force=False):
    """Compile rsa_oracle.c with gcc (generic x86-64, OpenMP)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(
        os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "rsa_oracle.h"))
    )
    if force or stale:
        subprocess.check_call(
            ["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall",
             "-Wextra", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.rsa_oracle_forward.restype = ctypes.c_int
        lib.rsa_oracle_forward.argtypes = [ctypes.POINTER(_Problem)] + [dp] * 7
        lib.rsa_oracle_backward.restype = ctypes.c_int
        lib.rsa_oracle_backward.argtypes = (
            [ctypes.POINTER(_Problem)] + [dp] * 7
            + [ctypes.POINTER(ctypes.c_int64), ctypes.c_int64, dp, dp]
        )
        lib.rsa_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads():
    """OpenMP threads the oracle will use."""
    return int(_load().rsa_oracle_threads())


def _f64(x, shape, name):
    a = np.ascontiguousarray(x, dtype=np.float64)
    if a.shape != shape:
        raise ValueError(f"{name}: expected shape {shape}, got {a.shape}")
    return a


def _ptr(a):
    if a is None:
        return None
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _problem(Q, K, q0, causal, scale):
    if K.ndim != 4 or Q.ndim != 4:
        raise ValueError("Q, K, V must be (B, Z, rows, A)")
    B, Z, L, A = K.shape
    Lq = Q.shape[2]
    if scale is None:
        scale = 1.0 / np.sqrt(float(A))
    return _Problem(B, Z, L, A, Lq, int(q0), int(bool(causal)), float(scale))


def forward(Q, K, V, q0=0, causal=False, scale=None, want_scores=False):
    """Steps 1-3 of the oracle.

    Q: (B,Z,Lq,A) query rows [q0, q0+Lq) of the sequence; K, V: (B,Z,L,A).
    Returns O (B,Z,Lq,A) and LSE (B,Z,Lq); with want_scores also the scaled
    scores S and the probabilities P, both (B,Z,Lq,L).
    """
    K = np.ascontiguousarray(K, dtype=np.float64)
    Q = np.ascontiguousarray(Q, dtype=np.float64)
    p = _problem(Q, K, q0, causal, scale)
    Q = _f64(Q, (p.B, p.Z, p.Lq, p.A), "Q")
    V = _f64(V, K.shape, "V")
    O = np.empty_like(Q)
    LSE = np.empty((p.B, p.Z, p.Lq), dtype=np.float64)
    S = P = None
    if want_scores:
        S = np.empty((p.B, p.Z, p.Lq, p.L), dtype=np.float64)
        P = np.empty_like(S)
    rc = _load().rsa_oracle_forward(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V),
                                    _ptr(O), _ptr(LSE), _ptr(S), _ptr(P))
    if rc != 0:
        raise ValueError("rsa_oracle_forward rejected its arguments")
    if want_scores:
        return O, LSE, S, P
    return O, LSE


def backward(Q, K, V, dO, q0=0, causal=False, scale=None, cols=None,
             want_scores=False):
    """Steps 4-9 of the oracle.

    Returns dQ (B,Z,Lq,A), dK, dV.  dK and dV cover all L keys, or only the
    key indices listed in cols (then (B,Z,len(cols),A)).  With want_scores
    also dP and dS, (B,Z,Lq,L).
    """
    K = np.ascontiguousarray(K, dtype=np.float64)
    Q = np.ascontiguousarray(Q, dtype=np.float64)
    p = _problem(Q, K, q0, causal, scale)
    Q = _f64(Q, (p.B, p.Z, p.Lq, p.A), "Q")
    V = _f64(V, K.shape, "V")
    dO = _f64(dO, Q.shape, "dO")
    dQ = np.empty_like(Q)
    if cols is None:
        cols_arr, cols_ptr, ncols = None, None, 0
        nk = p.L
    else:
        cols_arr = np.ascontiguousarray(cols, dtype=np.int64)
        cols_ptr = cols_arr.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
        ncols = nk = int(cols_arr.size)
    dK = np.empty((p.B, p.Z, nk, p.A), dtype=np.float64)
    dV = np.empty_like(dK)
    dP = dS = None
    if want_scores:
        dP = np.empty((p.B, p.Z, p.Lq, p.L), dtype=np.float64)
        dS = np.empty_like(dP)
    rc = _load().rsa_oracle_backward(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V),
                                     _ptr(dO), _ptr(dQ), _ptr(dK), _ptr(dV),
                                     cols_ptr, ncols, _ptr(dP), _ptr(dS))
    if rc != 0:
        raise ValueError("rsa_oracle_backward rejected its arguments")
    if want_scores:
        return dQ, dK, dV, dP, dS
    return dQ, dK, dV
