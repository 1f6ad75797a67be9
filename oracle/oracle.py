"""ctypes loader for the fp64 CPU oracle (oracle/entmax_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module,
and this module never imports the product package.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "entmax_oracle.c")
_LIB = os.path.join(_HERE, "libentmax_oracle.so")
_lib = None


class OracleParams(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32),
        ("H", ctypes.c_int32),
        ("Nq", ctypes.c_int32),
        ("Nk", ctypes.c_int32),
        ("D", ctypes.c_int32),
        ("causal", ctypes.c_int32),
        ("scale_layout", ctypes.c_int32),
        ("logn_mode", ctypes.c_int32),
        ("bias_mode", ctypes.c_int32),
        ("alpha", ctypes.c_double),
        ("delta", ctypes.c_double),
    ]


def build(force=False):
    """Compile the oracle with gcc (-O2, OpenMP) into oracle/libentmax_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double)) if a is not None else None


def _f64(a):
    return None if a is None else np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def num_threads():
    return int(_load().oracle_num_threads())


def entmax_row(s, alpha, force_generic=False):
    """Exact alpha-entmax of a 1-D score vector: returns (p, tau, support size)."""
    lib = _load()
    s = _f64(s)
    n = s.shape[0]
    p = np.empty(n, dtype=np.float64)
    tau = ctypes.c_double()
    sup = ctypes.c_int()
    lib.oracle_entmax_row(_dp(s), ctypes.c_int(n), ctypes.c_double(alpha), ctypes.c_int(int(force_generic)),
                          _dp(p), ctypes.byref(tau), ctypes.byref(sup))
    return p, tau.value, sup.value


def _params(Q, K, alpha, delta, causal, beta, logn_mode, bias_mode=0):
    B, H, Nq, D = Q.shape
    Nk = K.shape[2]
    if beta is None:
        layout = 0
    elif beta.ndim == 1:
        layout = 1
    else:
        layout = 2
    return OracleParams(B, H, Nq, Nk, D, int(causal), layout, int(logn_mode), int(bias_mode), float(alpha), float(delta))


def attn_fwd(Q, K, V, alpha, beta=None, gamma=None, delta=1.0, causal=True, logn_mode=0, want_p=False, slopes=None,
             bias_mode=0):
    """Exact entmax attention forward.  Q [B,H,Nq,D], K,V [B,H,Nk,D] (any float dtype, widened to fp64).
    slopes: optional ALiBi slopes [H] (0 = no positional bias for that head); bias_mode 0 puts the bias inside
    the scaled logit, 1 adds it after the scale.  Returns dict(O, tau, support[, P])."""
    lib = _load()
    Q, K, V, beta, gamma, slopes = _f64(Q), _f64(K), _f64(V), _f64(beta), _f64(gamma), _f64(slopes)
    prm = _params(Q, K, alpha, delta, causal, beta, logn_mode, bias_mode)
    B, H, Nq, D = Q.shape
    Nk = K.shape[2]
    O = np.empty((B, H, Nq, D), dtype=np.float64)
    tau = np.empty((B, H, Nq), dtype=np.float64)
    sup = np.empty((B, H, Nq), dtype=np.int32)
    P = np.empty((B, H, Nq, Nk), dtype=np.float64) if want_p else None
    lib.oracle_attn_fwd(ctypes.byref(prm), _dp(Q), _dp(K), _dp(V), _dp(beta), _dp(gamma), _dp(slopes), _dp(O), _dp(tau),
                        sup.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), _dp(P))
    out = {"O": O, "tau": tau, "support": sup}
    if want_p:
        out["P"] = P
    return out


def attn_bwd(Q, K, V, dO, alpha, beta=None, gamma=None, delta=1.0, causal=True, logn_mode=0, slopes=None, bias_mode=0):
    """Exact entmax attention backward.  Returns dict(dQ, dK, dV, dbeta, dgamma, dscale)."""
    lib = _load()
    Q, K, V, dO, beta, gamma, slopes = _f64(Q), _f64(K), _f64(V), _f64(dO), _f64(beta), _f64(gamma), _f64(slopes)
    prm = _params(Q, K, alpha, delta, causal, beta, logn_mode, bias_mode)
    B, H, Nq, D = Q.shape
    dQ = np.empty_like(Q)
    dK = np.empty_like(K)
    dV = np.empty_like(V)
    dscale = np.empty((B, H, Nq), dtype=np.float64)
    dbeta = np.zeros_like(beta) if beta is not None else None
    dgamma = np.zeros_like(gamma) if gamma is not None else None
    lib.oracle_attn_bwd(ctypes.byref(prm), _dp(Q), _dp(K), _dp(V), _dp(beta), _dp(gamma), _dp(slopes), _dp(dO), _dp(dQ), _dp(dK),
                        _dp(dV), _dp(dbeta), _dp(dgamma), _dp(dscale))
    return {"dQ": dQ, "dK": dK, "dV": dV, "dbeta": dbeta, "dgamma": dgamma, "dscale": dscale}


def tile_map(Q, K, alpha, tq, tk, beta=None, gamma=None, delta=1.0, causal=True, logn_mode=0, slopes=None, bias_mode=0):
    """Block sparsity of the exact attention matrix at tile shape tq x tk.
    Returns (nonzero, visible) uint8 arrays [B,H,ceil(Nq/tq),ceil(Nk/tk)]."""
    lib = _load()
    Q, K, beta, gamma, slopes = _f64(Q), _f64(K), _f64(beta), _f64(gamma), _f64(slopes)
    prm = _params(Q, K, alpha, delta, causal, beta, logn_mode, bias_mode)
    B, H, Nq, _ = Q.shape
    Nk = K.shape[2]
    nti, ntj = (Nq + tq - 1) // tq, (Nk + tk - 1) // tk
    nz = np.empty((B, H, nti, ntj), dtype=np.uint8)
    vis = np.empty((B, H, nti, ntj), dtype=np.uint8)
    u8 = ctypes.POINTER(ctypes.c_uint8)
    lib.oracle_tile_map(ctypes.byref(prm), _dp(Q), _dp(K), _dp(beta), _dp(gamma), _dp(slopes), ctypes.c_int(tq), ctypes.c_int(tk),
                        nz.ctypes.data_as(u8), vis.ctypes.data_as(u8))
    return nz, vis


def scale_proj_fwd(X, Wb, Wg, s):
    """ASEntmax scale projections: X [B,N,E], Wb, Wg [H,E] -> beta, gamma [B,H,N] (per-query layout)."""
    lib = _load()
    X, Wb, Wg = _f64(X), _f64(Wb), _f64(Wg)
    B, N, E = X.shape
    H = Wb.shape[0]
    beta = np.empty((B, H, N), dtype=np.float64)
    gamma = np.empty((B, H, N), dtype=np.float64)
    rc = lib.oracle_scale_proj_fwd(ctypes.c_int(B), ctypes.c_int(H), ctypes.c_int(N), ctypes.c_int(E), ctypes.c_double(s),
                                   _dp(X), _dp(Wb), _dp(Wg), _dp(beta), _dp(gamma))
    assert rc == 0
    return beta, gamma


def scale_proj_bwd(X, Wb, Wg, s, dbeta, dgamma):
    """Gradients of the scale projections: returns dict(dX, dWb, dWg)."""
    lib = _load()
    X, Wb, Wg, dbeta, dgamma = _f64(X), _f64(Wb), _f64(Wg), _f64(dbeta), _f64(dgamma)
    B, N, E = X.shape
    H = Wb.shape[0]
    dX, dWb, dWg = np.empty_like(X), np.empty_like(Wb), np.empty_like(Wg)
    rc = lib.oracle_scale_proj_bwd(ctypes.c_int(B), ctypes.c_int(H), ctypes.c_int(N), ctypes.c_int(E), ctypes.c_double(s),
                                   _dp(X), _dp(Wb), _dp(Wg), _dp(dbeta), _dp(dgamma), _dp(dX), _dp(dWb), _dp(dWg))
    assert rc == 0
    return dict(dX=dX, dWb=dWb, dWg=dWg)
