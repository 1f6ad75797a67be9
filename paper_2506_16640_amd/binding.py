"""Thin ctypes binding of the C ABI in include/entmax_attn.h.

Argument marshalling only: torch supplies device memory and the stream, every
step of the computation runs in the HIP kernels of lib/libentmax_attn.so.
There is no fallback: if the library is missing, importing this module fails.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "libentmax_attn.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libentmax_attn.so is not built: run `python -m paper_2506_16640_amd.build` "
        "(or __graft_entry__.build()) first; there is no CPU fallback")

_lib = ctypes.CDLL(LIB_PATH)

NUM_STATS = 24
STAT_NAMES = {
    "fwd_tiles_visible": 0, "fwd_qk_max": 1, "fwd_qk_solve": 2, "fwd_qk_pv": 3, "fwd_pv_tiles": 4,
    "fwd_solve_sweeps": 5, "fwd_blocks": 6, "fwd_eval_tiles": 7,
    "bwd_tiles_visible": 8, "bwd_qk_mask": 9, "bwd_active_tiles": 10, "bwd_dq_tiles": 11, "bwd_dkv_tiles": 12,
    "fwd_cand_tiles": 13, "fwd_candidates": 14, "fwd_support": 15, "fwd_sparse_blocks": 16, "fwd_list_qk": 17, "bwd_list_qk": 18, "bwd_support": 19,
    "fwd_window_skipped": 20,
}
FWD_NUM_PHASES = 5
BWD_NUM_PHASES = 8
FWD_PHASES = ("prepare", "lists", "finish", "transpose", "tiled")
BWD_PHASES = ("lists", "rows", "transpose", "mask", "dq", "dkv", "keys", "scale_grad")


class Params(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("H", ctypes.c_int32), ("Nq", ctypes.c_int32), ("Nk", ctypes.c_int32),
        ("D", ctypes.c_int32), ("dtype", ctypes.c_int32), ("causal", ctypes.c_int32),
        ("scale_layout", ctypes.c_int32), ("logn_mode", ctypes.c_int32), ("bias_mode", ctypes.c_int32),
        ("path", ctypes.c_int32),
        ("alpha", ctypes.c_float), ("delta", ctypes.c_float),
        ("q_stride_b", ctypes.c_int64), ("q_stride_h", ctypes.c_int64), ("q_stride_n", ctypes.c_int64),
        ("kv_stride_b", ctypes.c_int64), ("kv_stride_h", ctypes.c_int64), ("kv_stride_n", ctypes.c_int64),
    ]


_vp = ctypes.c_void_p
_lib.entmax_attn_fwd.restype = ctypes.c_int
_lib.entmax_attn_fwd.argtypes = [ctypes.POINTER(Params)] + [_vp] * 9 + [ctypes.c_size_t, _vp, _vp, ctypes.c_size_t, _vp,
                                                                     _vp]
_lib.entmax_attn_bwd.restype = ctypes.c_int
_lib.entmax_attn_bwd.argtypes = ([ctypes.POINTER(Params)] + [_vp] * 7 + [ctypes.c_size_t] + [_vp] * 10 +
                                 [ctypes.c_size_t, _vp, _vp])
_lib.entmax_attn_workspace_bytes.restype = ctypes.c_size_t
_lib.entmax_attn_workspace_bytes.argtypes = [ctypes.POINTER(Params), ctypes.c_int]
_lib.entmax_attn_saved_bytes.restype = ctypes.c_size_t
_lib.entmax_attn_saved_bytes.argtypes = [ctypes.POINTER(Params)]
_lib.entmax_attn_check_params.restype = ctypes.c_int
_lib.entmax_attn_check_params.argtypes = [ctypes.POINTER(Params)]
_lib.entmax_attn_fwd_noalloc.restype = ctypes.c_int
_lib.entmax_attn_fwd_noalloc.argtypes = [ctypes.POINTER(Params)] + [_vp] * 10
_lib.entmax_attn_noalloc_init.restype = ctypes.c_int
_lib.entmax_attn_noalloc_init.argtypes = []
_lib.entmax_attn_noalloc_scratch_bytes.restype = ctypes.c_size_t
_lib.entmax_attn_noalloc_scratch_bytes.argtypes = []
_lib.entmax_attn_mfma_probe.restype = ctypes.c_int
_lib.entmax_attn_mfma_probe.argtypes = [ctypes.c_int, ctypes.c_int, _vp, _vp]


class ProjParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("N", ctypes.c_int32), ("E", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("gamma_scale", ctypes.c_float)]


_lib.entmax_scale_proj_fwd.restype = ctypes.c_int
_lib.entmax_scale_proj_fwd.argtypes = [ctypes.POINTER(ProjParams)] + [_vp] * 6
_lib.entmax_scale_proj_bwd.restype = ctypes.c_int
_lib.entmax_scale_proj_bwd.argtypes = [ctypes.POINTER(ProjParams)] + [_vp] * 11 + [ctypes.c_size_t, _vp]
_lib.entmax_scale_proj_workspace_bytes.restype = ctypes.c_size_t
_lib.entmax_scale_proj_workspace_bytes.argtypes = [ctypes.POINTER(ProjParams)]
_lib.entmax_attn_strerror.restype = ctypes.c_char_p
_lib.entmax_attn_strerror.argtypes = [ctypes.c_int]


class EntmaxAttnError(RuntimeError):
    def __init__(self, code):
        self.code = code
        super().__init__("entmax_attn: %s (%d)" % (_lib.entmax_attn_strerror(code).decode(), code))


def strerror(code):
    return _lib.entmax_attn_strerror(int(code)).decode()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def make_params(q, k, alpha, delta, causal, beta, logn_mode, path=0, bias_mode=0):
    if q.dim() != 4 or k.dim() != 4 or q.shape[:2] != k.shape[:2] or q.shape[3] != k.shape[3]:
        raise ValueError("Q must be [B,H,Nq,D] and K [B,H,Nk,D]")
    B, H, Nq, D = q.shape
    Nk = k.shape[2]
    if q.dtype == torch.bfloat16:
        dt = 0
    elif q.dtype == torch.float32:
        dt = 1
    else:
        raise TypeError("Q must be bfloat16 or float32")
    layout = 0 if beta is None else (1 if beta.dim() == 1 else 2)
    p = Params(B, H, Nq, Nk, D, dt, int(bool(causal)), layout, int(logn_mode), int(bias_mode), int(path), float(alpha), float(delta),
               0, 0, 0, 0, 0, 0)
    if not q.is_contiguous():
        if q.stride(3) != 1:
            raise ValueError("the last dimension of Q must be contiguous")
        p.q_stride_b, p.q_stride_h, p.q_stride_n = q.stride(0), q.stride(1), q.stride(2)
    if not k.is_contiguous():
        if k.stride(3) != 1:
            raise ValueError("the last dimension of K must be contiguous")
        p.kv_stride_b, p.kv_stride_h, p.kv_stride_n = k.stride(0), k.stride(1), k.stride(2)
    return p


def _check_like(name, t, ref):
    """t must have ref's shape, strides, dtype and device (the ABI passes one set of strides per tensor family)."""
    if t.shape != ref.shape or t.stride() != ref.stride():
        raise ValueError("%s must have the shape and strides of its reference tensor" % name)
    if t.dtype != ref.dtype or t.device != ref.device:
        raise TypeError("%s must have the dtype and device of Q" % name)


def _check_scale(p, q, beta, gamma):
    if (beta is None) != (gamma is None):
        raise ValueError("beta and gamma come together")
    if beta is None:
        return
    want = (p.H,) if p.scale_layout == 1 else (p.B, p.H, p.Nq)
    for name, t in (("beta", beta), ("gamma", gamma)):
        if t.dtype != torch.float32 or not t.is_contiguous() or tuple(t.shape) != want or t.device != q.device:
            raise ValueError("%s must be a contiguous float32 tensor of shape %s on Q's device" % (name, want))


def _check_slopes(p, q, slopes):
    if slopes is None:
        return
    if slopes.dtype != torch.float32 or not slopes.is_contiguous() or tuple(slopes.shape) != (p.H,) or slopes.device != q.device:
        raise ValueError("alibi_slopes must be a contiguous float32 tensor of shape (%d,) on Q's device" % p.H)


def _check_aux(p, stats, saved, workspace, is_bwd):
    if stats is not None and (stats.numel() < NUM_STATS or stats.element_size() != 8 or not stats.is_contiguous()):
        raise ValueError("stats must be a contiguous 64-bit integer tensor with at least %d entries" % NUM_STATS)
    if saved is not None and (saved.dtype != torch.uint8 or not saved.is_contiguous()):
        raise ValueError("saved must be a contiguous uint8 tensor")
    if workspace is not None and (workspace.dtype != torch.uint8 or not workspace.is_contiguous()):
        raise ValueError("workspace must be a contiguous uint8 tensor")


def workspace_bytes(params, is_bwd):
    return int(_lib.entmax_attn_workspace_bytes(ctypes.byref(params), int(is_bwd)))


def saved_bytes(params):
    return int(_lib.entmax_attn_saved_bytes(ctypes.byref(params)))


def new_saved(params, device="cuda"):
    """Buffer that carries the forward's lists to the backward (pass it to both as `saved`), of the size the library
    asks for; a larger uint8 tensor holds longer lists."""
    return torch.empty(max(saved_bytes(params), 256), dtype=torch.uint8, device=device)


def check_params(params):
    return int(_lib.entmax_attn_check_params(ctypes.byref(params)))


def _events_arg(events, n):
    if events is None:
        return None
    if len(events) != n + 1:
        raise ValueError("phase_events needs %d handles" % (n + 1))
    arr = (ctypes.c_void_p * (n + 1))(*[ctypes.c_void_p(e) for e in events])
    return arr


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def entmax_attn_fwd(q, k, v, alpha=1.5, beta=None, gamma=None, delta=1.0, causal=True, logn_mode=0, path=0,
                    out=None, tau=None, stats=None, workspace=None, phase_events=None, saved=None, alibi_slopes=None,
                    bias_mode=0):
    """O, tau = entmax attention forward.  q [B,H,Nq,D], k,v [B,H,Nk,D] on the GPU, bf16 or fp32;
    beta,gamma fp32 [H] or [B,H,Nq] or None.  stats: optional uint64/int64 device tensor [NUM_STATS] (added to).
    path: 0 automatic, 1 tiled kernel only.  phase_events: optional list of FWD_NUM_PHASES + 1 hipEvent_t handles.
    saved: optional uint8 device tensor of at least saved_bytes(params) bytes, filled for the backward.
    alibi_slopes: optional fp32 [H] slopes of the linear distance bias (0 = head without bias); bias_mode 0 puts the
    bias inside the ASEntmax scale, 1 outside."""
    p = make_params(q, k, alpha, delta, causal, beta, logn_mode, path, bias_mode)
    _check_slopes(p, q, alibi_slopes)
    if k.dtype != q.dtype or k.device != q.device:
        raise TypeError("K must have the dtype and device of Q")
    _check_like("V", v, k)
    _check_scale(p, q, beta, gamma)
    _check_aux(p, stats, saved, workspace, False)
    if out is None:
        out = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    else:
        _check_like("out", out, q)
    if tau is None:
        tau = torch.empty(q.shape[:3], dtype=torch.float32, device=q.device)
    elif tau.dtype != torch.float32 or not tau.is_contiguous() or tau.shape != q.shape[:3]:
        raise ValueError("tau must be a contiguous float32 tensor [B,H,Nq]")
    need = workspace_bytes(p, 0)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    ev = _events_arg(phase_events, FWD_NUM_PHASES)
    rc = _lib.entmax_attn_fwd(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(beta), _ptr(gamma),
                              _ptr(alibi_slopes), _ptr(out), _ptr(tau), _ptr(saved),
                              0 if saved is None else saved.numel(), _ptr(stats),
                              _ptr(workspace), workspace.numel(), _stream(), ev)
    if rc != 0:
        raise EntmaxAttnError(rc)
    return out, tau


def mfma_probe(iters, blocks, sink):
    """Enqueue the matrix-pipeline probe; returns the flops it issues (the caller times it)."""
    rc = _lib.entmax_attn_mfma_probe(int(iters), int(blocks), _ptr(sink), _stream())
    if rc != 0:
        raise EntmaxAttnError(rc)
    return float(blocks) * 4 * iters * 4 * 2 * 32 * 32 * 16


def noalloc_scratch_bytes():
    return int(_lib.entmax_attn_noalloc_scratch_bytes())


def noalloc_init():
    rc = _lib.entmax_attn_noalloc_init()
    if rc != 0:
        raise EntmaxAttnError(rc)


def entmax_attn_fwd_noalloc(q, k, v, out, tau, alpha=1.5, beta=None, gamma=None, delta=1.0, causal=True, logn_mode=0,
                            path=0, stats=None, alibi_slopes=None, bias_mode=0):
    """Forward through the entry point that allocates nothing: the caller brings `out` and `tau`, the scratch is
    the library's built-in buffer (noalloc_scratch_bytes()).  Raises EntmaxAttnError(-6) for problems beyond it."""
    p = make_params(q, k, alpha, delta, causal, beta, logn_mode, path, bias_mode)
    _check_slopes(p, q, alibi_slopes)
    if k.dtype != q.dtype or k.device != q.device:
        raise TypeError("K must have the dtype and device of Q")
    _check_like("V", v, k)
    _check_like("out", out, q)
    _check_scale(p, q, beta, gamma)
    _check_aux(p, stats, None, None, False)
    if tau.dtype != torch.float32 or not tau.is_contiguous() or tau.shape != q.shape[:3]:
        raise ValueError("tau must be a contiguous float32 tensor [B,H,Nq]")
    rc = _lib.entmax_attn_fwd_noalloc(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(beta), _ptr(gamma),
                                      _ptr(alibi_slopes), _ptr(out), _ptr(tau), _ptr(stats), _stream())
    if rc != 0:
        raise EntmaxAttnError(rc)
    return out, tau


def entmax_attn_bwd(q, k, v, o, do, tau, alpha=1.5, beta=None, gamma=None, delta=1.0, causal=True, logn_mode=0, path=0,
                    stats=None, workspace=None, phase_events=None, saved=None, alibi_slopes=None, bias_mode=0):
    """dQ, dK, dV, dbeta, dgamma = entmax attention backward (dbeta/dgamma None without scale parameters).
    saved: the buffer the forward filled for the same inputs, or None.  alibi_slopes, bias_mode: as in the forward."""
    p = make_params(q, k, alpha, delta, causal, beta, logn_mode, path, bias_mode)
    _check_slopes(p, q, alibi_slopes)
    if k.dtype != q.dtype or k.device != q.device:
        raise TypeError("K must have the dtype and device of Q")
    _check_like("V", v, k)
    _check_like("dO", do, q)
    _check_scale(p, q, beta, gamma)
    _check_aux(p, stats, saved, workspace, True)
    if tau.dtype != torch.float32 or not tau.is_contiguous() or tau.shape != q.shape[:3]:
        raise ValueError("tau must be a contiguous float32 tensor [B,H,Nq]")
    dq = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    dk = torch.empty_strided(k.shape, k.stride(), dtype=k.dtype, device=k.device)
    dv = torch.empty_strided(v.shape, v.stride(), dtype=v.dtype, device=v.device)
    dbeta = torch.empty_like(beta) if beta is not None else None
    dgamma = torch.empty_like(gamma) if gamma is not None else None
    need = workspace_bytes(p, 1)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    ev = _events_arg(phase_events, BWD_NUM_PHASES)
    rc = _lib.entmax_attn_bwd(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(do), _ptr(tau), _ptr(saved),
                              0 if saved is None else saved.numel(), _ptr(beta), _ptr(gamma),
                              _ptr(alibi_slopes), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dbeta), _ptr(dgamma), _ptr(stats),
                              _ptr(workspace), workspace.numel(), _stream(), ev)
    if rc != 0:
        raise EntmaxAttnError(rc)
    return dq, dk, dv, dbeta, dgamma


def new_stats(device="cuda"):
    return torch.zeros(NUM_STATS, dtype=torch.int64, device=device)


def stats_dict(stats):
    vals = stats.cpu().tolist()
    return {name: int(vals[i]) for name, i in STAT_NAMES.items()}


def _proj_params(x, wb, wg, gamma_scale):
    if x.dim() != 3 or not x.is_contiguous():
        raise ValueError("X must be a contiguous [B,N,E] tensor")
    if x.dtype == torch.bfloat16:
        dt = 0
    elif x.dtype == torch.float32:
        dt = 1
    else:
        raise TypeError("X must be bfloat16 or float32")
    B, N, E = x.shape
    for name, w in (("Wb", wb), ("Wg", wg)):
        if w.dtype != torch.float32 or not w.is_contiguous() or w.dim() != 2 or w.shape[1] != E or w.device != x.device:
            raise ValueError("%s must be a contiguous float32 [H,E] tensor on X's device" % name)
    if wb.shape != wg.shape:
        raise ValueError("Wb and Wg must have the same shape")
    return ProjParams(B, wb.shape[0], N, E, dt, float(gamma_scale))


def scale_proj_fwd(x, wb, wg, gamma_scale=1.0):
    """beta, gamma [B,H,N] fp32 = softplus(X Wb^T), gamma_scale * tanh(X Wg^T), in the attention's per-query layout."""
    p = _proj_params(x, wb, wg, gamma_scale)
    beta = torch.empty(p.B, p.H, p.N, dtype=torch.float32, device=x.device)
    gamma = torch.empty_like(beta)
    rc = _lib.entmax_scale_proj_fwd(ctypes.byref(p), _ptr(x), _ptr(wb), _ptr(wg), _ptr(beta), _ptr(gamma), _stream())
    if rc != 0:
        raise EntmaxAttnError(rc)
    return beta, gamma


def scale_proj_bwd(x, wb, wg, beta, gamma, dbeta, dgamma, gamma_scale=1.0, workspace=None):
    """dX [B,N,E] (X's dtype), dWb, dWg [H,E] fp32 from the attention backward's d beta, d gamma."""
    p = _proj_params(x, wb, wg, gamma_scale)
    for name, t in (("beta", beta), ("gamma", gamma), ("dbeta", dbeta), ("dgamma", dgamma)):
        if t.dtype != torch.float32 or not t.is_contiguous() or tuple(t.shape) != (p.B, p.H, p.N) or t.device != x.device:
            raise ValueError("%s must be a contiguous float32 [B,H,N] tensor on X's device" % name)
    need = int(_lib.entmax_scale_proj_workspace_bytes(ctypes.byref(p)))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    elif workspace.dtype != torch.uint8 or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous uint8 tensor")
    dx = torch.empty_like(x)
    dwb, dwg = torch.empty_like(wb), torch.empty_like(wg)
    rc = _lib.entmax_scale_proj_bwd(ctypes.byref(p), _ptr(x), _ptr(wb), _ptr(wg), _ptr(beta), _ptr(gamma), _ptr(dbeta),
                                    _ptr(dgamma), _ptr(dx), _ptr(dwb), _ptr(dwg), _ptr(workspace), workspace.numel(),
                                    _stream())
    if rc != 0:
        raise EntmaxAttnError(rc)
    return dx, dwb, dwg
