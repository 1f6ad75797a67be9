"""Helpers for the GPU-vs-oracle parity tests: run the same seeded inputs through
the HIP library (via the ctypes binding) and through the fp64 CPU oracle."""
import numpy as np
import torch

TOL_O = 2e-2      # max-abs on outputs
TOL_TAU = 1e-3    # max-abs on the threshold
TOL_GRAD = 5e-2   # max|diff| / max|ref| per gradient tensor
DEFAULT_PATH = 0   # forward path the tests run when they do not say: 0 automatic, 1 tiled kernel only
DEFAULT_SAVED = False  # whether the backward gets the forward's lists (`saved` buffer)


def to_dev(x, dtype):
    if x is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t.float()


def gpu_run(data, alpha, dtype, causal=True, logn_mode=0, bwd=True, stats=False, layout_bnhd=False, path=None,
            use_saved=None, slopes=None, bias_mode=0, saved_factor=1):
    from paper_2506_16640_amd import binding
    path = DEFAULT_PATH if path is None else path
    use_saved = DEFAULT_SAVED if use_saved is None else use_saved
    q, k, v = (to_dev(data[n], dtype) for n in ("Q", "K", "V"))
    if layout_bnhd:  # same values, [B,n,H,D] memory order viewed as [B,H,n,D]
        q, k, v = (t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in (q, k, v))
    beta = None if data["beta"] is None else torch.from_numpy(data["beta"]).float().cuda()
    gamma = None if data["gamma"] is None else torch.from_numpy(data["gamma"]).float().cuda()
    st = binding.new_stats() if stats else None
    kw = dict(alpha=alpha, beta=beta, gamma=gamma, delta=data["delta"], causal=causal, logn_mode=logn_mode, stats=st,
              path=path, alibi_slopes=None if slopes is None else torch.from_numpy(slopes).float().cuda(),
              bias_mode=bias_mode)
    saved = None
    if use_saved:  # the forward's lists go to the backward, which then skips its own sweep
        prm = binding.make_params(q, k, alpha, data["delta"], causal, beta, logn_mode, path)
        saved = binding.new_saved(prm)
        if saved_factor != 1:  # a roomier pool for the support lists than the size the library asks for
            saved = torch.empty(saved.numel() * saved_factor, dtype=torch.uint8, device="cuda")
    o, tau = binding.entmax_attn_fwd(q, k, v, saved=saved, **kw)
    out = {"O": o.float().cpu().numpy().astype(np.float64), "tau": tau.cpu().numpy().astype(np.float64)}
    if bwd:
        do = to_dev(data["dO"], dtype)
        if layout_bnhd:
            do = do.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
        dq, dk, dv, db, dg = binding.entmax_attn_bwd(q, k, v, o, do, tau, saved=saved, **kw)
        out.update(dQ=dq.float().cpu().numpy().astype(np.float64), dK=dk.float().cpu().numpy().astype(np.float64),
                   dV=dv.float().cpu().numpy().astype(np.float64),
                   dbeta=None if db is None else db.cpu().numpy().astype(np.float64),
                   dgamma=None if dg is None else dg.cpu().numpy().astype(np.float64))
    torch.cuda.synchronize()
    if stats:
        out["stats"] = binding.stats_dict(st)
    return out


def oracle_run(data, alpha, causal=True, logn_mode=0, bwd=True, slopes=None, bias_mode=0):
    from oracle import oracle
    kw = dict(beta=data["beta"], gamma=data["gamma"], delta=data["delta"], causal=causal, logn_mode=logn_mode,
              slopes=slopes, bias_mode=bias_mode)
    out = oracle.attn_fwd(data["Q"], data["K"], data["V"], alpha, **kw)
    if bwd:
        out.update(oracle.attn_bwd(data["Q"], data["K"], data["V"], data["dO"], alpha, **kw))
    return out


def rel_err(a, b):
    denom = np.abs(b).max()
    return float(np.abs(a - b).max() / denom) if denom > 0 else float(np.abs(a).max())


def compare(gpu, ref, bwd=True, tol_o=TOL_O, tol_tau=TOL_TAU, tol_grad=TOL_GRAD, label=""):
    errs = {"tau": float(np.abs(gpu["tau"] - ref["tau"]).max()) if gpu["tau"].size else 0.0,
            "O": float(np.abs(gpu["O"] - ref["O"]).max()) if gpu["O"].size else 0.0}
    assert np.isfinite(gpu["O"]).all() and np.isfinite(gpu["tau"]).all(), label
    assert errs["tau"] <= tol_tau, (label, errs)
    assert errs["O"] <= tol_o, (label, errs)
    if bwd:
        for name in ("dQ", "dK", "dV", "dbeta", "dgamma"):
            if ref.get(name) is None or ref[name].size == 0:
                continue
            assert np.isfinite(gpu[name]).all(), (label, name)
            errs[name] = rel_err(gpu[name], ref[name])
            assert errs[name] <= tol_grad, (label, name, errs)
    return errs


def threshold_residual(sub, tau_rows, rows, alpha, causal=True, logn_mode=0, band=1e-4):
    """For the given rows of ONE head (sub: Q,K [1,1,n,d], per-head beta/gamma or None), from the definition in
    fp64 (numpy only): |f(tau)| with f(tau) = sum_j [(alpha-1) s_ij - tau]_+^(1/(alpha-1)) - 1 at the thresholds
    `tau_rows`, and the number of visible scores within band * max(1, |tau|) of the threshold."""
    Q, K = sub["Q"][0, 0].astype(np.float64), sub["K"][0, 0].astype(np.float64)
    nq, d = Q.shape
    nk = K.shape[0]
    resid, near = [], 0
    for i, t in zip(rows, tau_rows):
        nvis = min(max(i + (nk - nq) + 1, 0), nk) if causal else nk
        if nvis == 0:
            continue
        scale = sub["delta"]
        if sub["beta"] is not None:
            n_log = nk if logn_mode == 0 else nvis
            if n_log > 1:
                b, g = float(np.ravel(sub["beta"])[0]), float(np.ravel(sub["gamma"])[0])
                scale = sub["delta"] + b * np.log(n_log) ** g
        y = (alpha - 1.0) * scale * (K[:nvis] @ Q[i]) / np.sqrt(d)
        x = np.maximum(y - t, 0.0)
        resid.append(abs(float(np.sum(x ** (1.0 / (alpha - 1.0)))) - 1.0))
        near += int(np.sum(np.abs(y - t) < band * max(1.0, abs(t))))
    return (max(resid) if resid else 0.0), near
