"""Parity at the benchmark's full sizes, in the launch configuration bench.py times: the GPU runs the
whole workload and the fp64 oracle recomputes whole heads (a head of the full run is compared element by
element with the oracle run on that head alone; the headline workload is compared on every head)."""
import numpy as np
import pytest

from paper_2506_16640_amd import synth
from tests.parity_util import TOL_GRAD, TOL_O, TOL_TAU, gpu_run, oracle_run, rel_err, threshold_residual

pytestmark = pytest.mark.gpu


def _head_slice(data, b, h):
    sub = {k: data[k][b:b + 1, h:h + 1] for k in ("Q", "K", "V", "dO") if k in data}
    sub["beta"] = None if data["beta"] is None else data["beta"][h:h + 1]
    sub["gamma"] = None if data["gamma"] is None else data["gamma"][h:h + 1]
    sub["delta"] = data["delta"]
    return sub


def _heads_slice(data, h):
    """All batches of head h (the per-head parameter gradients sum over the batch)."""
    sub = {k: data[k][:, h:h + 1] for k in ("Q", "K", "V", "dO") if k in data}
    sub.update(beta=data["beta"][h:h + 1], gamma=data["gamma"][h:h + 1], delta=data["delta"])
    return sub


def _compare_head(name, g, r, b, h, bwd, worst):
    errs = {"tau": np.abs(g["tau"][b, h] - r["tau"][0, 0]).max(), "O": np.abs(g["O"][b, h] - r["O"][0, 0]).max()}
    assert errs["tau"] <= TOL_TAU and errs["O"] <= TOL_O, (name, b, h, errs)
    if bwd:
        for t in ("dQ", "dK", "dV"):
            errs[t] = rel_err(g[t][b, h], r[t][0, 0])
            assert errs[t] <= TOL_GRAD, (name, b, h, t, errs)
    for k, v in errs.items():
        worst[k] = max(worst.get(k, 0.0), float(v))


def _check_heads(name, heads, alpha=None, bwd=None, seed=0, use_saved=None, data=None, g=None):
    data = synth.make_config(name, seed=seed) if data is None else data
    cfg = data["cfg"]
    alpha = cfg["alpha"] if alpha is None else alpha
    bwd = cfg["bwd"] if bwd is None else bwd
    if g is None:
        g = gpu_run(data, alpha, cfg["dtype"], bwd=bwd, stats=True, use_saved=use_saved)
    worst = {}
    for (b, h) in heads:
        _compare_head(name, g, oracle_run(_head_slice(data, b, h), alpha, bwd=bwd), b, h, bwd, worst)
    print(name, alpha, "worst errors over", len(heads), "heads", worst, flush=True)
    return data, g


def _check_scale_grads(name, data, g, alpha, heads):
    """d beta, d gamma of the given heads: oracle on all batches of each head."""
    worst = {}
    for h in heads:
        r = oracle_run(_heads_slice(data, h), alpha)
        for t in ("dbeta", "dgamma"):
            err = abs(g[t][h] - r[t][0]) / abs(r[t][0])
            assert err <= TOL_GRAD, (name, h, t, err)
            worst[t] = max(worst.get(t, 0.0), float(err))
    print(name, alpha, "worst d beta / d gamma error over heads", heads, worst, flush=True)


def _report_residual(name, data, g, alpha, heads, nrows=256):
    """|f(tau_gpu)| in fp64 from the definition, on sampled rows; printed beside the 1e-3 bar on tau."""
    n = data["Q"].shape[2]
    rows = np.unique(np.linspace(0, n - 1, nrows).astype(np.int64))
    worst, near = 0.0, 0
    for (b, h) in heads:
        res, nr = threshold_residual(_head_slice(data, b, h), g["tau"][b, h][rows], rows, alpha)
        worst, near = max(worst, res), near + nr
    print(name, alpha, "max |f_fp64(tau_gpu)| over %d sampled rows of %d heads: %.3g; scores within 1e-4 of the "
          "threshold: %d" % (len(rows), len(heads), worst, near), flush=True)
    # f' = -r sum x^(r-1) is at most r n in magnitude but O(1) for these sparse rows: |f| tracks the tau error
    assert worst < 5e-2, worst
    return worst


def test_c2_full_forward():
    data = synth.make_config("c2")
    g = gpu_run(data, 1.5, "bf16", bwd=False)
    r = oracle_run(data, 1.5, bwd=False)
    assert np.abs(g["tau"] - r["tau"]).max() <= TOL_TAU
    assert np.abs(g["O"] - r["O"]).max() <= TOL_O
    assert np.abs(g["O"]).max() > 1.0


def test_c3_headline_fwd_bwd_every_head():
    data = synth.make_config("c3")
    g = gpu_run(data, 1.5, "bf16", stats=True)
    r = oracle_run(data, 1.5)  # the whole workload: 48 heads, forward and backward
    worst = {"tau": float(np.abs(g["tau"] - r["tau"]).max()), "O": float(np.abs(g["O"] - r["O"]).max())}
    assert worst["tau"] <= TOL_TAU and worst["O"] <= TOL_O, worst
    B, H = data["Q"].shape[:2]
    for t in ("dQ", "dK", "dV"):
        per_head = [rel_err(g[t][b, h], r[t][b, h]) for b in range(B) for h in range(H)]
        worst[t] = max(per_head)
        assert worst[t] <= TOL_GRAD, (t, per_head)
    for t in ("dbeta", "dgamma"):
        per_head = np.abs(g[t] - r[t]) / np.abs(r[t])
        worst[t] = float(per_head.max())
        assert worst[t] <= TOL_GRAD, (t, per_head)
    print("c3 worst errors over all 48 heads", worst, flush=True)
    _report_residual("c3", data, g, 1.5, [(0, 0), (1, 7), (3, 11)])
    st = g["stats"]
    assert st["fwd_sparse_blocks"] > 0.9 * 4 * 12 * 32  # the headline workload is sparse: the list kernel finishes it
    assert st["bwd_active_tiles"] == st["bwd_dq_tiles"] == st["bwd_dkv_tiles"] == 0  # no head needed the tiled backward
    assert st["bwd_support"] == st["fwd_support"]
    assert abs(st["fwd_support"] - int(r["support"].sum())) <= 1e-4 * int(r["support"].sum())
    # the launch configuration bench.py times: the forward's lists handed to the backward (no second sweep),
    # again against the oracle on every head
    g2 = gpu_run(data, 1.5, "bf16", stats=True, use_saved=True)
    st2 = g2["stats"]
    assert st2["bwd_list_qk"] == 0 and st2["bwd_support"] == st["bwd_support"]
    assert st2["bwd_active_tiles"] == st2["bwd_dq_tiles"] == st2["bwd_dkv_tiles"] == 0
    assert np.array_equal(g2["O"], g["O"]) and np.array_equal(g2["tau"], g["tau"])
    worst2 = {}
    for t in ("dQ", "dK", "dV"):
        worst2[t] = max(rel_err(g2[t][b, h], r[t][b, h]) for b in range(B) for h in range(H))
        assert worst2[t] <= TOL_GRAD, (t, worst2)
    for t in ("dbeta", "dgamma"):
        worst2[t] = float((np.abs(g2[t] - r[t]) / np.abs(r[t])).max())
        assert worst2[t] <= TOL_GRAD, (t, worst2)
    print("c3 with the forward's lists: worst errors over all 48 heads", worst2, flush=True)


def test_c3_dense_companion_sampled_heads():
    data, g = _check_heads("c3d", [(0, 3), (2, 10), (3, 0)])
    _check_scale_grads("c3d", data, g, 1.5, [10])


def _extreme_heads(data, n):
    """Heads with the smallest and the largest ASEntmax multiplier beta (ln n)^gamma, and two in between."""
    mult = data["beta"] * np.log(n) ** data["gamma"]
    order = np.argsort(mult)
    return [int(order[0]), int(order[len(order) // 3]), int(order[2 * len(order) // 3]), int(order[-1])]


def test_c4_long_context_forward_heads_and_skip_rate():
    from oracle import oracle
    data = synth.make_config("c4")
    g = gpu_run(data, 1.5, "bf16", bwd=False, stats=True)
    heads = _extreme_heads(data, 32768)
    worst = {}
    for h in heads:
        sub = _head_slice(data, 0, h)
        r = oracle_run(sub, 1.5, bwd=False)
        _compare_head("c4", g, r, 0, h, False, worst)
    print("c4 heads", heads, "worst errors", worst, flush=True)
    _report_residual("c4", data, g, 1.5, [(0, heads[0]), (0, heads[-1])], nrows=64)
    # tile-skip cross-check on one head: the kernel's executed P.V tiles against the oracle's block sparsity
    h = heads[1]
    sub = _head_slice(data, 0, h)
    r = oracle_run(sub, 1.5, bwd=False)
    nz, vis = oracle.tile_map(sub["Q"], sub["K"], 1.5, 32, 32, sub["beta"], sub["gamma"], delta=sub["delta"])
    # tiled kernel alone: the P.V tiles it executes are exactly the oracle's non-zero tiles
    gt = gpu_run(sub, 1.5, "bf16", bwd=False, stats=True, path=1)["stats"]
    assert gt["fwd_tiles_visible"] == int(vis.sum())
    assert abs(gt["fwd_pv_tiles"] - int(nz.sum())) <= 1e-3 * int(nz.sum()) + 2
    # list kernel: its candidate tiles cover the non-zero tiles, and its support count is the oracle's
    gl = gpu_run(sub, 1.5, "bf16", bwd=False, stats=True, path=0)["stats"]
    assert gl["fwd_tiles_visible"] == int(vis.sum())
    if gl["fwd_sparse_blocks"] == 32768 // 128:
        assert gl["fwd_cand_tiles"] >= int(nz.sum())
        assert abs(gl["fwd_support"] - int(r["support"].sum())) <= 1e-3 * int(r["support"].sum()) + 2
    st = g["stats"]
    skip = 1.0 - (st["fwd_cand_tiles"] + st["fwd_pv_tiles"]) / st["fwd_tiles_visible"]
    print("c4 tile-skip rate (32x32 tiles)", skip, "oracle head", 1.0 - nz.sum() / vis.sum(), flush=True)
    assert skip > 0.5


def test_c4_dense_companion_one_head():
    # the low-sparsity companion of the long-context workload: one head (12 would take the tiled kernels
    # half a minute), against the oracle
    data = synth.make_config("c4d")
    sub = _head_slice(data, 0, 7)
    g = gpu_run(sub, 1.5, "bf16", bwd=False, stats=True)
    r = oracle_run(sub, 1.5, bwd=False)
    errs = {"tau": float(np.abs(g["tau"] - r["tau"]).max()), "O": float(np.abs(g["O"] - r["O"]).max())}
    print("c4d head 7", errs, "support per row", float(r["support"].mean()), flush=True)
    assert errs["tau"] <= TOL_TAU and errs["O"] <= TOL_O, errs


@pytest.mark.parametrize("alpha", [1.25, 1.5, 2.0])
def test_c5_alpha_sweep_d128_sampled_heads(alpha):
    data, g = _check_heads("c5", [(0, 2), (1, 2), (1, 13)], alpha=alpha, use_saved=True)
    _check_scale_grads("c5", data, g, alpha, [2])
    _report_residual("c5", data, g, alpha, [(0, 2), (1, 13)], nrows=128)
    if alpha == 2.0:
        # alpha = 2: g = 1 on the support and 0 off it, so a score within rounding of the threshold flips a
        # gradient term by O(1/|S|).  Count such rows of one head and give the dQ error with and without them.
        b, h = 0, 2
        sub = _head_slice(data, b, h)
        r = oracle_run(sub, alpha)
        n = sub["Q"].shape[2]
        rows = np.arange(0, n, 8)
        near_rows = [int(i) for i in rows
                     if threshold_residual(sub, r["tau"][0, 0][[i]], [i], alpha)[1] > 0]
        keep = np.ones(n, dtype=bool)
        keep[near_rows] = False
        e_all = rel_err(g["dQ"][b, h][rows], r["dQ"][0, 0][rows])
        e_wo = rel_err(g["dQ"][b, h][rows][keep[rows]], r["dQ"][0, 0][rows][keep[rows]])
        print("c5 alpha=2 head (0,2): %d of %d sampled rows hold a score within 1e-4 of the threshold; dQ error on "
              "the sampled rows %.3g, without those rows %.3g" % (len(near_rows), len(rows), e_all, e_wo), flush=True)


@pytest.mark.parametrize("bias_mode", [0, 1])
def test_c3_nape_fwd_bwd_sampled_heads(bias_mode):
    """The headline workload with the NAPE arrangement of Sec. 4.2 (every other head carries the linear distance
    bias): biased and unbiased heads against the oracle, with the forward's lists handed to the backward, and
    the parameter gradients of one head of each kind."""
    data = synth.make_config("c3")
    slopes = synth.nape_slopes(12)
    g = gpu_run(data, 1.5, "bf16", stats=True, use_saved=True, slopes=slopes, bias_mode=bias_mode)
    worst = {}
    for (b, h) in ((0, 0), (1, 1), (2, 4), (3, 7), (0, 10), (3, 11)):
        r = oracle_run(_head_slice(data, b, h), 1.5, slopes=slopes[h:h + 1], bias_mode=bias_mode)
        _compare_head("c3 nape", g, r, b, h, True, worst)
    print("c3 nape mode", bias_mode, "worst errors over 6 heads", worst, flush=True)
    wg = {}
    for h in (4, 7):
        r = oracle_run(_heads_slice(data, h), 1.5, slopes=slopes[h:h + 1], bias_mode=bias_mode)
        for t in ("dbeta", "dgamma"):
            err = abs(g[t][h] - r[t][0]) / abs(r[t][0])
            assert err <= TOL_GRAD, (h, t, err)
            wg[t] = max(wg.get(t, 0.0), float(err))
    st = g["stats"]
    print("c3 nape mode", bias_mode, "d beta / d gamma", wg, "window-skipped fraction of visible tiles",
          st["fwd_window_skipped"] / st["fwd_tiles_visible"], flush=True)
    # half of the heads are biased with slopes >= 1/2: most of their tiles lie beyond the window (outside the
    # scale -- mode 1 -- the bias is weaker relative to the scaled content scores, and the window wider)
    assert st["fwd_window_skipped"] > (0.4 if bias_mode == 0 else 0.25) * st["fwd_tiles_visible"]


def test_c4_nape_long_context_forward():
    data = synth.make_config("c4")
    slopes = synth.nape_slopes(12)
    g = gpu_run(data, 1.5, "bf16", bwd=False, stats=True, slopes=slopes)
    worst = {}
    for h in (0, 5, 6, 11):
        r = oracle_run(_head_slice(data, 0, h), 1.5, bwd=False, slopes=slopes[h:h + 1])
        _compare_head("c4 nape", g, r, 0, h, False, worst)
    st = g["stats"]
    skip = 1.0 - (st["fwd_cand_tiles"] + st["fwd_pv_tiles"]) / st["fwd_tiles_visible"]
    print("c4 nape worst errors", worst, "tile-skip rate", skip, "never visited (window)",
          st["fwd_window_skipped"] / st["fwd_tiles_visible"], flush=True)
    assert st["fwd_window_skipped"] > 0.4 * st["fwd_tiles_visible"]


@pytest.mark.parametrize("nq", [1, 8])
def test_decode_full_size(nq):
    """The decode workload bench.py times (B=4, H=12, Nk=32768, d=64, bf16): every row against the oracle,
    which needs only Nq rows per head."""
    data = synth.make_inputs(B=4, H=12, n=nq, nk=32768, d=64, dtype="bf16", scale="head", seed=0, want_dO=False)
    g = gpu_run(data, 1.5, "bf16", bwd=False)
    r = oracle_run(data, 1.5, bwd=False)
    errs = {"tau": float(np.abs(g["tau"] - r["tau"]).max()), "O": float(np.abs(g["O"] - r["O"]).max())}
    print("decode full size", nq, errs, "support per row", float(r["support"].mean()))
    assert errs["tau"] <= TOL_TAU and errs["O"] <= TOL_O, errs
