"""Parity at the benchmark's full sizes, in the launch configuration bench.py times: the GPU runs the
whole workload; the fp64 oracle recomputes a few whole heads (heads are independent, so a head of the
full run is compared element by element with the oracle run on that head alone)."""
import numpy as np
import pytest

from paper_2506_16640_amd import synth
from tests.parity_util import TOL_GRAD, TOL_O, TOL_TAU, gpu_run, oracle_run, rel_err

pytestmark = pytest.mark.gpu


def _head_slice(data, b, h):
    sub = {k: data[k][b:b + 1, h:h + 1] for k in ("Q", "K", "V", "dO") if k in data}
    sub["beta"] = None if data["beta"] is None else data["beta"][h:h + 1]
    sub["gamma"] = None if data["gamma"] is None else data["gamma"][h:h + 1]
    sub["delta"] = data["delta"]
    return sub


def _check_heads(name, heads, alpha=None, bwd=None, seed=0):
    data = synth.make_config(name, seed=seed)
    cfg = data["cfg"]
    alpha = cfg["alpha"] if alpha is None else alpha
    bwd = cfg["bwd"] if bwd is None else bwd
    g = gpu_run(data, alpha, cfg["dtype"], bwd=bwd, stats=True)
    worst = {}
    for (b, h) in heads:
        r = oracle_run(_head_slice(data, b, h), alpha, bwd=bwd)
        errs = {"tau": np.abs(g["tau"][b, h] - r["tau"][0, 0]).max(), "O": np.abs(g["O"][b, h] - r["O"][0, 0]).max()}
        assert errs["tau"] <= TOL_TAU and errs["O"] <= TOL_O, (name, b, h, errs)
        if bwd:
            for t in ("dQ", "dK", "dV"):
                errs[t] = rel_err(g[t][b, h], r[t][0, 0])
                assert errs[t] <= TOL_GRAD, (name, b, h, t, errs)
        for k, v in errs.items():
            worst[k] = max(worst.get(k, 0.0), float(v))
    print(name, alpha, "worst errors over heads", heads, worst)
    return data, g


def test_c2_full_forward():
    data = synth.make_config("c2")
    g = gpu_run(data, 1.5, "bf16", bwd=False)
    r = oracle_run(data, 1.5, bwd=False)
    assert np.abs(g["tau"] - r["tau"]).max() <= TOL_TAU
    assert np.abs(g["O"] - r["O"]).max() <= TOL_O
    assert np.abs(g["O"]).max() > 1.0


def test_c3_headline_fwd_bwd_sampled_heads():
    data, g = _check_heads("c3", [(0, 0), (1, 7), (3, 11)])
    # per-head parameter gradients sum over the batch: oracle on all batches of one head
    h = 4
    sub = {k: data[k][:, h:h + 1] for k in ("Q", "K", "V", "dO")}
    sub.update(beta=data["beta"][h:h + 1], gamma=data["gamma"][h:h + 1], delta=data["delta"])
    r = oracle_run(sub, 1.5)
    assert abs(g["dbeta"][h] - r["dbeta"][0]) <= TOL_GRAD * abs(r["dbeta"][0])
    assert abs(g["dgamma"][h] - r["dgamma"][0]) <= TOL_GRAD * abs(r["dgamma"][0])
    st = g["stats"]
    assert st["fwd_sparse_blocks"] > 0.9 * 4 * 12 * 32  # the headline workload is sparse: the list kernel finishes it
    assert st["bwd_active_tiles"] == st["bwd_dq_tiles"] == st["bwd_dkv_tiles"] == 0  # no head needed the tiled backward
    assert st["bwd_support"] == st["fwd_support"]
    # the launch configuration bench.py times: the forward's lists handed to the backward (no second sweep).
    # Same supports, same per-entry arithmetic; only the order of a row's entries may differ.
    g2 = gpu_run(data, 1.5, "bf16", stats=True, use_saved=True)
    st2 = g2["stats"]
    assert st2["bwd_list_qk"] == 0 and st2["bwd_support"] == st["bwd_support"]
    assert st2["bwd_active_tiles"] == st2["bwd_dq_tiles"] == st2["bwd_dkv_tiles"] == 0
    assert np.array_equal(g2["O"], g["O"]) and np.array_equal(g2["tau"], g["tau"])
    for t in ("dQ", "dK", "dV"):
        assert rel_err(g2[t], g[t]) <= 2e-3, t
    for t in ("dbeta", "dgamma"):
        assert np.abs(g2[t] - g[t]).max() <= 2e-3 * np.abs(g[t]).max(), t


def test_c3_dense_companion_sampled_heads():
    _check_heads("c3d", [(0, 3), (2, 10)])


def test_c4_long_context_forward_one_head_and_skip_rate():
    from oracle import oracle
    data = synth.make_config("c4")
    g = gpu_run(data, 1.5, "bf16", bwd=False, stats=True)
    h = 5
    sub = _head_slice(data, 0, h)
    r = oracle_run(sub, 1.5, bwd=False)
    assert np.abs(g["tau"][0, h] - r["tau"][0, 0]).max() <= TOL_TAU
    assert np.abs(g["O"][0, h] - r["O"][0, 0]).max() <= TOL_O
    # tile-skip cross-check on that head: the kernel's executed P.V tiles against the oracle's block sparsity
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
    print("c4 tile-skip rate (32x32 tiles)", skip, "oracle head", 1.0 - nz.sum() / vis.sum())
    assert skip > 0.5


@pytest.mark.parametrize("alpha", [1.25, 1.5, 2.0])
def test_c5_alpha_sweep_d128_sampled_heads(alpha):
    _check_heads("c5", [(0, 2), (1, 13)], alpha=alpha)


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
