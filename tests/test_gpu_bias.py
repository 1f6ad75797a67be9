"""GPU parity with the linear distance bias (Sec. 4.2 NAPE: ALiBi heads beside heads without positional bias;
App. B ALiBi definition and proposition): the HIP library through the C ABI against the fp64 oracle, element by
element, for both placements of the bias (inside / outside the ASEntmax scale), on every forward / backward
path.  Same bars as the other parity tests: 2e-2 on O, 1e-3 on tau, 5e-2 relative on every gradient."""
import numpy as np
import pytest

from paper_2506_16640_amd import synth
from tests.parity_util import compare, gpu_run, oracle_run

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=[(0, False), (0, True), (1, False)], ids=["auto", "auto-saved", "tiled"])
def forward_path(request):
    from tests import parity_util
    parity_util.DEFAULT_PATH, parity_util.DEFAULT_SAVED = request.param
    yield request.param[0]
    parity_util.DEFAULT_PATH, parity_util.DEFAULT_SAVED = 0, False


def _case(B, H, nq, nk, d, dtype, scale, seed=0):
    return synth.make_inputs(B=B, H=H, n=nq, nk=nk, d=d, dtype=dtype, scale=scale, seed=seed)


def _run(data, alpha, dtype, slopes, bias_mode, label, **kw):
    gpu_only = {k: kw.pop(k) for k in ("path", "use_saved") if k in kw}  # how the library runs it, not what is computed
    g = gpu_run(data, alpha, dtype, slopes=slopes, bias_mode=bias_mode, stats=True, **kw, **gpu_only)
    r = oracle_run(data, alpha, slopes=slopes, bias_mode=bias_mode, **kw)
    errs = compare(g, r, label=label)
    print(label, errs, {k: v for k, v in g["stats"].items() if v and k in ("fwd_tiles_visible", "fwd_window_skipped")})
    return g, r


@pytest.mark.parametrize("bias_mode", [0, 1])
@pytest.mark.parametrize("alpha", [1.5, 2.0, 1.25, 1.4])
@pytest.mark.parametrize("d", [64, 128])
def test_nape_small_causal(alpha, d, bias_mode):
    # four heads, every other one biased; several query blocks and key tiles, ragged tail
    data = _case(2, 4, 300, 300, d, "bf16", "head", seed=11)
    _run(data, alpha, "bf16", synth.nape_slopes(4), bias_mode, f"nape a{alpha} d{d} m{bias_mode}")


@pytest.mark.parametrize("bias_mode", [0, 1])
@pytest.mark.parametrize("nq,nk,causal", [(641, 641, True), (200, 333, False), (333, 200, True)])
def test_nape_long_sequence_kernels_at_small_sizes(nq, nk, causal, bias_mode):
    # params.path = 2: the list kernels made for long sequences (two adjacent query blocks per workgroup, block
    # bits), here with the bias as the accumulator's start and the distance window
    data = _case(2, 4, nq, nk, 64, "bf16", "head", seed=14)
    _run(data, 1.5, "bf16", synth.nape_slopes(4), bias_mode, f"nape long kernels {nq} {nk} {causal} m{bias_mode}",
         causal=causal, path=2, use_saved=True)


@pytest.mark.parametrize("bias_mode", [0, 1])
@pytest.mark.parametrize("scale,alpha,dtype", [("none", 1.5, "bf16"), ("dense", 1.5, "bf16"), ("none", 1.25, "fp32"),
                                               ("dense", 2.0, "fp32")])
def test_gentle_slopes_wide_supports(scale, alpha, dtype, bias_mode):
    # slopes of the usual geometric ALiBi family (2^-2 .. 2^-8): the bias competes with the content scores over
    # tens to hundreds of keys, so supports are long and straddle several tiles
    data = _case(1, 4, 700, 700, 64, dtype, scale, seed=12)
    slopes = np.array([2.0 ** -2, 2.0 ** -4, 2.0 ** -6, 2.0 ** -8], dtype=np.float32)
    g, r = _run(data, alpha, dtype, slopes, bias_mode, f"gentle {scale} a{alpha} {dtype} m{bias_mode}")
    assert r["support"].mean() > 2


@pytest.mark.parametrize("bias_mode", [0, 1])
@pytest.mark.parametrize("causal,nq,nk", [(False, 200, 333), (True, 200, 333), (True, 333, 200), (False, 129, 64),
                                           (True, 1, 70), (True, 33, 33)])
def test_bias_rectangular_and_noncausal(causal, nq, nk, bias_mode):
    # the query's position in the key sequence is i + (Nk - Nq); without the causal mask the keys after it carry no bias
    data = _case(1, 2, nq, nk, 64, "bf16", "head", seed=13)
    slopes = np.array([0.25, 0.03125], dtype=np.float32)
    _run(data, 1.5, "bf16", slopes, bias_mode, f"rect {causal} {nq} {nk} m{bias_mode}", causal=causal)


@pytest.mark.parametrize("bias_mode", [0, 1])
@pytest.mark.parametrize("scale,logn_mode", [("query", 0), ("query", 1), ("head", 1)])
def test_bias_with_scale_layouts(scale, logn_mode, bias_mode):
    data = _case(2, 2, 260, 260, 64, "bf16", scale, seed=14)
    slopes = np.array([0.5, 0.0625], dtype=np.float32)
    _run(data, 1.5, "bf16", slopes, bias_mode, f"layout {scale} {logn_mode} m{bias_mode}", logn_mode=logn_mode)


@pytest.mark.parametrize("bias_mode", [0, 1])
def test_negative_scale_turns_the_penalty_into_a_reward(bias_mode):
    # beta < 0 with delta = 0 makes scale_i < 0: inside the scale (mode 0) the bias then grows with distance, and no
    # window exists; outside the scale (mode 1) it still penalises distance
    data = _case(1, 2, 300, 300, 64, "bf16", "head", seed=15)
    data["beta"] = -np.abs(data["beta"]) * 0.05
    data["delta"] = 0.0
    slopes = np.array([0.125, 0.015625], dtype=np.float32)
    g, r = _run(data, 1.5, "bf16", slopes, bias_mode, f"negative scale m{bias_mode}")
    if bias_mode == 0:
        assert g["stats"]["fwd_window_skipped"] == 0


@pytest.mark.parametrize("bias_mode", [0, 1])
def test_far_heavy_keys_stay_in_the_support(bias_mode):
    """A few keys get a norm far above the rest and are aligned with late queries, so that they stay in those
    rows' supports from one or two thousand positions away.  The window is derived from the largest key norm of
    the head, so it must widen enough not to cut them."""
    data = _case(1, 2, 2304, 2304, 64, "bf16", "none", seed=16)
    Q, K = data["Q"], data["K"]
    for h in range(2):
        for (j, i) in ((5, 2000), (130, 2300), (1000, 1999)):
            K[0, h, j] = synth.bf16_round((40.0 * Q[0, h, i] / np.linalg.norm(Q[0, h, i])).astype(np.float32))
    slopes = np.array([1.0 / 64, 1.0 / 32], dtype=np.float32)
    g, r = _run(data, 1.5, "bf16", slopes, bias_mode, f"heavy keys m{bias_mode}")
    from oracle import oracle
    P = oracle.attn_fwd(Q, K, data["V"], 1.5, beta=data["beta"], gamma=data["gamma"], delta=data["delta"],
                        slopes=slopes, bias_mode=bias_mode, want_p=True)["P"]
    assert P[0, 0, 2000, 5] > 0 and P[0, 1, 1999, 1000] > 0


@pytest.mark.parametrize("bias_mode", [0, 1])
def test_window_with_moderately_heavy_keys(bias_mode):
    # keys of twice the usual norm, aligned with queries a few hundred positions later: the window is wider than
    # for plain Gaussian keys but still skips most of the sequence
    data = _case(1, 2, 2304, 2304, 64, "bf16", "none", seed=20)
    Q, K = data["Q"], data["K"]
    for h in range(2):
        for (j, i) in ((1500, 1530), (2000, 2020), (700, 711)):
            K[0, h, j] = synth.bf16_round((16.0 * Q[0, h, i] / np.linalg.norm(Q[0, h, i])).astype(np.float32))
    slopes = np.array([0.5, 0.25], dtype=np.float32)
    g, r = _run(data, 1.5, "bf16", slopes, bias_mode, f"window moderate m{bias_mode}")
    assert g["stats"]["fwd_window_skipped"] > 0


def test_window_skip_rate_without_heavy_keys():
    # Gaussian keys of ordinary norm: with slopes 1 and 1/2 the window is a few dozen keys wide
    data = _case(1, 2, 2304, 2304, 64, "bf16", "head", seed=17)
    slopes = np.array([1.0, 0.5], dtype=np.float32)
    g, r = _run(data, 1.5, "bf16", slopes, 0, "window plain")
    st = g["stats"]
    assert st["fwd_window_skipped"] > 0.5 * st["fwd_tiles_visible"], st


@pytest.mark.parametrize("bias_mode", [0, 1])
@pytest.mark.parametrize("nq,nk", [(1, 4096), (8, 3001), (3, 5)])
def test_bias_decode_shapes(nq, nk, bias_mode):
    data = _case(2, 2, nq, nk, 64, "bf16", "head", seed=18)
    slopes = np.array([0.0, 0.0078125], dtype=np.float32)
    g = gpu_run(data, 1.5, "bf16", bwd=False, slopes=slopes, bias_mode=bias_mode)
    r = oracle_run(data, 1.5, bwd=False, slopes=slopes, bias_mode=bias_mode)
    print(nq, nk, compare(g, r, bwd=False, label=f"decode {nq} {nk} m{bias_mode}"))


def test_zero_slopes_equal_no_bias_bitwise():
    # all slopes zero run the bias-enabled kernels on the same numbers: bit-identical to the run without slopes
    data = _case(1, 2, 300, 300, 64, "bf16", "head", seed=19)
    a = gpu_run(data, 1.5, "bf16", slopes=np.zeros(2, dtype=np.float32))
    b = gpu_run(data, 1.5, "bf16")
    for k in ("O", "tau", "dQ", "dK", "dV"):
        assert np.array_equal(a[k], b[k]), k
