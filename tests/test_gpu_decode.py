"""GPU parity of the decode shapes (a few query rows against a long key sequence, the regime of the
paper's long-context evaluation): the split-key kernels behind entmax_attn_fwd against the fp64 oracle.
Same bars as the other parity tests: max-abs 2e-2 on O, 1e-3 on tau, 5e-2 relative on gradients."""
import numpy as np
import pytest

from paper_2506_16640_amd import synth
from tests.parity_util import compare, gpu_run, oracle_run

pytestmark = pytest.mark.gpu


def _case(nq, nk, d, dtype, scale, seed, B=2, H=3):
    return synth.make_inputs(B=B, H=H, n=nq, nk=nk, d=d, dtype=dtype, scale=scale, seed=seed)


@pytest.mark.parametrize("nq,nk", [(1, 1), (1, 70), (1, 5000), (3, 1500), (8, 777), (8, 4133)])
@pytest.mark.parametrize("alpha", [1.5, 2.0, 1.25, 1.7])
def test_decode_forward(nq, nk, alpha):
    # key chunks of 512: 4133 and 5000 span several with a ragged last one; causal rows see nk - nq + i + 1 keys
    data = _case(nq, nk, 64, "bf16", "head", seed=11)
    g = gpu_run(data, alpha, "bf16", bwd=False)
    r = oracle_run(data, alpha, bwd=False)
    print(nq, nk, alpha, compare(g, r, bwd=False, label=f"decode {nq}x{nk} a{alpha}"))


@pytest.mark.parametrize("nq,nk,decode", [(9, 600, True), (15, 1000, True), (16, 1100, True), (17, 1100, True), (33, 2200, True), (64, 4133, True), (64, 4000, False),
                                          (65, 5000, False)])
def test_decode_more_rows_against_long_keys(nq, nk, decode):
    # up to 64 rows take the split-key kernels when the keys are at least 64 times as many; the tile counters
    # (which only the training kernels keep) tell which path ran
    data = _case(nq, nk, 64, "bf16", "head", seed=18, B=1, H=2)
    g = gpu_run(data, 1.5, "bf16", bwd=False, stats=True)
    r = oracle_run(data, 1.5, bwd=False)
    print(nq, nk, compare(g, r, bwd=False, label=f"decode {nq}x{nk}"))
    assert (g["stats"]["fwd_list_qk"] + g["stats"]["fwd_qk_max"] == 0) == decode


@pytest.mark.parametrize("d,dtype", [(64, "fp32"), (128, "bf16"), (128, "fp32")])
@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("nq", [5, 20])
def test_decode_dtypes_and_head_dims(d, dtype, causal, nq):
    data = _case(nq, 1300, d, dtype, "head", seed=12)
    g = gpu_run(data, 1.5, dtype, causal=causal, bwd=False)
    r = oracle_run(data, 1.5, causal=causal, bwd=False)
    print(d, dtype, causal, compare(g, r, bwd=False, label=f"decode d{d} {dtype}"))


@pytest.mark.parametrize("scale,logn_mode", [("none", 0), ("query", 0), ("query", 1), ("head", 1)])
def test_decode_scale_layouts(scale, logn_mode):
    data = _case(4, 900, 64, "bf16", scale, seed=13)
    g = gpu_run(data, 1.5, "bf16", logn_mode=logn_mode, bwd=False)
    r = oracle_run(data, 1.5, logn_mode=logn_mode, bwd=False)
    print(scale, logn_mode, compare(g, r, bwd=False, label=f"decode scale {scale} {logn_mode}"))


def test_decode_negative_and_zero_scale():
    data = _case(2, 600, 64, "bf16", "head", seed=14, B=1)
    data["beta"] = np.array([-0.8, 0.0, 0.5], dtype=np.float32)  # negative multiplier; scale = delta = 0; ordinary
    data["gamma"] = np.ones(3, dtype=np.float32)
    data["delta"] = 0.0
    g = gpu_run(data, 1.5, "bf16", bwd=False)
    r = oracle_run(data, 1.5, bwd=False)
    print(compare(g, r, bwd=False, label="decode neg/zero scale"))


@pytest.mark.parametrize("alpha", [1.5, 2.0, 1.25, 1.1])
def test_decode_long_supports(alpha):
    """Supports longer than the solver's in-LDS candidate list (4096 keys): zero queries give equal scores, so
    every visible key is in the support with p = 1/n_i, tau = -(n_i)^-(alpha-1) and O the mean of the values;
    the dense recipe (delta = 0, gamma = -1/2) keeps most of 6000 keys within reach of the threshold."""
    nq, nk = 3, 6000
    data = _case(nq, nk, 64, "bf16", "dense", seed=15, B=1, H=2)
    data["Q"][:, 0] = 0.0
    g = gpu_run(data, alpha, "bf16", bwd=False)
    r = oracle_run(data, alpha, bwd=False)
    print(alpha, compare(g, r, bwd=False, label=f"decode long a{alpha}"))
    for i in range(nq):
        n_i = nk - nq + i + 1
        assert abs(g["tau"][0, 0, i] + n_i ** -(alpha - 1.0)) < 1e-3
        np.testing.assert_allclose(g["O"][0, 0, i], data["V"][0, 0, :n_i].mean(axis=0), atol=2e-2)


def test_decode_rows_without_keys():
    # more query rows than keys under the causal mask: the first rows see nothing, O = 0 and tau = 0 there
    data = _case(6, 4, 64, "bf16", "head", seed=16, B=1, H=2)
    g = gpu_run(data, 1.5, "bf16", bwd=False)
    r = oracle_run(data, 1.5, bwd=False)
    print(compare(g, r, bwd=False, label="decode empty rows"))
    assert np.all(g["O"][:, :, :2] == 0.0)


@pytest.mark.parametrize("use_saved", [False, True])
def test_decode_forward_then_backward(use_saved):
    # the backward kernels take tau from the decode forward (with `saved`: told to use the tiled kernels)
    data = _case(8, 700, 64, "bf16", "head", seed=17)
    g = gpu_run(data, 1.5, "bf16", use_saved=use_saved)
    r = oracle_run(data, 1.5)
    print(use_saved, compare(g, r, label="decode fwd+bwd"))
