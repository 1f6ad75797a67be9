"""The entry point that allocates nothing (entmax_attn_fwd_noalloc: scratch in a buffer built into the library)
against entmax_attn_fwd with a caller-owned workspace, through the C ABI: same kernels, so O and tau must agree
to the bit, on two calls in a row of which the second is the smaller problem (the shared buffer then still holds
the first call's contents)."""
import numpy as np
import pytest
import torch

from paper_2506_16640_amd import synth
from tests.parity_util import TOL_O, TOL_TAU, oracle_run, to_dev

pytestmark = pytest.mark.gpu


def _both(binding, data, alpha, dtype, causal=True):
    q, k, v = (to_dev(data[n], dtype) for n in ("Q", "K", "V"))
    beta = None if data["beta"] is None else torch.from_numpy(data["beta"]).float().cuda()
    gamma = None if data["gamma"] is None else torch.from_numpy(data["gamma"]).float().cuda()
    kw = dict(alpha=alpha, beta=beta, gamma=gamma, delta=data["delta"], causal=causal)
    o_ref, tau_ref = binding.entmax_attn_fwd(q, k, v, **kw)
    out = torch.full_like(q, float("nan"))
    tau = torch.full(q.shape[:3], float("nan"), dtype=torch.float32, device=q.device)
    binding.entmax_attn_fwd_noalloc(q, k, v, out, tau, **kw)
    torch.cuda.synchronize()
    assert torch.equal(out, o_ref) and torch.equal(tau, tau_ref)
    r = oracle_run(data, alpha, causal=causal, bwd=False)
    assert np.abs(tau.cpu().numpy().astype(np.float64) - r["tau"]).max() <= TOL_TAU
    assert np.abs(out.float().cpu().numpy().astype(np.float64) - r["O"]).max() <= TOL_O


def test_noalloc_forward_matches_workspace_forward_two_calls():
    from paper_2506_16640_amd import binding
    binding.noalloc_init()
    assert binding.noalloc_scratch_bytes() >= 1 << 20
    big = synth.make_inputs(B=1, H=3, n=700, d=64, dtype="bf16", scale="head", seed=21, want_dO=False)
    small = synth.make_inputs(B=1, H=2, n=130, d=64, dtype="bf16", scale="head", seed=22, want_dO=False)
    _both(binding, big, 1.5, "bf16")
    _both(binding, small, 1.5, "bf16")  # smaller problem over the first call's leftovers
    # the split-key kernels of the decode shapes and the tiled kernel use the same buffer
    dec = synth.make_inputs(B=2, H=3, n=4, nk=3000, d=64, dtype="bf16", scale="head", seed=23, want_dO=False)
    _both(binding, dec, 1.5, "bf16")
    dense = synth.make_inputs(B=1, H=2, n=200, d=128, dtype="fp32", scale="dense", seed=24, want_dO=False)
    _both(binding, dense, 2.0, "fp32")
    _both(binding, small, 1.25, "bf16", causal=False)


def test_noalloc_forward_refuses_problems_beyond_its_buffer():
    from paper_2506_16640_amd import binding
    q = torch.zeros(4, 12, 4096, 64, dtype=torch.bfloat16, device="cuda")
    prm = binding.make_params(q, q, 1.5, 1.0, True, None, 0)
    assert binding.workspace_bytes(prm, 0) > binding.noalloc_scratch_bytes()
    out, tau = torch.empty_like(q), torch.empty(4, 12, 4096, dtype=torch.float32, device="cuda")
    with pytest.raises(binding.EntmaxAttnError) as e:
        binding.entmax_attn_fwd_noalloc(q, q, q, out, tau)
    assert e.value.code == -6
