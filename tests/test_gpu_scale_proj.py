"""GPU parity of the ASEntmax scale projections (Sec. 4.1: beta = softplus(X w_beta), gamma = s tanh(X w_gamma))
and their gradients, through the C ABI, against the fp64 oracle on the same seeded inputs.

Tolerances, from the arithmetic: the forward accumulates E exact bf16 x (bf16 hi + lo) products in fp32, so a
pre-activation carries about E * 2^-24 of the sum of its terms' magnitudes, plus 2^-17 of each weight that the
hi + lo split drops: 1e-4 times max(1, largest |reference|) on beta and gamma covers E up to a few thousand.
The gradients are held to the attention's bar (5e-2 of the largest reference entry per tensor; dX is rounded to
bf16 on output)."""
import numpy as np
import pytest
import torch

from paper_2506_16640_amd import synth
from tests.parity_util import TOL_GRAD, rel_err

pytestmark = pytest.mark.gpu

TOL_ACT = 1e-4


def _inputs(B, N, E, H, dtype, seed, wscale=0.05):
    rng = np.random.Generator(np.random.Philox(key=[seed, 77]))
    X = rng.standard_normal((B, N, E)).astype(np.float32)
    if dtype == "bf16":
        X = synth.bf16_round(X)
    Wb = (wscale * rng.standard_normal((H, E))).astype(np.float32)
    Wg = (wscale * rng.standard_normal((H, E))).astype(np.float32)
    dbeta = rng.standard_normal((B, H, N)).astype(np.float32)
    dgamma = rng.standard_normal((B, H, N)).astype(np.float32)
    return X, Wb, Wg, dbeta, dgamma


def _run(B, N, E, H, dtype, s, seed=0, wscale=0.05):
    from oracle import oracle
    from paper_2506_16640_amd import binding
    X, Wb, Wg, dbeta, dgamma = _inputs(B, N, E, H, dtype, seed, wscale)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    x = torch.from_numpy(X).cuda().to(tdt)
    wb, wg = torch.from_numpy(Wb).cuda(), torch.from_numpy(Wg).cuda()
    beta, gamma = binding.scale_proj_fwd(x, wb, wg, s)
    rb, rg = oracle.scale_proj_fwd(X, Wb, Wg, s)
    eb = float(np.abs(beta.cpu().numpy() - rb).max()) if rb.size else 0.0
    eg = float(np.abs(gamma.cpu().numpy() - rg).max()) if rg.size else 0.0
    assert eb <= TOL_ACT * max(1.0, float(np.abs(rb).max()) if rb.size else 1.0) and eg <= TOL_ACT, (eb, eg)
    dx, dwb, dwg = binding.scale_proj_bwd(x, wb, wg, beta, gamma, torch.from_numpy(dbeta).cuda(),
                                          torch.from_numpy(dgamma).cuda(), s)
    torch.cuda.synchronize()
    r = oracle.scale_proj_bwd(X, Wb, Wg, s, dbeta, dgamma)
    errs = {"beta": eb, "gamma": eg}
    for name, got in (("dX", dx), ("dWb", dwb), ("dWg", dwg)):
        if r[name].size == 0:
            continue
        errs[name] = rel_err(got.float().cpu().numpy().astype(np.float64), r[name])
        assert errs[name] <= TOL_GRAD, (name, errs)
    # fp32 accumulation: the weight gradients are far inside the bar
    if r["dWb"].size and B * N > 0:
        assert errs["dWb"] <= 1e-4 and errs["dWg"] <= 1e-4, errs
    return errs


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("B,N,E,H", [(2, 300, 768, 12), (1, 77, 64, 3), (3, 129, 1040, 16), (1, 1, 16, 1),
                                     (2, 64, 2048, 5)])
def test_projection_parity_small(B, N, E, H, dtype):
    # ragged token counts (the last workgroup of either kernel is partly empty), every head-count bucket of the
    # backward (2H rounded up to 8, 16, 24, 32), an embedding width beyond one pass of the column loop
    print(B, N, E, H, dtype, _run(B, N, E, H, dtype, s=1.0, seed=B + N))


def test_projection_saturated_activations():
    # large weights drive softplus into its linear and exponential ends and tanh to +-s
    errs = _run(1, 200, 256, 4, "bf16", s=0.5, seed=9, wscale=1.0)
    print(errs)


def test_projection_empty_batch():
    from paper_2506_16640_amd import binding
    x = torch.zeros(0, 16, 64, dtype=torch.bfloat16, device="cuda")
    w = torch.ones(2, 64, device="cuda")
    beta, gamma = binding.scale_proj_fwd(x, w, w, 1.0)
    dx, dwb, dwg = binding.scale_proj_bwd(x, w, w, beta, gamma, beta, gamma, 1.0)
    torch.cuda.synchronize()
    assert beta.numel() == 0 and float(dwb.abs().max()) == 0.0 and float(dwg.abs().max()) == 0.0


def test_projection_full_size_feeds_attention():
    """The paper's language-model shape (hidden 768, 12 heads; App. G) at the headline batch: B = 4, n = 4096.
    The projections are checked against the oracle, then drive the attention in its per-query layout, whose
    d beta, d gamma go back through the projection backward -- the chain a training step runs."""
    from oracle import oracle
    from paper_2506_16640_amd import binding
    B, N, E, H = 4, 4096, 768, 12
    errs = _run(B, N, E, H, "bf16", s=1.0, seed=3)
    print("full size", errs)
    # chain on one batch element with the attention (oracle on 2 heads)
    X, Wb, Wg, _, _ = _inputs(1, 1024, E, H, "bf16", 5)
    data = synth.make_inputs(B=1, H=H, n=1024, d=64, dtype="bf16", scale="none", seed=5)
    x = torch.from_numpy(X).cuda().to(torch.bfloat16)
    wb, wg = torch.from_numpy(Wb).cuda(), torch.from_numpy(Wg).cuda()
    beta, gamma = binding.scale_proj_fwd(x, wb, wg, 1.0)
    q, k, v, do = (torch.from_numpy(data[n]).cuda().to(torch.bfloat16) for n in ("Q", "K", "V", "dO"))
    o, tau = binding.entmax_attn_fwd(q, k, v, alpha=1.5, beta=beta, gamma=gamma, logn_mode=1)
    dq, dk, dv, db, dg = binding.entmax_attn_bwd(q, k, v, o, do, tau, alpha=1.5, beta=beta, gamma=gamma, logn_mode=1)
    dx, dwb, dwg = binding.scale_proj_bwd(x, wb, wg, beta, gamma, db, dg, 1.0)
    torch.cuda.synchronize()
    rb, rg = oracle.scale_proj_fwd(X, Wb, Wg, 1.0)
    heads = [0, 7]
    sub = lambda a: a[:, heads]
    ro = oracle.attn_fwd(sub(data["Q"]), sub(data["K"]), sub(data["V"]), 1.5, beta=sub(rb), gamma=sub(rg), logn_mode=1)
    assert np.abs(o.float().cpu().numpy()[:, heads] - ro["O"]).max() <= 2e-2
    assert np.abs(tau.cpu().numpy()[:, heads] - ro["tau"]).max() <= 1e-3
    rbw = oracle.attn_bwd(sub(data["Q"]), sub(data["K"]), sub(data["V"]), sub(data["dO"]), 1.5, beta=sub(rb), gamma=sub(rg),
                          logn_mode=1)
    rp = oracle.scale_proj_bwd(X, Wb[heads], Wg[heads], 1.0, rbw["dbeta"], rbw["dgamma"])
    for name, got in (("dWb", dwb), ("dWg", dwg)):
        e = rel_err(got.cpu().numpy()[heads].astype(np.float64), rp[name])
        print("chain", name, e)
        assert e <= TOL_GRAD, (name, e)
