"""GPU parity: the HIP library (through the C ABI) against the fp64 CPU oracle,
element by element on the same seeded inputs.  Bars: max-abs 2e-2 on O, 1e-3 on
tau, 5e-2 relative (max|diff|/max|ref|) on every gradient tensor."""
import math

import numpy as np
import pytest

from paper_2506_16640_amd import synth
from tests.parity_util import compare, gpu_run, oracle_run

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=[(0, False), (0, True), (1, False)], ids=["auto", "auto-saved", "tiled"])
def forward_path(request):
    """Every case runs three times: with the automatic path (list kernels, tiled fallback) where the backward
    rebuilds the supports itself, the same with the forward's lists handed to the backward, and with the
    tiled kernels alone."""
    from tests import parity_util
    parity_util.DEFAULT_PATH, parity_util.DEFAULT_SAVED = request.param
    yield request.param[0]
    parity_util.DEFAULT_PATH, parity_util.DEFAULT_SAVED = 0, False


def _case(B, H, nq, nk, d, dtype, scale, seed=0, planted=0.0):
    return synth.make_inputs(B=B, H=H, n=nq, nk=nk, d=d, dtype=dtype, scale=scale, seed=seed,
                             planted=planted if nq == nk else 0.0)


def test_c1_fp32_single_head():
    data = synth.make_config("c1")
    g = gpu_run(data, 1.5, "fp32")
    r = oracle_run(data, 1.5)
    errs = compare(g, r, label="c1")
    print("c1 errors", errs)


@pytest.mark.parametrize("alpha", [1.5, 2.0, 1.25, 1.4])
@pytest.mark.parametrize("d", [64, 128])
def test_bf16_small_causal(alpha, d):
    # several 128-row blocks, several key tiles, ragged tail (n = 300 is no multiple of 32)
    data = _case(2, 3, 300, 300, d, "bf16", "head", seed=1)
    g = gpu_run(data, alpha, "bf16")
    r = oracle_run(data, alpha)
    print(alpha, d, compare(g, r, label=f"a{alpha} d{d}"))


@pytest.mark.parametrize("alpha", [1.5, 2.0, 1.25, 1.7])
def test_bf16_dense_regime(alpha):
    # delta = 0, gamma = -1/2: nearly every key stays in the support
    data = _case(1, 2, 257, 257, 64, "bf16", "dense", seed=2)
    g = gpu_run(data, alpha, "bf16")
    r = oracle_run(data, alpha)
    assert r["support"].mean() > (20 if alpha < 1.6 else 4)
    print(alpha, compare(g, r, label=f"dense a{alpha}"))


def test_dense_blocks_leave_the_list_kernel_early(forward_path):
    """Rows that keep most of their keys (delta = 0, gamma = -1/2) are recognised on the list kernel's first key
    tile, and the block goes to the tiled kernel after two tiles instead of a full sweep: same results, and the
    list kernel computes only a fraction of the visible tiles."""
    if forward_path == 1:
        pytest.skip("the list kernel is the subject")
    n = 1536
    data = _case(1, 2, n, n, 64, "bf16", "dense", seed=4)
    g = gpu_run(data, 1.5, "bf16", stats=True)
    r = oracle_run(data, 1.5)
    st = g["stats"]
    print(compare(g, r, label="dense early exit"), {k: v for k, v in st.items() if v})
    assert st["fwd_sparse_blocks"] == 0 and st["fwd_blocks"] > 0
    # 12 blocks a head: the first has one tile and makes no verdict, the others stop after two tiles (8 blocks of 32 keys)
    assert st["fwd_list_qk"] <= 2 * 4 * (4 + 11 * 8) + 64, st


@pytest.mark.parametrize("causal,nq,nk", [(True, 273, 273), (False, 130, 337), (True, 448, 448), (False, 64, 65),
                                           (True, 100, 1100)])
@pytest.mark.parametrize("alpha", [1.5, 1.25])
def test_split_blocks_take_key_tiles_in_pairs(causal, nq, nk, alpha):
    """A few dense blocks run split in the tiled forward, whose K-only sweeps at D = 64 stage two 64-key tiles per
    step: odd tile counts (the second tile of the last step lies beyond the sweep), a ragged last tile, a single
    tile, and a causal window that ends inside a pair."""
    data = _case(1, 2, nq, nk, 64, "bf16", "dense", seed=11)
    g = gpu_run(data, alpha, "bf16", causal=causal, stats=True)
    r = oracle_run(data, alpha, causal=causal)
    st = g["stats"]
    print(causal, nq, nk, alpha, compare(g, r, label=f"split pairs {causal} {nq} {nk} a{alpha}"), {k: v for k, v in st.items() if v})
    assert st["fwd_blocks"] > 0  # the tiled kernel did run


@pytest.mark.parametrize("n", [256, 300])
def test_many_heads_take_query_blocks_one_by_one(n):
    """From 128 causal pairs of query blocks up to 767 the forward's list kernel runs one block per workgroup
    (B 8, H 16: 128 heads of two or three blocks); smaller launches, as in the other cases here, keep the pairs."""
    data = _case(8, 16, n, n, 64, "bf16", "head", seed=21, planted=0.05)
    g = gpu_run(data, 1.5, "bf16", stats=True)
    r = oracle_run(data, 1.5)
    print(n, compare(g, r, label=f"unpaired n{n}"), {k: v for k, v in g["stats"].items() if v})


@pytest.mark.parametrize("scale,alpha,dtype", [("none", 1.5, "bf16"), ("none", 1.7, "bf16"), ("head", 1.25, "bf16"),
                                               ("none", 1.7, "fp32")])
def test_moderate_support(scale, alpha, dtype):
    # supports of 5..40 keys per row: long candidate lists, some half rows beyond the list capacities
    data = _case(1, 2, 768, 768, 64, dtype, scale, seed=7)
    g = gpu_run(data, alpha, dtype, stats=True)
    r = oracle_run(data, alpha)
    print(scale, alpha, dtype, compare(g, r, label=f"moderate {scale} a{alpha}"), {k: v for k, v in g["stats"].items() if v})


@pytest.mark.parametrize("causal,nq,nk", [(False, 200, 333), (True, 200, 333), (True, 333, 200), (False, 129, 64),
                                           (True, 1, 1), (True, 1, 70), (True, 33, 33)])
@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_ragged_and_rectangular(causal, nq, nk, dtype):
    data = _case(1, 2, nq, nk, 64, dtype, "head", seed=3)
    g = gpu_run(data, 1.5, dtype, causal=causal)
    r = oracle_run(data, 1.5, causal=causal)
    print(causal, nq, nk, dtype, compare(g, r, label=f"rect {causal} {nq} {nk} {dtype}"))


@pytest.mark.parametrize("scale,logn_mode", [("none", 0), ("head", 1), ("query", 0), ("query", 1)])
def test_scale_layouts(scale, logn_mode):
    data = _case(2, 2, 192, 192, 64, "bf16", scale, seed=4)
    g = gpu_run(data, 1.5, "bf16", logn_mode=logn_mode)
    r = oracle_run(data, 1.5, logn_mode=logn_mode)
    print(scale, logn_mode, compare(g, r, label=f"scale {scale} {logn_mode}"))


def test_negative_and_zero_scale():
    data = _case(1, 3, 160, 160, 64, "bf16", "head", seed=5)
    data["beta"] = np.array([-0.8, 0.0, 0.5], dtype=np.float32)  # head 0: negative multiplier, head 1: scale = delta = 0
    data["gamma"] = np.array([1.0, 1.0, 1.0], dtype=np.float32)
    data["delta"] = 0.0
    g = gpu_run(data, 1.5, "bf16")
    r = oracle_run(data, 1.5)
    print(compare(g, r, label="neg/zero scale"))


def test_strided_bnhd_layout():
    data = _case(2, 3, 150, 150, 64, "bf16", "head", seed=6)
    g = gpu_run(data, 1.5, "bf16", layout_bnhd=True)
    r = oracle_run(data, 1.5)
    print(compare(g, r, label="bnhd"))


@pytest.mark.parametrize("alpha", [1.25, 1.5, 2.0])
def test_two_level_closed_form_on_gpu(alpha):
    """Two-level lemma realised through Q and K: tau = (alpha-1) M - k^-(alpha-1), p = 1/k, so
    every output row is the mean of the values of the k high keys (non-causal)."""
    n, d, k = 320, 64, 5
    rng = np.random.default_rng(0)
    hi = rng.choice(n, size=k, replace=False)
    gap = 1.0 / (alpha - 1.0) + 0.5
    Q = np.zeros((1, 1, n, d), np.float32)
    Q[..., 0] = 2.0
    K = np.zeros((1, 1, n, d), np.float32)
    K[0, 0, hi, 0] = gap * math.sqrt(d) / 2.0
    V = synth.bf16_round(rng.standard_normal((1, 1, n, d)).astype(np.float32))
    data = dict(Q=Q, K=K, V=V, beta=None, gamma=None, delta=1.0)
    g = gpu_run(data, alpha, "bf16", causal=False, bwd=False)
    assert np.abs(g["tau"] - ((alpha - 1) * gap - k ** (-(alpha - 1)))).max() < 1e-3
    assert np.abs(g["O"] - V[0, 0, hi].astype(np.float64).mean(0)).max() < 2e-2


def _mid_band_case(alpha, nq=128, nk=64, d=64):
    """Two-level logits (the two-level lemma of the appendix) plus a middle band: 10 equal top keys carry the
    whole mass, 50 more keys sit above the lower bound of the threshold that the list kernel can derive but
    below the threshold itself: every row lists 60 candidates for a support of 10 (non-causal)."""
    if alpha == 1.5:
        s_top, s_mid, s_low = 2.0, 1.0, -10.0  # tau = M/2 - 10^-1/2: support needs s > M - 0.63; candidates s > M - 1.41
    else:
        s_top, s_mid, s_low = 4.0, 1.0, -16.0  # tau = M/4 - 10^-1/4: support needs s > M - 2.25; candidates s > M - 4
    rng = np.random.default_rng(3)
    level = np.full(nk, s_low)
    # lane half hh of a row holds the keys with (j % 8) // 4 == hh: 5 top and 25 middle keys in each half
    for hh in (0, 1):
        keys = np.array([j for j in range(nk) if (j % 8) // 4 == hh])
        rng.shuffle(keys)
        level[keys[:5]] = s_top
        level[keys[5:30]] = s_mid
    Q = np.zeros((1, 2, nq, d), np.float32)
    Q[..., 0] = 2.0
    # keys differ in the features the queries do not look at (so that dQ is not identically zero)
    K = synth.bf16_round(rng.standard_normal((1, 2, nk, d)).astype(np.float32))
    K[..., 0] = level * math.sqrt(d) / 2.0  # logits <q,k>/sqrt(d) = level, exactly representable in bf16
    V = synth.bf16_round(rng.standard_normal((1, 2, nk, d)).astype(np.float32))
    dO = synth.bf16_round(rng.standard_normal((1, 2, nq, d)).astype(np.float32))
    return dict(Q=Q, K=K, V=V, dO=dO, beta=None, gamma=None, delta=1.0), s_top


@pytest.mark.parametrize("alpha", [1.5, 1.25])
def test_candidates_far_beyond_support(alpha):
    """With 60 candidates for a support of 10 per row the forward's per-key candidate counts add up to more than
    the backward's key-major arrays hold per head; the backward must notice and must not drop or misplace
    entries (all three path variants run this)."""
    data, s_top = _mid_band_case(alpha)
    g = gpu_run(data, alpha, "bf16", causal=False, stats=True)
    r = oracle_run(data, alpha, causal=False)
    assert int(r["support"].min()) == int(r["support"].max()) == 10
    assert np.abs(g["tau"] - ((alpha - 1) * s_top - 10.0 ** (-(alpha - 1)))).max() < 1e-3
    print(alpha, compare(g, r, label=f"mid band a{alpha}"), {k: v for k, v in g["stats"].items() if v})


@pytest.mark.parametrize("roomy", [False, True])
def test_saved_pool_runs_out(roomy):
    """The `saved` buffer packs the rows' support lists into a pool sized for six entries per row on average; a
    32-row group reserves its piece by its candidate counts (at most 16 per half row).  Here every half row lists
    30 candidates, so a buffer of the size the library asks for cannot hold every group: the blocks that find the
    pool used up must go to the backward's tiled kernels, and a roomier buffer must keep them all on the lists.
    Either way the gradients match the oracle."""
    data, _ = _mid_band_case(1.5)
    g = gpu_run(data, 1.5, "bf16", causal=False, stats=True, path=0, use_saved=True, saved_factor=4 if roomy else 1)
    r = oracle_run(data, 1.5, causal=False)
    st = g["stats"]
    print(roomy, compare(g, r, label=f"saved pool roomy={roomy}"), {k: v for k, v in st.items() if v})
    if roomy:
        assert st["bwd_support"] == 2 * 128 * 10 and st["bwd_dq_tiles"] == 0, st
    else:
        assert st["bwd_dq_tiles"] > 0, st


def test_hot_keys_beyond_the_forward_numbering():
    """The forward numbers each support entry among its key's entries (the backward places it in the key's segment
    by that number), in 10 bits next to the key index.  Here ten keys are in the support of all 1300 rows: their
    entries beyond the 1023rd take their place from the backward's cursor instead.  With the forward's lists
    (roomy buffer, so that every block stays on the list path) and without."""
    data, _ = _mid_band_case(1.5, nq=1300)
    r = oracle_run(data, 1.5, causal=False)
    for use_saved in (True, False):
        g = gpu_run(data, 1.5, "bf16", causal=False, stats=True, path=0, use_saved=use_saved, saved_factor=8)
        st = g["stats"]
        print(use_saved, compare(g, r, label=f"hot keys saved={use_saved}"), {k: v for k, v in st.items() if v})
        assert st["bwd_support"] == 2 * 1300 * 10 and st["bwd_dq_tiles"] == 0, st


def test_long_sequence_skips_blocks_in_the_second_sweep():
    """From 16384 keys on, the list kernel's first sweep keeps one bit per (32-row group, 32-key block) and the
    second sweep computes only the marked blocks.  Ragged length beyond the range the bits cover is not needed
    for that (the full-size n = 32768 tests cover it); here every row of one head is compared, and two rows get a
    late maximum preceded by near ties early in the sequence, which must all stay on their lists."""
    n = 16384 + 37
    data = _case(1, 1, n, n, 64, "bf16", "head", seed=5, planted=0.05)
    data["beta"][:] = 1.0
    data["gamma"][:] = 1.0
    q, k = data["Q"][0, 0], data["K"][0, 0]
    for early, row in ((3, n - 1), (9, n - 700)):
        unit = q[row] / np.linalg.norm(q[row]) ** 2
        for key in (early, early + 37, row - 5):  # three equal logits <q,k>/sqrt(d) (up to bf16 rounding) well above the background
            k[key] = synth.bf16_round((5.6 * 8.0 * unit).astype(np.float32))
    g = gpu_run(data, 1.5, "bf16", stats=True)
    r = oracle_run(data, 1.5)
    st = g["stats"]
    print(compare(g, r, label="long sequence"), {k_: v for k_, v in st.items() if v})
    for row in (n - 1, n - 700):
        assert r["support"][0, 0, row] >= 3
    if st["fwd_sparse_blocks"] > 0:  # (the tiled variant of this test makes no lists)
        assert st["fwd_list_qk"] < 2 * st["fwd_tiles_visible"] * 0.9, st  # the second sweep skipped blocks


@pytest.mark.parametrize("n,path", [(30720 + 300, 0), (65536 + 200, 2)])
def test_block_bits_end_before_the_sequence(n, path, forward_path):
    """The block bits of the long-sequence list kernels cover 30720 keys (one block per workgroup) or 65536 keys
    (two blocks per workgroup, forced here with params.path = 2); key blocks beyond that range must always be
    computed in the second sweep.  One head, forward, every row against the oracle."""
    if forward_path == 1:
        pytest.skip("the list kernels are the subject")
    data = synth.make_inputs(B=1, H=1, n=n, d=64, dtype="bf16", scale="head", planted=0.05, seed=17, want_dO=False)
    g = gpu_run(data, 1.5, "bf16", bwd=False, stats=True, path=path)
    r = oracle_run(data, 1.5, bwd=False)
    st = g["stats"]
    print(n, path, compare(g, r, bwd=False, label=f"bits range n{n}"), {k_: v for k_, v in st.items() if v})
    assert st["fwd_sparse_blocks"] == (n + 127) // 128 and st["fwd_list_qk"] < 2 * st["fwd_tiles_visible"], st


@pytest.mark.parametrize("causal,nq,nk,alpha,scale", [(True, 300, 300, 1.5, "head"), (True, 641, 641, 1.5, "head"),
                                                      (False, 200, 333, 1.5, "head"), (True, 333, 200, 2.0, "head"),
                                                      (True, 200, 333, 1.25, "head"), (True, 1, 70, 1.5, "head"),
                                                      (True, 520, 520, 1.7, "none"), (True, 257, 257, 1.5, "dense")])
@pytest.mark.parametrize("d", [64, 128])
def test_long_sequence_kernels_at_small_sizes(causal, nq, nk, alpha, scale, d):
    """params.path = 2 runs the list kernels made for long sequences at any size: at D = 64 the kernel that takes
    two adjacent query blocks per workgroup (odd numbers of blocks end on a single one; 641 rows are five blocks
    and a ragged sixth), at D = 128 the one-block kernel with the block bits.  Same bar as everywhere; the
    backward gets the forward's lists."""
    data = _case(2, 3, nq, nk, d, "bf16", scale, seed=13)
    g = gpu_run(data, alpha, "bf16", causal=causal, path=2, use_saved=True, stats=True)
    r = oracle_run(data, alpha, causal=causal)
    print(causal, nq, nk, alpha, scale, d, compare(g, r, label=f"long kernels {causal} {nq} {nk} a{alpha} {scale} d{d}"),
          {k: v for k, v in g["stats"].items() if v})


def test_empty_inputs():
    import torch
    from paper_2506_16640_amd import binding
    q = torch.zeros(1, 2, 40, 64, dtype=torch.bfloat16, device="cuda")
    k = torch.zeros(1, 2, 0, 64, dtype=torch.bfloat16, device="cuda")
    o, tau = binding.entmax_attn_fwd(q, k, k.clone(), causal=False)
    assert float(o.float().abs().max()) == 0.0 and float(tau.abs().max()) == 0.0
    dq, dk, dv, _, _ = binding.entmax_attn_bwd(q, k, k.clone(), o, torch.ones_like(q), tau, causal=False)
    assert float(dq.float().abs().max()) == 0.0 and dk.numel() == 0
    q0 = torch.zeros(1, 2, 0, 64, dtype=torch.bfloat16, device="cuda")
    k1 = torch.randn(1, 2, 50, 64, device="cuda").to(torch.bfloat16)
    o0, tau0 = binding.entmax_attn_fwd(q0, k1, k1.clone(), causal=False)
    assert o0.numel() == 0
    dq, dk, dv, _, _ = binding.entmax_attn_bwd(q0, k1, k1.clone(), o0, q0.clone(), tau0, causal=False)
    torch.cuda.synchronize()
    assert float(dk.float().abs().max()) == 0.0 and float(dv.float().abs().max()) == 0.0


def test_saved_from_tiled_forward_sends_backward_to_tiled_kernels():
    # a forward that made no lists (path 1) marks every block in `saved`: the backward, although on the automatic
    # path, must then take the tiled kernels for every head and still match the oracle
    import torch
    from paper_2506_16640_amd import binding
    from tests.parity_util import to_dev
    data = _case(1, 2, 300, 300, 64, "bf16", "head", seed=11)
    q, k, v, do = (to_dev(data[n], "bf16") for n in ("Q", "K", "V", "dO"))
    beta, gamma = (torch.from_numpy(data[n]).float().cuda() for n in ("beta", "gamma"))
    kw = dict(alpha=1.5, beta=beta, gamma=gamma, delta=data["delta"], causal=True)
    saved = binding.new_saved(binding.make_params(q, k, 1.5, data["delta"], True, beta, 0, 0))
    o, tau = binding.entmax_attn_fwd(q, k, v, path=1, saved=saved, **kw)
    st = binding.new_stats()
    dq, dk, dv, db, dg = binding.entmax_attn_bwd(q, k, v, o, do, tau, path=0, saved=saved, stats=st, **kw)
    torch.cuda.synchronize()
    sd = binding.stats_dict(st)
    assert sd["bwd_support"] == 0 and sd["bwd_dq_tiles"] > 0  # no list work, tiled work
    r = oracle_run(data, 1.5)
    g = {"O": o, "tau": tau, "dQ": dq, "dK": dk, "dV": dv, "dbeta": db, "dgamma": dg}
    g = {n: t.float().cpu().numpy().astype(np.float64) for n, t in g.items()}
    print(compare(g, r, label="saved from tiled forward"))


def test_bitwise_reproducible():
    data = _case(1, 2, 300, 300, 64, "bf16", "head", seed=8)
    a = gpu_run(data, 1.5, "bf16")
    b = gpu_run(data, 1.5, "bf16")
    # every key has fewer than 64 entries here, so the list path sums in a fixed order too
    for name in ("O", "tau", "dQ", "dK", "dV", "dbeta", "dgamma"):
        assert np.array_equal(a[name], b[name]), name


@pytest.mark.parametrize("alpha,dtype", [(1.5, "bf16"), (1.25, "bf16"), (1.5, "fp32")])
def test_backward_splits_a_head_between_the_paths(alpha, dtype, forward_path):
    """One head whose early query blocks have short supports and whose late blocks have long ones (a scale that
    shrinks along the sequence): the list kernels take the former, the tiled kernels the latter, and dK, dV are
    the sum of both paths' contributions."""
    n = 1024
    data = _case(1, 1, n, n, 64, dtype, "query", seed=21)
    ramp = np.linspace(3.0, 0.05, n, dtype=np.float32)
    data["beta"] = (data["beta"] * 0 + ramp[None, None, :]).astype(np.float32)
    data["gamma"] = (data["gamma"] * 0 + 1.0).astype(np.float32)
    data["delta"] = 0.0
    g = gpu_run(data, alpha, dtype, stats=True)
    r = oracle_run(data, alpha)
    print(alpha, dtype, compare(g, r, label=f"split head a{alpha} {dtype}"), {k: v for k, v in g["stats"].items() if v})
    if forward_path == 0:
        st = g["stats"]
        assert st["bwd_support"] > 0 and st["bwd_dq_tiles"] > 0, st  # both paths worked on this one head


@pytest.mark.parametrize("dtype,d,alpha", [("bf16", 64, 1.5), ("bf16", 128, 1.25), ("fp32", 64, 2.0), ("bf16", 64, 1.7)])
@pytest.mark.parametrize("heads", [3, 70])
def test_tiled_forward_shares_blocks_out_both_ways(dtype, d, alpha, heads, forward_path):
    """Dense rows send every block to the tiled forward.  With 3 heads x 5 blocks it runs four workgroups to a
    block (the waves of a workgroup share out the keys of one 32-row group and combine maxima, threshold sums and
    outputs); with 70 x 5 = 350 blocks, more than the limit for that, it runs the blocks whole, in pairs.  Both
    against the oracle, forward only (the backward does not depend on how the forward was shared out)."""
    n = 577  # five blocks, a ragged last one; 18.03 key blocks of 32: the split's wave shares differ
    data = _case(1, heads, n, n, d, dtype, "dense", seed=31)
    g = gpu_run(data, alpha, dtype, bwd=False, stats=True)
    r = oracle_run(data, alpha, bwd=False)
    print(dtype, d, alpha, heads, compare(g, r, bwd=False, label=f"share-out {dtype} d{d} a{alpha} H{heads}"))
    if forward_path == 0 and alpha <= 1.5:
        assert g["stats"]["fwd_blocks"] == heads * 5, g["stats"]  # every block took the tiled kernel


def test_randomised_small_configurations():
    """Forty seeded draws over the whole parameter space of the entry points (shapes with ragged tails, both
    element types and head dimensions, every alpha path, scale layouts, log-n modes, causal or not, distance bias
    in both placements): each against the oracle, with the bars of this file."""
    rng = np.random.Generator(np.random.Philox(key=[2024, 5]))
    for case in range(40):
        nq = int(rng.integers(1, 400))
        nk = nq if rng.random() < 0.5 else int(rng.integers(1, 400))
        d = int(rng.choice([64, 128]))
        dtype = str(rng.choice(["bf16", "fp32"]))
        alpha = float(rng.choice([1.5, 2.0, 1.25, 1.1, 1.4, 1.75]))
        scale = str(rng.choice(["none", "head", "query", "dense"]))
        causal = bool(rng.random() < 0.7)
        logn_mode = int(rng.integers(0, 2))
        H = int(rng.integers(1, 4))
        B = int(rng.integers(1, 3))
        data = _case(B, H, nq, nk, d, dtype, scale, seed=100 + case)
        slopes, bias_mode = None, 0
        if rng.random() < 0.4:
            slopes = (2.0 ** -rng.integers(0, 8, size=H)).astype(np.float32) * (rng.random(H) < 0.7)
            slopes = slopes.astype(np.float32)
            bias_mode = int(rng.integers(0, 2))
        label = f"case {case}: B{B} H{H} nq{nq} nk{nk} d{d} {dtype} a{alpha} {scale} causal{causal} logn{logn_mode} bias{bias_mode} {slopes}"
        print(label, flush=True)
        g = gpu_run(data, alpha, dtype, causal=causal, logn_mode=logn_mode, slopes=slopes, bias_mode=bias_mode)
        r = oracle_run(data, alpha, causal=causal, logn_mode=logn_mode, slopes=slopes, bias_mode=bias_mode)
        compare(g, r, label=label)
