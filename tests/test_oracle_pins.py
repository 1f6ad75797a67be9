"""Pins for the fp64 CPU oracle: everything here checks oracle/ against facts
fixed by the paper or by mathematics, never against the oracle's own formulas
and never against the GPU path.

Citations are to the paper's sections / equations / lemmas.
"""
import itertools
import math
import os

import numpy as np
import pytest
from scipy.optimize import brentq

from oracle import oracle

ALPHAS = [1.25, 1.5, 1.75, 2.0]
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split("=")
            vals[k.strip()] = float(v)
    return vals


# ---------------------------------------------------------------- row map ---


def sparsemax_textbook(z):
    """Martins & Astudillo's sparsemax: k = max{k : 1 + k z_(k) > sum_{j<=k} z_(j)},
    tau = (sum_{j<=k} z_(j) - 1)/k.  (Sec. 2.2: alpha = 2 is sparsemax.)"""
    zs = np.sort(z)[::-1]
    cs = np.cumsum(zs)
    ks = np.arange(1, len(z) + 1)
    k = ks[1 + ks * zs > cs].max()
    tau = (cs[k - 1] - 1.0) / k
    return np.maximum(z - tau, 0.0), tau


@pytest.mark.parametrize("seed", range(5))
@pytest.mark.parametrize("n,spread", [(1, 1.0), (2, 0.3), (7, 1.0), (64, 0.1), (64, 3.0), (1000, 1.0)])
def test_alpha2_is_sparsemax(seed, n, spread):
    z = np.random.default_rng(seed).normal(size=n) * spread
    p, tau, sup = oracle.entmax_row(z, 2.0)
    pref, tref = sparsemax_textbook(z)
    np.testing.assert_allclose(p, pref, atol=1e-13)
    assert abs(tau - tref) < 1e-13
    assert sup == int((pref > 0).sum())


@pytest.mark.parametrize("alpha", [1.1, 1.25, 1.5, 1.75, 2.0])
@pytest.mark.parametrize("n,k", [(5, 1), (16, 3), (300, 7), (300, 300 - 1)])
def test_two_level_closed_form(alpha, n, k):
    """Two-level lemma: k logits at M, n-k at m; if M - m >= k^-(alpha-1)/(alpha-1) then
    tau = (alpha-1) M - k^-(alpha-1), p = 1/k on the high tokens and exactly 0 elsewhere."""
    a1 = alpha - 1.0
    gap_min = k ** (-a1) / a1
    rng = np.random.default_rng(n * 31 + k)
    for gap in (gap_min, gap_min * 1.5, gap_min + 10.0):
        M = rng.normal()
        z = np.full(n, M - gap)
        hi = rng.choice(n, size=k, replace=False)
        z[hi] = M
        p, tau, sup = oracle.entmax_row(z, alpha)
        assert abs(tau - (a1 * M - k ** (-a1))) < 1e-12
        mask = np.zeros(n, bool)
        mask[hi] = True
        np.testing.assert_allclose(p[mask], 1.0 / k, rtol=0, atol=1e-12)
        if gap > gap_min:
            assert np.all(p[~mask] == 0.0) and sup == k
        else:  # low tokens sit on the threshold up to rounding
            assert np.all(p[~mask] < 1e-12)


def test_two_level_below_gap_is_dense():
    """Same lemma, other side: with a smaller gap the low tokens keep mass."""
    alpha, n, k = 1.5, 20, 4
    gap = 0.5 * k ** (-(alpha - 1)) / (alpha - 1)
    z = np.zeros(n)
    z[:k] = gap
    p, _, sup = oracle.entmax_row(z, alpha)
    assert sup == n and np.all(p > 0) and abs(p.sum() - 1) < 1e-13


def test_paper_worked_example_sparsemax():
    """Counterexample to representational collapse (appendix, 'Specific counterexample'):
    alpha=2, logits [0,..,0,.5,.5] -> [0,..,0,1/2,1/2]; logits [0,..,0,.5] -> dense with
    p_n -> 0.5; L1 gap of the outputs -> 0.354."""
    g = _read_golden("sparsemax_worked_example.txt")
    for n in (3, 10, 1000):
        z = np.full(n + 1, g["b"])
        z[-2:] = g["phi"]
        p, tau, sup = oracle.entmax_row(z, g["alpha"])
        assert np.all(p[:-2] == g["sparse_head"])  # the zeros sit exactly on the threshold
        assert p[-2] == g["sparse_tail_0"] and p[-1] == g["sparse_tail_1"] and sup == 2
        zd = np.full(n, g["b"])
        zd[-1] = g["phi"]
        pd, _, supd = oracle.entmax_row(zd, g["alpha"])
        assert supd == n and np.all(pd[:-1] > 0) and np.all(pd[:-1] < pd[-1]) and pd[-1] < 1
        # by hand: tau = (phi - 1)/n, so p_b = (1-phi)/n and p_n = phi + (1-phi)/n
        assert abs(pd[-1] - (g["phi"] + (1 - g["phi"]) / n)) < 1e-14
        assert abs(pd[0] - (1 - g["phi"]) / n) < 1e-14
    assert abs(pd[-1] - g["p_star"]) < 1e-3
    # outputs of the last token: values are 0 for the n-1 first tokens and sqrt(phi) for v_a
    va = math.sqrt(g["phi"])
    out_dense = pd[-1] * va
    out_sparse = (p[-1] + p[-2]) * va
    assert abs(abs(out_dense - out_sparse) - g["l1_gap_limit"]) < 1e-3


def brute_force_entmax(z, alpha):
    """Enumerate every non-empty support, solve sum_{j in S}((alpha-1) z_j - tau)^r = 1 on it,
    keep the support consistent with its tau (it is unique)."""
    a1 = alpha - 1.0
    r = 1.0 / a1
    n = len(z)
    found = []
    for size in range(1, n + 1):
        for S in itertools.combinations(range(n), size):
            y = a1 * z[list(S)]
            top = y.min()
            f = lambda t: np.sum((y - t) ** r) - 1.0  # noqa: E731
            if f(top) >= 0:  # even with the smallest member at zero mass there is too much
                continue
            tau = brentq(f, top - 1.0 - 1e-9, top, xtol=1e-15, rtol=1e-15, maxiter=500)
            rest = [j for j in range(n) if j not in S]
            if all(a1 * z[j] <= tau for j in rest) and np.all(y > tau):
                found.append((S, tau))
    assert len(found) == 1
    S, tau = found[0]
    p = np.zeros(n)
    p[list(S)] = (a1 * z[list(S)] - tau) ** r
    return p, tau


@pytest.mark.parametrize("alpha", [1.2, 1.5, 1.75, 2.0])
@pytest.mark.parametrize("seed", range(6))
def test_brute_force_support_enumeration(alpha, seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(2, 7))
    z = rng.normal(size=n) * rng.choice([0.3, 1.0, 3.0])
    p, tau, _ = oracle.entmax_row(z, alpha)
    pb, tb = brute_force_entmax(z, alpha)
    np.testing.assert_allclose(p, pb, atol=1e-10)
    assert abs(tau - tb) < 1e-10


def test_alpha_to_one_is_softmax():
    """Sec. 2.2 / App. A: alpha -> 1+ recovers softmax; the gap shrinks about linearly in alpha-1."""
    z = np.random.default_rng(3).normal(size=12)
    sm = np.exp(z - z.max())
    sm /= sm.sum()
    errs = []
    for alpha in (1.1, 1.05, 1.025, 1.0125):
        p, _, _ = oracle.entmax_row(z, alpha)
        errs.append(np.abs(p - sm).max())
    assert errs[-1] < 1.5e-2
    for a, b in zip(errs[:-1], errs[1:]):
        assert 0.45 < b / a < 0.56  # halving alpha-1 about halves the error


@pytest.mark.parametrize("alpha", ALPHAS + [1.1])
@pytest.mark.parametrize("seed", range(4))
def test_row_invariants(alpha, seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 400))
    z = rng.normal(size=n) * rng.choice([0.2, 1.0, 5.0])
    p, tau, sup = oracle.entmax_row(z, alpha)
    a1 = alpha - 1.0
    assert np.all(p >= 0) and abs(p.sum() - 1.0) < 1e-12
    # support <=> threshold (App. A: entries with (alpha-1) z <= tau are exactly zero)
    assert np.array_equal(p > 0, a1 * z > tau) and sup == int((p > 0).sum())
    # bracket of App. A eq. (bounds), un-normalised: (a-1)max - 1 <= tau <= (a-1)max - n^(1-alpha)
    assert a1 * z.max() - 1.0 - 1e-12 <= tau <= a1 * z.max() - n ** (1 - alpha) + 1e-12
    # ratio on the support (NoPE analysis): p_j/p_i = ((z_j - tau')/(z_i - tau'))^(1/(alpha-1))
    idx = np.flatnonzero(p > 0)
    if len(idx) >= 2:
        i, j = idx[0], idx[-1]
        tp = tau / a1
        assert abs(p[j] / p[i] - ((z[j] - tp) / (z[i] - tp)) ** (1 / a1)) < 1e-9 * max(1.0, p[j] / p[i])
    # shift: entmax(z + c) = entmax(z), tau moves by (alpha-1) c
    p2, tau2, _ = oracle.entmax_row(z + 2.5, alpha)
    np.testing.assert_allclose(p2, p, atol=1e-12)
    assert abs(tau2 - tau - a1 * 2.5) < 1e-12
    # generic fixed-support solve agrees with the alpha = 1.5 / 2 closed forms
    p3, tau3, _ = oracle.entmax_row(z, alpha, force_generic=True)
    np.testing.assert_allclose(p3, p, atol=1e-12)
    assert abs(tau3 - tau) < 1e-12


@pytest.mark.parametrize("alpha", ALPHAS)
def test_non_vanishing_lemma(alpha):
    """Non-vanishing attention lemma: appending a logit b <= tau/(alpha-1) leaves every
    probability unchanged; any appended logit can only raise tau and lower p_n."""
    rng = np.random.default_rng(11)
    z = rng.normal(size=30)
    p, tau, _ = oracle.entmax_row(z, alpha)
    b_max = tau / (alpha - 1.0)
    for b in (b_max, b_max - 0.1, b_max - 50.0):
        ze = np.concatenate([z[:-1], [b], z[-1:]])
        pe, taue, _ = oracle.entmax_row(ze, alpha)
        np.testing.assert_allclose(np.delete(pe, -2), p, atol=1e-13)
        assert pe[-2] < 1e-13 and abs(taue - tau) < 1e-13
    for b in (b_max + 0.05, b_max + 1.0, z.max() + 3.0):
        ze = np.concatenate([z[:-1], [b], z[-1:]])
        pe, taue, _ = oracle.entmax_row(ze, alpha)
        assert taue > tau and pe[-1] <= p[-1] + 1e-15 and pe[-2] > 0


def tsallis_objective(p, z, alpha):
    return p @ z + np.sum(p - p**alpha) / (alpha * (alpha - 1.0))


@pytest.mark.parametrize("alpha", ALPHAS)
def test_variational_optimality(alpha):
    """App. A: entmax is the maximiser of p.z + H_alpha(p) (Tsallis entropy) over the simplex."""
    rng = np.random.default_rng(5)
    for n in (3, 6, 12):
        z = rng.normal(size=n) * 1.5
        p, _, _ = oracle.entmax_row(z, alpha)
        best = tsallis_objective(p, z, alpha)
        cand = rng.dirichlet(np.ones(n) * 0.5, size=3000)
        vals = cand @ z + np.sum(cand - cand**alpha, axis=1) / (alpha * (alpha - 1.0))
        assert best >= vals.max() - 1e-12
        for _ in range(300):  # local feasible perturbations
            d = rng.normal(size=n) * 1e-3
            q = np.maximum(p + d - d.mean(), 0)
            q /= q.sum()
            assert best >= tsallis_objective(q, z, alpha) - 1e-13


# -------------------------------------------------------------- attention ---


def _rand_problem(seed, B=2, H=3, Nq=9, Nk=9, D=4, layout=1):
    rng = np.random.default_rng(seed)
    Q = rng.normal(size=(B, H, Nq, D))
    K = rng.normal(size=(B, H, Nk, D))
    V = rng.normal(size=(B, H, Nk, D))
    dO = rng.normal(size=(B, H, Nq, D))
    if layout == 0:
        beta = gamma = None
    elif layout == 1:
        beta, gamma = rng.uniform(0.5, 1.5, H), rng.uniform(-0.7, 1.5, H)
    else:
        beta, gamma = rng.uniform(0.5, 1.5, (B, H, Nq)), rng.uniform(-0.7, 1.5, (B, H, Nq))
    return Q, K, V, dO, beta, gamma


@pytest.mark.parametrize("alpha", [1.5, 2.0, 1.3])
@pytest.mark.parametrize("causal,Nq,Nk", [(True, 9, 9), (False, 9, 9), (True, 5, 11), (False, 7, 3)])
@pytest.mark.parametrize("layout,logn_mode", [(0, 0), (1, 0), (1, 1), (2, 1)])
def test_attention_forward_composition(alpha, causal, Nq, Nk, layout, logn_mode):
    """Sec. 2.1 + eq. (asentmax): rows of P are entmax of scale * <q,k>/sqrt(d) over the visible
    keys (j <= i + Nk - Nq), and O = P V.  Scores and the product are rebuilt with numpy."""
    Q, K, V, _, beta, gamma = _rand_problem(7, Nq=Nq, Nk=Nk, layout=layout)
    delta = 0.8
    out = oracle.attn_fwd(Q, K, V, alpha, beta, gamma, delta=delta, causal=causal, logn_mode=logn_mode, want_p=True)
    B, H, _, D = Q.shape
    Z = np.einsum("bhid,bhjd->bhij", Q, K) / math.sqrt(D)
    for b in range(B):
        for h in range(H):
            for i in range(Nq):
                nv = min(Nk, i + Nk - Nq + 1) if causal else Nk
                nlog = Nk if logn_mode == 0 else nv
                if layout == 0 or nlog <= 1:
                    sc = delta
                else:
                    bt = beta[h] if layout == 1 else beta[b, h, i]
                    gm = gamma[h] if layout == 1 else gamma[b, h, i]
                    sc = delta + bt * math.log(nlog) ** gm
                p, tau, sup = oracle.entmax_row(sc * Z[b, h, i, :nv], alpha)
                np.testing.assert_allclose(out["P"][b, h, i, :nv], p, atol=1e-13)
                assert np.all(out["P"][b, h, i, nv:] == 0)
                assert abs(out["tau"][b, h, i] - tau) < 1e-13 and out["support"][b, h, i] == sup
    np.testing.assert_allclose(out["O"], out["P"] @ V, atol=1e-12)


@pytest.mark.parametrize("alpha", ALPHAS)
def test_attention_two_level_end_to_end(alpha):
    """Two-level logits realised through Q and K (q = a e1, k_j = b_j e1): every row's output
    is the plain mean of the values of its k high keys, for any n (two-level lemma)."""
    n, d, k = 64, 8, 3
    a = 2.0
    rng = np.random.default_rng(2)
    hi = rng.choice(n, size=k, replace=False)
    gap = 1.0 / (alpha - 1.0) + 0.5  # >= k^-(alpha-1)/(alpha-1) for every k >= 1
    bj = np.zeros(n)
    bj[hi] = gap * math.sqrt(d) / a
    Q = np.zeros((1, 1, n, d))
    Q[..., 0] = a
    K = np.zeros((1, 1, n, d))
    K[0, 0, :, 0] = bj
    V = rng.normal(size=(1, 1, n, d))
    out = oracle.attn_fwd(Q, K, V, alpha, causal=False)
    np.testing.assert_allclose(out["O"][0, 0], np.tile(V[0, 0, hi].mean(0), (n, 1)), atol=1e-12)
    assert np.all(out["support"] == k)
    np.testing.assert_allclose(out["tau"], (alpha - 1) * gap - k ** (-(alpha - 1)), atol=1e-12)
    # causal: row i sees only keys <= i; before the first high key all visible logits are equal
    outc = oracle.attn_fwd(Q, K, V, alpha, causal=True)
    first = hi.min()
    for i in range(n):
        vis_hi = hi[hi <= i]
        ref = V[0, 0, : i + 1].mean(0) if i < first else V[0, 0, vis_hi].mean(0)
        np.testing.assert_allclose(outc["O"][0, 0, i], ref, atol=1e-12)
    # single visible key (causal row 0): p = 1, tau = (alpha-1) s - 1  (ALiBi appendix, single support)
    assert abs(outc["tau"][0, 0, 0] - ((alpha - 1) * a * bj[0] / math.sqrt(d) - 1.0)) < 1e-12


def _loss(Q, K, V, dO, alpha, beta, gamma, **kw):
    return float(np.sum(oracle.attn_fwd(Q, K, V, alpha, beta, gamma, **kw)["O"] * dO))


@pytest.mark.parametrize("alpha", [1.25, 1.5, 1.75, 2.0])
@pytest.mark.parametrize("causal,Nq,Nk,layout,logn_mode",
                         [(True, 6, 6, 1, 0), (False, 5, 7, 2, 0), (True, 4, 7, 2, 1), (True, 6, 6, 0, 0)])
def test_backward_matches_finite_differences(alpha, causal, Nq, Nk, layout, logn_mode):
    """The backward is the derivative of the (pinned) forward: central differences of
    sum(O * dO) with respect to every input and scale parameter, on generic tiny inputs."""
    B, H, D = 1, 2, 3
    Q, K, V, dO, beta, gamma = _rand_problem(21, B=B, H=H, Nq=Nq, Nk=Nk, D=D, layout=layout)
    kw = dict(delta=0.9, causal=causal, logn_mode=logn_mode)
    g = oracle.attn_bwd(Q, K, V, dO, alpha, beta, gamma, **kw)
    h = 1e-6

    def fd(arr, set_fn):
        out = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = arr[idx]
            arr[idx] = old + h
            fp = set_fn()
            arr[idx] = old - h
            fm = set_fn()
            arr[idx] = old
            out[idx] = (fp - fm) / (2 * h)
        return out

    f = lambda: _loss(Q, K, V, dO, alpha, beta, gamma, **kw)  # noqa: E731
    tol = dict(atol=2e-6, rtol=1e-5)
    np.testing.assert_allclose(g["dQ"], fd(Q, f), **tol)
    np.testing.assert_allclose(g["dK"], fd(K, f), **tol)
    np.testing.assert_allclose(g["dV"], fd(V, f), **tol)
    if layout != 0:
        np.testing.assert_allclose(g["dbeta"], fd(beta, f), **tol)
        np.testing.assert_allclose(g["dgamma"], fd(gamma, f), **tol)


def _jacobian_probe(z, alpha, w):
    """J(z) w through the oracle's attention backward: non-causal, V = I, K = sqrt(d) I, one query
    row q = z, so that s = z, O = entmax(z) and dQ = J dO."""
    n = len(z)
    Q = z.reshape(1, 1, 1, n)
    K = (np.eye(n) * math.sqrt(n)).reshape(1, 1, n, n)
    V = np.eye(n).reshape(1, 1, n, n)
    g = oracle.attn_bwd(Q, K, V, w.reshape(1, 1, 1, n), alpha, causal=False)
    return g["dQ"].reshape(n)


def test_jacobian_closed_forms():
    rng = np.random.default_rng(9)
    z = rng.normal(size=8)
    u, w = rng.normal(size=8), rng.normal(size=8)
    # alpha = 2: J = I_S - 1 1^T / |S| on the support
    p, _, _ = oracle.entmax_row(z, 2.0)
    S = p > 0
    ref = np.where(S, w - w[S].mean(), 0.0)
    np.testing.assert_allclose(_jacobian_probe(z, 2.0, w), ref, atol=1e-13)
    for alpha in ALPHAS:
        Jw, Ju = _jacobian_probe(z, alpha, w), _jacobian_probe(z, alpha, u)
        assert abs(Jw.sum()) < 1e-13  # 1^T J = 0: probabilities keep summing to one
        assert abs(u @ Jw - w @ Ju) < 1e-13  # J symmetric
        assert np.abs(_jacobian_probe(z, alpha, np.ones(8))).max() < 1e-13  # J 1 = 0
    # alpha -> 1: J -> diag(p) - p p^T of softmax
    sm = np.exp(z - z.max())
    sm /= sm.sum()
    ref = sm * w - sm * (sm @ w)
    assert np.abs(_jacobian_probe(z, 1.01, w) - ref).max() < 3e-2 * np.abs(ref).max()
    assert np.abs(_jacobian_probe(z, 1.1, w) - ref).max() > np.abs(_jacobian_probe(z, 1.01, w) - ref).max()


def test_tile_map_matches_full_matrix():
    Q, K, V, _, beta, gamma = _rand_problem(4, B=1, H=2, Nq=37, Nk=37, D=4, layout=1)
    beta = beta * 6  # sharpen so that some tiles are empty
    out = oracle.attn_fwd(Q, K, V, 1.5, beta, gamma, want_p=True)
    nz, vis = oracle.tile_map(Q, K, 1.5, 8, 4, beta, gamma)
    P = out["P"]
    for ti in range(nz.shape[2]):
        for tj in range(nz.shape[3]):
            blk = P[:, :, ti * 8:(ti + 1) * 8, tj * 4:(tj + 1) * 4]
            assert np.array_equal(nz[:, :, ti, tj] > 0, (blk > 0).any(axis=(2, 3)))
            assert bool(vis[0, 0, ti, tj]) == (tj * 4 <= min(ti * 8 + 7, 36))
    assert 0 < nz.sum() < vis.sum()


# ------------------------------------------------------------------ positional bias (ALiBi / NAPE)

def _alibi(slopes, h, i, j, Nq, Nk):
    """Bias of the ALiBi definition (positional-encoding appendix): -m_h * distance for keys at or before the
    query's position i + (Nk - Nq), zero for later keys."""
    return -slopes[h] * max(i + (Nk - Nq) - j, 0)


@pytest.mark.parametrize("alpha", [1.5, 2.0, 1.3])
@pytest.mark.parametrize("causal,Nq,Nk", [(True, 9, 9), (False, 9, 9), (True, 5, 11), (False, 7, 3)])
@pytest.mark.parametrize("layout,bias_mode", [(0, 0), (1, 0), (1, 1), (2, 1)])
def test_alibi_forward_composition(alpha, causal, Nq, Nk, layout, bias_mode):
    """Sec. 4.2 / App. B: z_ij = <q,k>/sqrt(d) + m_h (j - i); bias_mode 0 multiplies the whole of it by the
    ASEntmax scale (the bias is part of the logit of eq. (asentmax)), bias_mode 1 adds the bias after the
    scale.  Scores are rebuilt with numpy and go through the pinned row routine."""
    Q, K, V, _, beta, gamma = _rand_problem(11, Nq=Nq, Nk=Nk, layout=layout)
    slopes = np.array([0.7, 0.0, 0.05])  # NAPE-like: the middle head has no positional bias
    delta = 0.8
    out = oracle.attn_fwd(Q, K, V, alpha, beta, gamma, delta=delta, causal=causal, want_p=True, slopes=slopes,
                          bias_mode=bias_mode)
    B, H, _, D = Q.shape
    Z = np.einsum("bhid,bhjd->bhij", Q, K) / math.sqrt(D)
    for b in range(B):
        for h in range(H):
            for i in range(Nq):
                nv = min(Nk, i + Nk - Nq + 1) if causal else Nk
                if layout == 0:
                    sc = delta
                else:
                    bt = beta[h] if layout == 1 else beta[b, h, i]
                    gm = gamma[h] if layout == 1 else gamma[b, h, i]
                    sc = delta + bt * math.log(Nk) ** gm
                bias = np.array([_alibi(slopes, h, i, j, Nq, Nk) for j in range(nv)])
                s = sc * (Z[b, h, i, :nv] + bias) if bias_mode == 0 else sc * Z[b, h, i, :nv] + bias
                p, tau, sup = oracle.entmax_row(s, alpha)
                np.testing.assert_allclose(out["P"][b, h, i, :nv], p, atol=1e-13)
                assert abs(out["tau"][b, h, i] - tau) < 1e-13 and out["support"][b, h, i] == sup
    np.testing.assert_allclose(out["O"], out["P"] @ V, atol=1e-12)


@pytest.mark.parametrize("bias_mode", [0, 1])
def test_alibi_zero_slopes_are_nope_bit_for_bit(bias_mode):
    Q, K, V, dO, beta, gamma = _rand_problem(12)
    kw = dict(delta=0.9, causal=True)
    a = oracle.attn_fwd(Q, K, V, 1.5, beta, gamma, **kw)
    b = oracle.attn_fwd(Q, K, V, 1.5, beta, gamma, slopes=np.zeros(3), bias_mode=bias_mode, **kw)
    ga = oracle.attn_bwd(Q, K, V, dO, 1.5, beta, gamma, **kw)
    gb = oracle.attn_bwd(Q, K, V, dO, 1.5, beta, gamma, slopes=np.zeros(3), bias_mode=bias_mode, **kw)
    for k in ("O", "tau"):
        assert np.array_equal(a[k], b[k])
    for k in ("dQ", "dK", "dV", "dbeta", "dgamma"):
        assert np.array_equal(ga[k], gb[k])


@pytest.mark.parametrize("alpha", [1.25, 1.5, 2.0])
@pytest.mark.parametrize("m", [0.3, 1.0])
def test_alibi_hard_window(alpha, m):
    """Proposition on ALiBi with alpha-entmax: with raw logits in [z_min, z_max], a key further than
    d_max = floor((z_max - z_min + 1/(alpha-1)) / m + 1) behind the query gets exactly zero weight."""
    n, d = 96, 4
    rng = np.random.default_rng(5)
    Q = rng.normal(size=(1, 1, n, d))
    K = rng.normal(size=(1, 1, n, d))
    V = rng.normal(size=(1, 1, n, d))
    out = oracle.attn_fwd(Q, K, V, alpha, causal=True, want_p=True, slopes=np.array([m]))
    Z = (Q[0, 0] @ K[0, 0].T) / math.sqrt(d)
    vis = np.tril(np.ones((n, n), bool))
    zmax, zmin = Z[vis].max(), Z[vis].min()
    dmax = math.floor((zmax - zmin + 1.0 / (alpha - 1.0)) / m + 1)
    assert dmax < n - 1  # the bound bites at this size
    P = out["P"][0, 0]
    i, j = np.nonzero(P > 0)
    assert (i - j).max() <= dmax
    # and the window is not vacuous: without the bias the same rows reach further back
    P0 = oracle.attn_fwd(Q, K, V, alpha, causal=True, want_p=True)["P"][0, 0]
    i0, j0 = np.nonzero(P0 > 0)
    assert (i0 - j0).max() > (i - j).max()


def test_alibi_equal_content_is_entmax_of_a_ramp():
    """All content logits equal (q = 0): row i is the entmax of the ramp -m * (i - j), whose alpha = 2 solution
    is the textbook sparsemax of that ramp; keys after the query (non-causal call) carry no bias."""
    n, d, m = 12, 4, 0.2
    rng = np.random.default_rng(6)
    Q = np.zeros((1, 1, n, d))
    K = rng.normal(size=(1, 1, n, d))
    V = rng.normal(size=(1, 1, n, d))
    out = oracle.attn_fwd(Q, K, V, 2.0, causal=False, want_p=True, slopes=np.array([m]))
    for i in range(n):
        ramp = np.array([-m * max(i - j, 0) for j in range(n)])
        p, tau = sparsemax_textbook(ramp)
        np.testing.assert_allclose(out["P"][0, 0, i], p, atol=1e-13)
        assert abs(out["tau"][0, 0, i] - tau) < 1e-13


@pytest.mark.parametrize("alpha", [1.25, 1.5, 2.0])
@pytest.mark.parametrize("causal,Nq,Nk,layout,bias_mode", [(True, 6, 6, 1, 0), (True, 6, 6, 1, 1), (False, 5, 7, 2, 0),
                                                           (True, 4, 7, 2, 1), (True, 6, 6, 0, 0)])
def test_alibi_backward_matches_finite_differences(alpha, causal, Nq, Nk, layout, bias_mode):
    """With the bias inside the scaled logit the scale gradient sees z + b, outside it only z: central
    differences of sum(O * dO) decide (slopes are fixed numbers and get no gradient)."""
    B, H, D = 1, 2, 3
    Q, K, V, dO, beta, gamma = _rand_problem(23, B=B, H=H, Nq=Nq, Nk=Nk, D=D, layout=layout)
    kw = dict(delta=0.9, causal=causal, slopes=np.array([0.4, 0.05]), bias_mode=bias_mode)
    g = oracle.attn_bwd(Q, K, V, dO, alpha, beta, gamma, **kw)
    h = 1e-6

    def fd(arr):
        out = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = arr[idx]
            arr[idx] = old + h
            fp = _loss(Q, K, V, dO, alpha, beta, gamma, **kw)
            arr[idx] = old - h
            fm = _loss(Q, K, V, dO, alpha, beta, gamma, **kw)
            arr[idx] = old
            out[idx] = (fp - fm) / (2 * h)
        return out

    tol = dict(atol=2e-6, rtol=1e-5)
    np.testing.assert_allclose(g["dQ"], fd(Q), **tol)
    np.testing.assert_allclose(g["dK"], fd(K), **tol)
    np.testing.assert_allclose(g["dV"], fd(V), **tol)
    if layout != 0:
        np.testing.assert_allclose(g["dbeta"], fd(beta), **tol)
        np.testing.assert_allclose(g["dgamma"], fd(gamma), **tol)


# ------------------------------------------------------------------ ASEntmax scale projections (Sec. 4.1)

def _proj_case(seed, B=2, H=3, N=5, E=7, wscale=0.7):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((B, N, E)), wscale * rng.standard_normal((H, E)), wscale * rng.standard_normal((H, E)))


def test_scale_projection_special_values():
    """Zero projection vectors give beta = softplus(0) = ln 2 and gamma = 0 whatever X holds; a strongly positive
    pre-activation gives beta = u (softplus is asymptotically the identity) and gamma = s, a strongly negative one
    beta = e^u and gamma = -s."""
    X, Wb, Wg = _proj_case(0)
    beta, gamma = oracle.scale_proj_fwd(X, 0 * Wb, 0 * Wg, 1.5)
    assert np.allclose(beta, math.log(2.0), rtol=0, atol=1e-15) and np.all(gamma == 0.0)
    x = np.zeros((1, 2, 4))
    x[0, 0, 0], x[0, 1, 0] = 50.0, -50.0
    w = np.zeros((1, 4))
    w[0, 0] = 1.0
    beta, gamma = oracle.scale_proj_fwd(x, w, w, 0.8)
    assert abs(beta[0, 0, 0] - 50.0) < 1e-12 and abs(beta[0, 0, 1] / math.exp(-50.0) - 1.0) < 1e-12
    assert abs(gamma[0, 0, 0] - 0.8) < 1e-15 and abs(gamma[0, 0, 1] + 0.8) < 1e-15


def test_scale_projection_composition():
    # the projections through library routines: einsum for the inner products, logaddexp(0, u) = ln(1 + e^u), tanh
    X, Wb, Wg = _proj_case(1, B=2, H=4, N=9, E=16)
    beta, gamma = oracle.scale_proj_fwd(X, Wb, Wg, 2.0)
    assert beta.shape == (2, 4, 9)
    assert np.allclose(beta, np.logaddexp(0.0, np.einsum("bne,he->bhn", X, Wb)), rtol=1e-13, atol=1e-14)
    assert np.allclose(gamma, 2.0 * np.tanh(np.einsum("bne,he->bhn", X, Wg)), rtol=1e-13, atol=1e-14)
    assert (beta > 0).all() and (np.abs(gamma) < 2.0).all()  # the ranges the paper states


def test_scale_projection_backward_finite_differences():
    X, Wb, Wg = _proj_case(2)
    s = 1.3
    rng = np.random.default_rng(3)
    dbeta, dgamma = rng.standard_normal((2, 3, 5)), rng.standard_normal((2, 3, 5))

    def loss(X_, Wb_, Wg_):
        b, g = oracle.scale_proj_fwd(X_, Wb_, Wg_, s)
        return float((b * dbeta).sum() + (g * dgamma).sum())

    grads = oracle.scale_proj_bwd(X, Wb, Wg, s, dbeta, dgamma)
    h = 1e-6
    for name, arr, idx in (("dX", X, (1, 2, 3)), ("dX", X, (0, 0, 6)), ("dWb", Wb, (2, 4)), ("dWb", Wb, (0, 0)),
                           ("dWg", Wg, (1, 5)), ("dWg", Wg, (2, 1))):
        args = {"dX": [X.copy(), Wb, Wg], "dWb": [X, Wb.copy(), Wg], "dWg": [X, Wb, Wg.copy()]}[name]
        k = {"dX": 0, "dWb": 1, "dWg": 2}[name]
        args[k][idx] += h
        up = loss(*args)
        args[k][idx] -= 2 * h
        dn = loss(*args)
        fd = (up - dn) / (2 * h)
        assert abs(fd - grads[name][idx]) < 1e-7 * max(1.0, abs(fd)), (name, idx, fd, grads[name][idx])


def test_scale_projection_chain_into_attention():
    """The projections feed the attention's per-query beta, gamma: the derivative of sum(O * dO) with respect to a
    projection weight, by finite differences through both oracles, equals the projection backward applied to the
    attention backward's d beta, d gamma."""
    rng = np.random.default_rng(4)
    B, H, N, E, D = 1, 2, 6, 5, 4
    X = rng.standard_normal((B, N, E))
    Wb, Wg = 0.5 * rng.standard_normal((H, E)), 0.5 * rng.standard_normal((H, E))
    Q, K, V, dO = (rng.standard_normal((B, H, N, D)) for _ in range(4))
    s, alpha = 1.0, 1.5

    def loss(Wb_, Wg_):
        beta, gamma = oracle.scale_proj_fwd(X, Wb_, Wg_, s)
        return float((oracle.attn_fwd(Q, K, V, alpha, beta=beta, gamma=gamma, logn_mode=1)["O"] * dO).sum())

    beta, gamma = oracle.scale_proj_fwd(X, Wb, Wg, s)
    g = oracle.attn_bwd(Q, K, V, dO, alpha, beta=beta, gamma=gamma, logn_mode=1)
    grads = oracle.scale_proj_bwd(X, Wb, Wg, s, g["dbeta"], g["dgamma"])
    h = 1e-6
    for name, idx in (("dWb", (0, 1)), ("dWb", (1, 4)), ("dWg", (0, 0)), ("dWg", (1, 2))):
        Wb2, Wg2 = Wb.copy(), Wg.copy()
        tgt = Wb2 if name == "dWb" else Wg2
        tgt[idx] += h
        up = loss(Wb2, Wg2)
        tgt[idx] -= 2 * h
        dn = loss(Wb2, Wg2)
        fd = (up - dn) / (2 * h)
        assert abs(fd - grads[name][idx]) < 2e-6 * max(1.0, abs(fd)), (name, idx, fd, grads[name][idx])
