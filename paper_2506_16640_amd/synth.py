"""Seeded synthetic inputs for entmax attention: the only module shared by the
CPU oracle's tests and the GPU path's tests / benchmark.

It holds none of the method's arithmetic (no entmax, no attention): it draws
Q, K, V, dO and the ASEntmax scale parameters with the shapes and structure of
the paper's language-model workloads (12 heads x d=64, hidden 768; App. G) and
rounds them to the working dtype, so that both sides receive the very same
numbers.  Values are returned as float32 numpy arrays that are exactly
representable in the working dtype (bf16 or fp32).
"""
import math

import numpy as np

# Named workloads.  "c1".."c5" follow the benchmark configurations; the "*d"
# variants are the dense-regime companions (delta = 0, gamma = -1/2, the
# constant-logit-range setting of Sec. 4.1) where little can be skipped.
CONFIGS = {
    "c1": dict(B=1, H=1, n=256, d=64, dtype="fp32", alpha=1.5, scale="none", planted=0.0, bwd=True),
    "c2": dict(B=8, H=12, n=1024, d=64, dtype="bf16", alpha=1.5, scale="head", planted=0.0, bwd=False),
    "c3": dict(B=4, H=12, n=4096, d=64, dtype="bf16", alpha=1.5, scale="head", planted=0.05, bwd=True),
    "c4": dict(B=1, H=12, n=32768, d=64, dtype="bf16", alpha=1.5, scale="head", planted=0.05, bwd=False),
    "c5": dict(B=2, H=16, n=8192, d=128, dtype="bf16", alpha=1.5, scale="head", planted=0.0, bwd=True),
    "c3d": dict(B=4, H=12, n=4096, d=64, dtype="bf16", alpha=1.5, scale="dense", planted=0.05, bwd=True),
    "c4d": dict(B=1, H=12, n=32768, d=64, dtype="bf16", alpha=1.5, scale="dense", planted=0.05, bwd=False),
    "c5d": dict(B=2, H=16, n=8192, d=128, dtype="bf16", alpha=1.5, scale="dense", planted=0.0, bwd=True),
}


def bf16_round(x):
    """Round float32 to the nearest bfloat16 (ties to even); result kept as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    bias = ((u >> 16) & 1) + 0x7FFF
    r = ((u + bias) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(x.shape)


def _rng(seed, stream):
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def _plant(Q, K, frac, rng):
    """For a fraction of the keys of every head, move the key along one random
    later query so that their logit <q_i,k_j>/sqrt(d) equals +4 (four standard
    deviations of the background): k_j += ((4 sqrt d - <q_i,k_j>)/|q_i|^2) q_i."""
    B, H, n, d = K.shape
    m = int(math.ceil(frac * n))
    for b in range(B):
        for h in range(H):
            js = rng.choice(n, size=m, replace=False)
            is_ = js + (rng.random(m) * (n - js)).astype(np.int64)
            is_ = np.minimum(is_, n - 1)
            q = Q[b, h, is_].astype(np.float64)
            k = K[b, h, js].astype(np.float64)
            cur = np.sum(q * k, axis=1)
            coef = (4.0 * math.sqrt(d) - cur) / np.sum(q * q, axis=1)
            K[b, h, js] = (k + coef[:, None] * q).astype(np.float32)
    return K


def make_inputs(B, H, n, d, dtype="bf16", scale="head", planted=0.0, seed=0, nk=None, want_dO=True, **_unused):
    """Draw one workload.  Returns a dict of float32 arrays:
    Q [B,H,n,d], K,V [B,H,nk,d], dO [B,H,n,d] ~ N(0,1) rounded to `dtype`;
    beta,gamma [H] (None for scale="none"), delta (float).

    scale: "none"  -> plain 1/sqrt(d) logits (delta=1, no beta/gamma);
           "head"  -> per-head beta,gamma ~ U(0.5,1.5), delta=1;
           "dense" -> per-head beta ~ U(0.5,1.5), gamma=-0.5, delta=0;
           "query" -> per-query beta,gamma [B,H,n] ~ U(0.5,1.5), delta=1.
    """
    nk = n if nk is None else nk
    Q = _rng(seed, 1).standard_normal((B, H, n, d), dtype=np.float32)
    K = _rng(seed, 2).standard_normal((B, H, nk, d), dtype=np.float32)
    V = _rng(seed, 3).standard_normal((B, H, nk, d), dtype=np.float32)
    if dtype == "bf16":
        Q = bf16_round(Q)
    if planted > 0.0:
        assert nk == n
        K = _plant(Q, K, planted, _rng(seed, 5))
    out = {}
    if dtype == "bf16":
        K, V = bf16_round(K), bf16_round(V)
    out["Q"], out["K"], out["V"] = Q, K, V
    if want_dO:
        dO = _rng(seed, 4).standard_normal((B, H, n, d), dtype=np.float32)
        out["dO"] = bf16_round(dO) if dtype == "bf16" else dO
    prng = _rng(seed, 6)
    if scale == "none":
        out["beta"], out["gamma"], out["delta"] = None, None, 1.0
    elif scale == "head":
        out["beta"] = prng.uniform(0.5, 1.5, size=H).astype(np.float32)
        out["gamma"] = prng.uniform(0.5, 1.5, size=H).astype(np.float32)
        out["delta"] = 1.0
    elif scale == "dense":
        out["beta"] = prng.uniform(0.5, 1.5, size=H).astype(np.float32)
        out["gamma"] = np.full(H, -0.5, dtype=np.float32)
        out["delta"] = 0.0
    elif scale == "query":
        out["beta"] = prng.uniform(0.5, 1.5, size=(B, H, n)).astype(np.float32)
        out["gamma"] = prng.uniform(0.5, 1.5, size=(B, H, n)).astype(np.float32)
        out["delta"] = 1.0
    else:
        raise ValueError(scale)
    return out


def make_config(name, seed=0, **overrides):
    cfg = dict(CONFIGS[name])
    cfg.update(overrides)
    data = make_inputs(seed=seed, **cfg)
    data["cfg"] = cfg
    return data


def nape_slopes(H, first_biased=True):
    """Slopes of the distance bias for the NAPE arrangement of Sec. 4.2: every other head biased, the rest zero.
    The biased heads take m = 2^(-k/K), k = 1..K (App. B, ALiBi definition, over the K biased heads)."""
    m = np.zeros(H, dtype=np.float32)
    idx = np.arange(0 if first_biased else 1, H, 2)
    for k, h in enumerate(idx):
        m[h] = 2.0 ** (-(k + 1) / len(idx))
    return m


def dense_equiv_flops(B, H, n, d, causal=True, bwd=False):
    """Usual attention convention: forward 4 B H n^2 d (half under a causal mask), backward 2.5x."""
    f = 4.0 * B * H * n * n * d * (0.5 if causal else 1.0)
    return f * (2.5 if bwd else 1.0)
