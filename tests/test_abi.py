"""Host-side checks of the C ABI: the library loads, exports every entry point the header
declares, and validates arguments without touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "entmax_attn.h")
LIB = os.path.join(ROOT, "paper_2506_16640_amd", "lib", "libentmax_attn.so")


@pytest.fixture(scope="module")
def binding():
    if not os.path.exists(LIB):
        from paper_2506_16640_amd import build
        build.build_library()
    from paper_2506_16640_amd import binding as b
    return b


def test_exports_every_declared_symbol(binding):
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(entmax_(?:attn|scale_proj)_[a-z_]+)\s*\(", text))
    assert {"entmax_attn_fwd", "entmax_attn_bwd", "entmax_attn_workspace_bytes", "entmax_attn_saved_bytes",
            "entmax_attn_strerror", "entmax_attn_check_params", "entmax_scale_proj_fwd", "entmax_scale_proj_bwd",
            "entmax_scale_proj_workspace_bytes"} <= names
    lib = ctypes.CDLL(LIB)
    for n in names:
        assert hasattr(lib, n), n


def _params(b, **kw):
    base = dict(B=2, H=3, Nq=100, Nk=100, D=64, dtype=0, causal=1, scale_layout=1, logn_mode=0, path=0, alpha=1.5,
                delta=1.0)
    base.update(kw)
    p = b.Params()
    for k, v in base.items():
        setattr(p, k, v)
    return p


def test_parameter_validation(binding):
    b = binding
    assert b.check_params(_params(b)) == 0
    assert b.check_params(_params(b, D=32)) == -2
    assert b.check_params(_params(b, D=96)) == -2
    assert b.check_params(_params(b, alpha=1.0)) == -1
    assert b.check_params(_params(b, alpha=2.5)) == -1
    assert b.check_params(_params(b, alpha=float("nan"))) == -1
    assert b.check_params(_params(b, dtype=3)) == -1
    assert b.check_params(_params(b, causal=2)) == -1
    assert b.check_params(_params(b, scale_layout=5)) == -1
    assert b.check_params(_params(b, Nq=-1)) == -1
    assert b.check_params(_params(b, path=2)) == 0  # the long-sequence kernels at any size (test aid)
    assert b.check_params(_params(b, path=3)) == -1
    assert b.check_params(_params(b, q_stride_b=64 * 100 * 3, q_stride_h=64, q_stride_n=3 * 64)) == 0
    assert b.check_params(_params(b, q_stride_b=6400, q_stride_h=6400, q_stride_n=65)) == -3  # 130 bytes: misaligned
    assert b.check_params(_params(b, q_stride_b=6400, q_stride_h=6400, q_stride_n=32)) == -1  # rows overlap
    assert b.check_params(_params(b, Nq=1 << 23)) == -2
    for code in (0, -1, -2, -3, -4, -5, -99):
        assert isinstance(b.strerror(code), str) and b.strerror(code)


def test_workspace_sizes(binding):
    b = binding
    p = _params(b, B=4, H=12, Nq=4096, Nk=4096)
    fwd, bwd = b.workspace_bytes(p, 0), b.workspace_bytes(p, 1)
    assert fwd >= 48 * 64 * 4096 * 2  # one transposed copy of V plus candidate lists, strips and flags
    assert bwd > 3 * 48 * 64 * 4096 * 2
    assert b.workspace_bytes(_params(b, D=32), 0) == 0
    # the buffer that carries the forward's support lists: a pool of (key, score) entries, six per row on average,
    # behind the per-half-row places, the block flags and the per-key counts -- under half the size of O
    assert b.saved_bytes(p) >= 48 * 4096 * 6 * 8 + 48 * 4096 * 2 * 4 + 48 * 32 * 4 + 48 * 4096 * 4
    assert b.saved_bytes(p) <= 48 * 4096 * 64 * 2 // 2
    assert b.saved_bytes(_params(b, D=32)) == 0
    # ragged lengths are padded to 128 rows in the transposed copies
    small = b.workspace_bytes(_params(b, B=1, H=1, Nq=65, Nk=65), 0)
    assert small >= 64 * 128 * 2 and b.workspace_bytes(_params(b, B=1, H=1, Nq=65, Nk=129), 0) - small == 64 * 128 * 2
    # decode shapes (Nq <= 8, or Nq <= 64 with Nk >= 64 Nq): fp32 score rows (Nk rounded up to 4) and one maximum per chunk of 512 keys
    for nq, nk, dt in ((1, 32768, 0), (8, 32768, 0), (8, 1001, 1), (3, 5, 1), (64, 4096, 1), (32, 32768, 0)):
        need = 48 * nq * ((nk + 3) // 4 * 4) * 4 + 48 * nq * ((nk + 511) // 512) * 4
        assert b.workspace_bytes(_params(b, B=4, H=12, Nq=nq, Nk=nk, dtype=dt), 0) >= need


def test_entry_points_reject_bad_arguments_before_any_launch(binding):
    b = binding
    lib = ctypes.CDLL(LIB)
    lib.entmax_attn_fwd.restype = ctypes.c_int
    p = _params(b)
    null = ctypes.c_void_p(None)
    fake = ctypes.c_void_p(4096)
    bad = ctypes.c_void_p(4100)  # not 16-byte aligned
    def args(**kw):
        a = [kw.get(k, null if k in ("saved", "slopes") else fake)
             for k in ("Q", "K", "V", "beta", "gamma", "slopes", "O", "tau", "saved", "stats", "ws")]
        a.insert(9, ctypes.c_size_t(kw.get("saved_bytes", 0)))  # saved_bytes follows saved
        return a

    call = lambda prm, a, wsb=1 << 30: lib.entmax_attn_fwd(ctypes.byref(prm), *a, ctypes.c_size_t(wsb), null, null)  # noqa
    assert call(_params(b, D=32), args()) == -2
    assert call(p, args(Q=null)) == -1
    assert call(p, args(beta=null)) == -1
    assert call(p, args(K=bad)) == -3
    assert call(p, args(stats=null), wsb=16) == -4
    assert call(p, args(saved=bad)) == -3
    assert call(p, args(slopes=ctypes.c_void_p(4098))) == -3
    assert call(_params(b, bias_mode=2), args()) == -1
    # a saved buffer smaller than the parameters need is refused like a small workspace
    need = b.saved_bytes(p)
    assert call(p, args(saved=fake, saved_bytes=need - 1)) == -4
    assert call(p, args(saved=fake, saved_bytes=0)) == -4
    lib.entmax_attn_bwd.restype = ctypes.c_int
    a = [fake] * 18
    a[6] = null  # saved is optional
    a[7] = ctypes.c_size_t(0)
    a[10] = null  # so are the slopes of the distance bias
    assert lib.entmax_attn_bwd(ctypes.byref(_params(b, alpha=3.0)), *a, ctypes.c_size_t(1 << 30), null, null) == -1
    a[5] = null  # tau
    assert lib.entmax_attn_bwd(ctypes.byref(p), *a, ctypes.c_size_t(1 << 30), null, null) == -1
    a[5] = fake
    assert lib.entmax_attn_bwd(ctypes.byref(p), *a, ctypes.c_size_t(16), null, null) == -4
    a[6], a[7] = fake, ctypes.c_size_t(need - 1)
    assert lib.entmax_attn_bwd(ctypes.byref(p), *a, ctypes.c_size_t(1 << 30), null, null) == -4


def test_binding_rejects_mismatched_tensors(binding):
    """The Python layer raises (never asserts) on tensors the C ABI cannot describe; CPU tensors suffice because
    the checks run before the library is called."""
    import torch
    b = binding
    q = torch.zeros(1, 2, 16, 64, dtype=torch.bfloat16)
    k = torch.zeros(1, 2, 16, 64, dtype=torch.bfloat16)
    beta = torch.ones(2)
    with pytest.raises(TypeError):
        b.entmax_attn_fwd(q, k.float(), k.float())
    with pytest.raises(ValueError):
        b.entmax_attn_fwd(q, k, k[:, :, :8])
    with pytest.raises(ValueError):
        b.entmax_attn_fwd(q, k, k, beta=beta, gamma=None)
    with pytest.raises(ValueError):
        b.entmax_attn_fwd(q, k, k, beta=beta.double(), gamma=beta.double())
    with pytest.raises(ValueError):
        b.entmax_attn_fwd(q, k, k, beta=torch.ones(3), gamma=torch.ones(3))
    with pytest.raises(ValueError):
        b.entmax_attn_fwd(q, k, k, stats=torch.zeros(16, dtype=torch.int64))
    with pytest.raises(ValueError):
        b.entmax_attn_fwd(q, k, k, tau=torch.zeros(1, 2, 15))
    with pytest.raises(ValueError):
        b.entmax_attn_bwd(q, k, k, q, q[:, :, :8], torch.zeros(1, 2, 16))
    with pytest.raises(TypeError):
        b.make_params(q.half(), k.half(), 1.5, 1.0, True, None, 0)


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU's share; asked for more it says so and exits without touching a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_forward_list_launch_shapes():
    """Host arithmetic of the forward's list launch, seen through the workspace size: causal pairs of query blocks
    by default (one scratch strip per pair), single blocks from 128 pairs up to 767 (one strip per block)."""
    import ctypes
    from paper_2506_16640_amd import binding as b
    lib = b._lib

    def ws(B, H, n):
        p = b.Params()
        p.B, p.H, p.Nq, p.Nk, p.D = B, H, n, n, 64
        p.dtype, p.causal, p.alpha, p.delta = 0, 1, 1.5, 1.0
        p.q_stride_b = p.kv_stride_b = H * n * 64
        p.q_stride_h = p.kv_stride_h = n * 64
        p.q_stride_n = p.kv_stride_n = 64
        assert lib.entmax_attn_check_params(ctypes.byref(p)) == 0
        return int(lib.entmax_attn_workspace_bytes(ctypes.byref(p), 0))

    strip = 256 * 32 * 20  # threads x cells per thread x bytes per cell
    # n = 1024: 8 blocks, 4 pairs per head.  12 and 24 heads (48, 96 pairs) keep the pairs, 48 heads (192 pairs) do not
    w12, w24, w48 = ws(1, 12, 1024), ws(2, 12, 1024), ws(4, 12, 1024)
    extra = (w48 - w24) - 2 * (w24 - w12)
    assert abs(extra - 48 * 4 * strip) < 65536, extra
    # from 768 pairs on the pairs are back: 192 and 384 heads (768, 1536 pairs)
    w192, w384, w96 = ws(16, 12, 1024), ws(32, 12, 1024), ws(8, 12, 1024)
    assert abs((w384 - w192) - 192 * ((w24 - w12) // 12)) < 65536
    assert w96 > w192 // 2 + 96 * 3 * strip  # 96 heads (384 pairs) carry a strip per block
