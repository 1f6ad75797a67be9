#!/usr/bin/env python3
"""Benchmark of the entmax attention hot path on one MI355X.

A step is one forward + one backward of the whole path (C ABI calls
entmax_attn_fwd and entmax_attn_bwd) over one batch of the headline workload:
the 120M-class LM attention layer at training length (B=4, H=12, n=4096, d=64,
bf16, causal, alpha=1.5, per-head ASEntmax scale, 5% planted keys), seeded and
synthetic, resident in HBM before the timed region.  Prints ONE JSON line whose
`value` is that workload's tokens per second; the other benchmark configurations
(n=1024 forward, n=32768 forward, the alpha sweep at d=128, the dense-regime
companion, decode shapes) are timed the same way and reported as extra objects of
the same line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3] [--alpha A]
                  [--no-cpu-baseline] [--no-extra] [--no-decode]
"""
import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA peak (data sheet)
# HBM bytes per launch of the kernels of the c3 workload: written by `python -m paper_2506_16640_amd.profile_summary`
# from rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this same command (calibrated on a copy kernel of known size)
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_c3_fwd_bwd.txt")


class HipEvents:
    """hipEvent_t handles for the library's profiling hook (recorded on the launch stream)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.all = []

    def make(self, n):
        out = []
        for _ in range(n):
            ev = ctypes.c_void_p()
            rc = self.hip.hipEventCreate(ctypes.byref(ev))
            if rc != 0:
                raise RuntimeError("hipEventCreate failed: %d" % rc)
            out.append(ev.value)
            self.all.append(ev.value)
        return out

    def record(self, ev, stream):
        rc = self.hip.hipEventRecord(ctypes.c_void_p(ev), ctypes.c_void_p(stream))
        if rc != 0:
            raise RuntimeError("hipEventRecord failed: %d" % rc)

    def elapsed_ms(self, a, b):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), ctypes.c_void_p(a), ctypes.c_void_p(b))
        if rc != 0:
            raise RuntimeError("hipEventElapsedTime failed: %d" % rc)
        return float(ms.value)

    def close(self):
        for e in self.all:
            self.hip.hipEventDestroy(ctypes.c_void_p(e))
        self.all = []


def tile_flops(d):
    return 2.0 * 32 * 32 * d  # one 32x32 tile of a product contracting over d (or d outputs over 32 keys)


def read_traffic():
    """kernel name -> HBM bytes per launch, from the committed profile summary (None if absent)."""
    if not os.path.exists(TRAFFIC_FILE):
        return None
    out = {}
    for line in open(TRAFFIC_FILE):
        parts = line.split()
        if len(parts) >= 2 and not line.startswith("#"):
            try:
                out[parts[0]] = float(parts[1])
            except ValueError:
                pass
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c3")
    ap.add_argument("--alpha", type=float, default=None, help="entmax alpha instead of the workload's own (1.5)")
    ap.add_argument("--nape", action="store_true", help="every other head with the linear distance bias (Sec. 4.2)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the other benchmark configurations (c2, c4, c5, c3d)")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode-shape (Nk = 32768) measurements")
    ap.add_argument("--decode-rows", default="1,8,64", help="query rows of the decode-shape measurements")
    ap.add_argument("--projection-only", action="store_true",
                    help="of the extra measurements run only the scale projections (for profiling them alone)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2506_16640_amd import binding, synth

    assert torch.cuda.is_available(), "needs an MI355X"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    hev = HipEvents()

    def upload(name, want_dO=True):
        data = synth.make_config(name, seed=0)
        cfg = data["cfg"]
        tdt = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
        t = {k: torch.from_numpy(data[k]).to(dev).to(tdt) for k in ("Q", "K", "V")}
        if want_dO:
            t["dO"] = torch.from_numpy(data["dO"]).to(dev).to(tdt)
        t["beta"] = None if data["beta"] is None else torch.from_numpy(data["beta"]).to(dev)
        t["gamma"] = None if data["gamma"] is None else torch.from_numpy(data["gamma"]).to(dev)
        return data, cfg, t

    def measure(name, steps, warmup, alpha=None, want_events=True, nape=False, per_query=False):
        """Times `steps` steps of workload `name` (forward, plus backward with the forward's saved buffer where the
        workload has one) wall-clock with no events inside, then once more with the library's phase events."""
        data, cfg, t = upload(name, want_dO=bool(synth.CONFIGS[name]["bwd"]))
        B, H, n, d = cfg["B"], cfg["H"], cfg["n"], cfg["d"]
        alpha = cfg["alpha"] if alpha is None else alpha
        do_bwd = bool(cfg["bwd"])
        logn_mode = 0
        if per_query:
            # beta, gamma per query (what the scale projections produce) with n = keys visible to the row: the
            # per-head values spread over the rows with a seeded +-10 % variation
            rq = np.random.Generator(np.random.Philox(key=[0, 99]))
            for nm in ("beta", "gamma"):
                base = data[nm][None, :, None] * (1.0 + 0.1 * rq.uniform(-1, 1, size=(B, H, n)))
                t[nm] = torch.from_numpy(base.astype(np.float32)).to(dev)
            logn_mode = 1
        kw = dict(alpha=alpha, beta=t["beta"], gamma=t["gamma"], delta=data["delta"], causal=True, logn_mode=logn_mode)
        if nape:  # Sec. 4.2: every other head carries the linear distance bias, inside the ASEntmax scale
            kw.update(alibi_slopes=torch.from_numpy(synth.nape_slopes(H)).to(dev), bias_mode=0)
        prm = binding.make_params(t["Q"], t["K"], alpha, data["delta"], True, t["beta"], logn_mode)
        ws = torch.empty(max(binding.workspace_bytes(prm, 0), binding.workspace_bytes(prm, 1) if do_bwd else 0),
                         dtype=torch.uint8, device=dev)
        out = torch.empty_like(t["Q"])
        tau = torch.empty(B, H, n, dtype=torch.float32, device=dev)
        # what a training step keeps between forward and backward: O, tau and the rows' support lists
        saved = binding.new_saved(prm, dev) if do_bwd else None

        def step(fwd_ev=None, bwd_ev=None, stats=None):
            binding.entmax_attn_fwd(t["Q"], t["K"], t["V"], out=out, tau=tau, workspace=ws, stats=stats,
                                    phase_events=fwd_ev, saved=saved, **kw)
            if do_bwd:
                binding.entmax_attn_bwd(t["Q"], t["K"], t["V"], out, t["dO"], tau, workspace=ws, stats=stats,
                                        phase_events=bwd_ev, saved=saved, **kw)

        st = binding.new_stats(dev)  # tile counters (one untimed step): executed work and tile-skip rate
        step(stats=st)
        torch.cuda.synchronize()
        sd = binding.stats_dict(st)
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()  # the timed region: exactly `steps` steps, no events inside
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps

        F = tile_flops(d)
        # algorithmic flops per launch: 2*32*32*D per 32x32 score tile, times the tiles the kernel's own counters
        # report.  The finish / row / key kernels of the list path are gathers over a few entries per row: no tile work.
        algo = {
            "fwd_lists": F * sd["fwd_list_qk"], "fwd_finish": 0.0,
            "fwd_tiled": F * (sd["fwd_qk_max"] + sd["fwd_qk_solve"] + sd["fwd_qk_pv"] + sd["fwd_pv_tiles"]),
            "bwd_lists": F * sd["bwd_list_qk"], "bwd_rows": 0.0, "bwd_keys": 0.0,
            # the dQ kernel forms the scores of every tile it visits and three more products on the active ones
            "bwd_dq": F * (sd["bwd_qk_mask"] + 3 * sd["bwd_dq_tiles"]), "bwd_dkv": F * 4 * sd["bwd_dkv_tiles"],
        }
        res = {"cfg": cfg, "alpha": alpha, "ms": ms, "stats": sd, "algo": algo, "do_bwd": do_bwd, "data": data}
        if want_events:
            fwd_sets = [hev.make(binding.FWD_NUM_PHASES + 1) for _ in range(steps)]
            bwd_sets = [hev.make(binding.BWD_NUM_PHASES + 1) for _ in range(steps)] if do_bwd else [None] * steps
            torch.cuda.synchronize()
            for k in range(steps):
                step(fwd_sets[k], bwd_sets[k])
            torch.cuda.synchronize()

            def phase_ms(sets, names):
                return {nm: float(np.mean([hev.elapsed_ms(s[pi], s[pi + 1]) for s in sets])) for pi, nm in enumerate(names)}

            fwd_ms = phase_ms(fwd_sets, binding.FWD_PHASES)
            bwd_ms = phase_ms(bwd_sets, binding.BWD_PHASES) if do_bwd else {}
            kernel_ms = {"fwd_lists": fwd_ms["lists"], "fwd_finish": fwd_ms["finish"], "fwd_tiled": fwd_ms["tiled"]}
            if do_bwd:
                # (phases that launch nothing -- "mask" always, "lists" when the forward's lists are handed over --
                # still show the few microseconds between two event records)
                kernel_ms.update(bwd_lists=bwd_ms["lists"], bwd_rows=bwd_ms["rows"], bwd_keys=bwd_ms["keys"],
                                 bwd_dq=bwd_ms["dq"], bwd_dkv=bwd_ms["dkv"])
            res.update(fwd_ms=float(np.mean([hev.elapsed_ms(s[0], s[-1]) for s in fwd_sets])),
                       bwd_ms=float(np.mean([hev.elapsed_ms(s[0], s[-1]) for s in bwd_sets])) if do_bwd else 0.0,
                       phase_ms={"fwd": fwd_ms, "bwd": bwd_ms}, kernel_ms=kernel_ms)
        return res

    def summary(r):
        """The figures every workload reports."""
        cfg, sd, ms = r["cfg"], r["stats"], r["ms"]
        B, H, n, d = cfg["B"], cfg["H"], cfg["n"], cfg["d"]
        dense = synth.dense_equiv_flops(B, H, n, d, True, False) + (
            synth.dense_equiv_flops(B, H, n, d, True, True) if r["do_bwd"] else 0.0)
        executed = sum(r["algo"].values())
        out = {
            "workload": "%s B=%d H=%d n=%d d=%d %s causal alpha=%g, %s" % (
                cfg.get("scale", ""), B, H, n, d, cfg["dtype"], r["alpha"], "fwd+bwd" if r["do_bwd"] else "fwd"),
            "ms": ms, "tokens_per_s": B * n / (ms * 1e-3),
            "executed_tflops": executed / (ms * 1e-3) / 1e12,
            "frac_bf16_mfma_peak_executed": executed / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "dense_equiv_tflops": dense / (ms * 1e-3) / 1e12,
            "list_blocks_fraction": sd["fwd_sparse_blocks"] / max(B * H * ((n + 127) // 128), 1),
            # tiles that can hold a non-zero probability: candidate tiles of the list kernel (an upper bound of the
            # non-zero tiles) plus the P.V tiles the tiled kernel executed
            "tile_skip_rate_fwd": 1.0 - (sd["fwd_cand_tiles"] + sd["fwd_pv_tiles"]) / max(sd["fwd_tiles_visible"], 1),
            "support_per_row": (sd["fwd_support"] if sd["fwd_support"] else sd["bwd_support"]) / max(B * H * n, 1),
        }
        if sd["fwd_window_skipped"]:  # distance bias: visible tiles beyond every row's window, never visited
            out["window_skipped_fraction"] = sd["fwd_window_skipped"] / max(sd["fwd_tiles_visible"], 1)
        if "kernel_ms" in r:
            out["kernel_ms"] = r["kernel_ms"]
        return out

    # ---------------------------------------------------------------- headline workload
    main_r = measure(args.workload, args.steps, args.warmup, alpha=args.alpha, nape=args.nape)
    cfg, sd, ms_per_step = main_r["cfg"], main_r["stats"], main_r["ms"]
    B, H, n, d, alpha = cfg["B"], cfg["H"], cfg["n"], cfg["d"], main_r["alpha"]
    kernel_ms, algo = main_r["kernel_ms"], main_r["algo"]
    # the roofline object describes the longest kernel among those that do tile (MFMA) work
    dominant = max((k for k in kernel_ms if algo[k] > 0), key=kernel_ms.get, default=max(kernel_ms, key=kernel_ms.get))
    achieved = algo[dominant] / (kernel_ms[dominant] * 1e-3) / 1e12
    traffic = read_traffic() if args.workload == "c3" and args.alpha is None and not args.nape else None
    s_main = summary(main_r)

    # what the matrix pipeline sustains with nothing else in the way (measured beside the data-sheet peak)
    sink = torch.zeros(1, dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    binding.mfma_probe(2000, 2048, sink)
    torch.cuda.synchronize()
    e0, e1 = hev.make(2)
    hev.record(e0, stream)
    probe_flops = binding.mfma_probe(20000, 2048, sink)
    hev.record(e1, stream)
    torch.cuda.synchronize()
    mfma_measured = probe_flops / (hev.elapsed_ms(e0, e1) * 1e-3) / 1e12

    result = {
        "metric": "entmax attention fwd+bwd tokens/s at n=4096 (TFLOP/s, %% of bf16 MFMA peak and fwd at n=32768 alongside)",
        "value": s_main["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if cfg["dtype"] == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": "%s: B=%d H=%d n=%d d=%d %s causal alpha=%g ASEntmax per-head scale, %g%% planted keys, %s%s"
                               % (args.workload, B, H, n, d, cfg["dtype"], alpha, 100 * cfg["planted"],
                                  "fwd+bwd" if main_r["do_bwd"] else "fwd", ", NAPE distance bias" if args.nape else ""),
                   "B": B, "H": H, "n": n, "d": d, "alpha": alpha, "tile": "32x32"},
        "tokens_per_s": s_main["tokens_per_s"],
        # matrix-core work the kernels executed (their own tile counters) per second of the whole step, and the usual
        # attention convention (4 B H n^2 d, half under the causal mask, backward 2.5x): work the method mostly skips
        "executed_tflops": s_main["executed_tflops"],
        "frac_bf16_mfma_peak_executed": s_main["frac_bf16_mfma_peak_executed"],
        "dense_equiv_tflops": s_main["dense_equiv_tflops"],
        "fwd_ms": main_r["fwd_ms"],
        "bwd_ms": main_r["bwd_ms"],
        "kernel_ms": kernel_ms,
        "phase_ms": main_r["phase_ms"],
        "tile_skip_rate_fwd": s_main["tile_skip_rate_fwd"],
        "list_blocks_fraction": s_main["list_blocks_fraction"],
        "support_per_row": s_main["support_per_row"],
        "candidates_per_row": sd["fwd_candidates"] / max(B * H * n, 1),
        "solve_sweeps_per_tiled_block": sd["fwd_solve_sweeps"] / max(sd["fwd_blocks"], 1),
        "tile_stats": sd,
        "mfma_peak_measured_tflops": mfma_measured,
        "roofline": {"bound": "mfma", "kernel": dominant, "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                     "frac_of_measured_peak": achieved / mfma_measured,
                     "traffic": None if not traffic else traffic.get(dominant)},
    }
    data_main = main_r.pop("data")
    do_bwd = main_r["do_bwd"]
    del main_r
    torch.cuda.empty_cache()

    if not args.no_extra and not args.projection_only and args.workload == "c3" and args.alpha is None and not args.nape:
        k4 = max(3, args.steps // 4)
        extra = {}
        extra["c2_n1024_fwd"] = summary(measure("c2", args.steps, args.warmup))
        torch.cuda.empty_cache()
        extra["c4_n32768_fwd"] = summary(measure("c4", k4, 1))
        torch.cuda.empty_cache()
        for a5 in (1.25, 1.5, 2.0):
            extra["c5_n8192_d128_alpha%g" % a5] = summary(measure("c5", k4, 1, alpha=a5))
            torch.cuda.empty_cache()
        extra["c3d_dense_regime"] = summary(measure("c3d", k4, 1))
        torch.cuda.empty_cache()
        extra["c3_per_query_scale_logn_visible"] = summary(measure("c3", args.steps, args.warmup, per_query=True))
        torch.cuda.empty_cache()
        extra["c3_alpha1.25"] = summary(measure("c3", k4, 1, alpha=1.25))
        torch.cuda.empty_cache()
        extra["c3_nape_fwd_bwd"] = summary(measure("c3", args.steps, args.warmup, nape=True))
        torch.cuda.empty_cache()
        extra["c4_nape_fwd"] = summary(measure("c4", k4, 1, nape=True))
        torch.cuda.empty_cache()
        for v in extra.values():
            v.pop("data", None)
        result["other_workloads"] = extra
        result["fwd_n32768"] = extra["c4_n32768_fwd"]

    if not args.no_extra and args.workload == "c3" and args.alpha is None and not args.nape:
        # the step right before the attention: beta = softplus(X w), gamma = s tanh(X w) from the layer's token
        # embeddings (hidden 768, the paper's model width), and its backward; bound by reading X / writing dX
        Bp, Np, Ep, Hp = B, n, 768, H
        rngp = np.random.Generator(np.random.Philox(key=[0, 77]))
        xp = torch.from_numpy(rngp.standard_normal((Bp, Np, Ep)).astype(np.float32)).to(dev).to(torch.bfloat16)
        wbp = torch.from_numpy((0.05 * rngp.standard_normal((Hp, Ep))).astype(np.float32)).to(dev)
        wgp = torch.from_numpy((0.05 * rngp.standard_normal((Hp, Ep))).astype(np.float32)).to(dev)
        dbp = torch.from_numpy(rngp.standard_normal((Bp, Hp, Np)).astype(np.float32)).to(dev)
        wsp = torch.empty(64 << 20, dtype=torch.uint8, device=dev)
        bp, gp = binding.scale_proj_fwd(xp, wbp, wgp, 1.0)
        for _ in range(3):
            binding.scale_proj_fwd(xp, wbp, wgp, 1.0)
            binding.scale_proj_bwd(xp, wbp, wgp, bp, gp, dbp, dbp, 1.0, workspace=wsp)
        evs = [hev.make(3) for _ in range(args.steps)]
        torch.cuda.synchronize()
        for e3 in evs:
            hev.record(e3[0], stream)
            binding.scale_proj_fwd(xp, wbp, wgp, 1.0)
            hev.record(e3[1], stream)
            binding.scale_proj_bwd(xp, wbp, wgp, bp, gp, dbp, dbp, 1.0, workspace=wsp)
            hev.record(e3[2], stream)
        torch.cuda.synchronize()
        pf = float(np.mean([hev.elapsed_ms(e3[0], e3[1]) for e3 in evs]))
        pb = float(np.mean([hev.elapsed_ms(e3[1], e3[2]) for e3 in evs]))
        xbytes = Bp * Np * Ep * 2
        obytes = Bp * Hp * Np * 4
        result["scale_projection"] = {
            "workload": "B=%d n=%d E=%d H=%d bf16 X, fp32 projection vectors" % (Bp, Np, Ep, Hp),
            "fwd_ms": pf, "bwd_ms": pb,
            # algorithmic bytes: forward reads X and writes beta, gamma; backward reads X, beta, gamma, dbeta, dgamma
            # and writes dX
            "fwd_hbm_frac": (xbytes + 2 * obytes) / (pf * 1e-3) / 1e9 / 8000.0,
            "bwd_hbm_frac": (2 * xbytes + 4 * obytes) / (pb * 1e-3) / 1e9 / 8000.0,
        }
        del xp, wsp
        torch.cuda.empty_cache()

    if not args.no_decode and args.workload == "c3":
        # decode shapes: a few new query rows against a 32768-key cache; bound by one read of K from HBM
        result["decode_nk32768"] = {}
        for nq in [int(x) for x in args.decode_rows.split(",") if x]:  # from 16 rows on the scores come from the matrix cores
            dd = synth.make_inputs(B=4, H=12, n=nq, nk=32768, d=64, dtype="bf16", scale="head", seed=0, want_dO=False)
            td = {k: torch.from_numpy(dd[k]).to(dev).to(torch.bfloat16) for k in ("Q", "K", "V")}
            bd, gd = (torch.from_numpy(dd[k]).to(dev) for k in ("beta", "gamma"))
            kwd = dict(alpha=1.5, beta=bd, gamma=gd, delta=dd["delta"], causal=True)
            prmd = binding.make_params(td["Q"], td["K"], 1.5, dd["delta"], True, bd, 0)
            wsd = torch.empty(binding.workspace_bytes(prmd, 0), dtype=torch.uint8, device=dev)
            outd = torch.empty_like(td["Q"])
            taud = torch.empty(4, 12, nq, dtype=torch.float32, device=dev)
            # two copies of K (2 x 201 MB), taken in turn: a step must not find its K in the 256 MB last-level cache
            kcopies = [td["K"], td["K"].clone()]
            for _ in range(4):
                binding.entmax_attn_fwd(td["Q"], kcopies[_ % 2], td["V"], out=outd, tau=taud, workspace=wsd, **kwd)
            kd = max(5, args.steps)
            evd = [hev.make(binding.FWD_NUM_PHASES + 1) for _ in range(kd)]
            torch.cuda.synchronize()
            ta = time.perf_counter()
            for k in range(kd):
                binding.entmax_attn_fwd(td["Q"], kcopies[k % 2], td["V"], out=outd, tau=taud, workspace=wsd,
                                        phase_events=evd[k], **kwd)
            torch.cuda.synchronize()
            tb = time.perf_counter()
            scores_ms = float(np.mean([hev.elapsed_ms(s[1], s[2]) for s in evd]))
            solve_ms = float(np.mean([hev.elapsed_ms(s[2], s[3]) for s in evd]))
            algo_bytes = 4 * 12 * 32768 * (64 * 2 + nq * 4)  # K read once, the score rows written once
            result["decode_nk32768"]["nq%d" % nq] = {
                "workload": "B=4 H=12 Nq=%d Nk=32768 d=64 bf16 causal alpha=1.5 ASEntmax scale, fwd" % nq,
                "steps": kd, "ms": (tb - ta) * 1e3 / kd, "scores_kernel_ms": scores_ms, "solve_kernel_ms": solve_ms,
                "roofline": {"bound": "hbm", "kernel": "decode_scores" if nq < 16 else "decode_scores_mfma", "achieved": algo_bytes / (scores_ms * 1e-3) / 1e9,
                             "peak": 8000.0, "unit": "GB/s", "frac": algo_bytes / (scores_ms * 1e-3) / 1e9 / 8000.0},
            }
            del td, wsd, kcopies
    hev.close()

    if not args.no_cpu_baseline:
        # the fp64 oracle as it stands, on a bounded sample of the same workload: the first batches on all host
        # threads, and one head on a single thread
        from oracle import oracle
        bs = min(B, 2)
        sub = {k: data_main[k][:bs] for k in ("Q", "K", "V", "dO") if k in data_main}
        okw = dict(beta=data_main["beta"], gamma=data_main["gamma"], delta=data_main["delta"], causal=True)

        def run_oracle(s, kw):
            c0 = time.perf_counter()
            oracle.attn_fwd(s["Q"], s["K"], s["V"], alpha, **kw)
            if do_bwd:
                oracle.attn_bwd(s["Q"], s["K"], s["V"], s["dO"], alpha, **kw)
            return time.perf_counter() - c0

        t_all = run_oracle(sub, okw)
        one = {k: v[:1, :1] for k, v in sub.items()}
        okw1 = dict(okw)
        if okw1["beta"] is not None:
            okw1["beta"], okw1["gamma"] = okw1["beta"][:1], okw1["gamma"][:1]
        t_one = None
        try:
            # the oracle library reads the thread count per call through OpenMP's runtime routine
            omp = ctypes.CDLL("libgomp.so.1")
            nthreads = oracle.num_threads()
            omp.omp_set_num_threads(1)
            t_one = run_oracle(one, okw1)
            omp.omp_set_num_threads(nthreads)
        except OSError:
            pass
        result["cpu_baseline"] = {
            "value": bs * n / t_all, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "fp64 oracle %s on the first %d of %d batches (%d heads, n=%d), %.1f s wall"
                      % ("fwd+bwd" if do_bwd else "fwd", bs, B, bs * H, n, t_all),
            "one_core": None if t_one is None else {
                "value": n / H / t_one, "unit": "tokens/s",
                "sample": "one head (1/%d of a batch) on one thread, %.1f s wall" % (H, t_one)},
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
