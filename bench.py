#!/usr/bin/env python3
"""Benchmark of the entmax attention hot path on one MI355X.

A step is one forward + one backward of the whole path (C ABI calls
entmax_attn_fwd and entmax_attn_bwd) over one batch of the headline workload:
the 120M-class LM attention layer at training length (B=4, H=12, n=4096, d=64,
bf16, causal, alpha=1.5, per-head ASEntmax scale, 5% planted keys), seeded and
synthetic, resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3] [--alpha A] [--no-cpu-baseline] [--no-c4] [--no-decode]
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

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA peak
# HBM bytes per launch at the c3 workload, from rocprofv3 FETCH_SIZE + WRITE_SIZE runs of this same command scaled by
# what the counters read for a conversion kernel of known size (profiles/pmc_c3_fwd_bwd.md).  Other workloads: null.
MEASURED_HBM_BYTES_C3 = {
    "fwd_lists": 141.1e6, "fwd_finish": 78.5e6, "bwd_rows": 177.2e6, "bwd_keys": 156.3e6,
}


class HipEvents:
    """hipEvent_t handles for the library's profiling hook (recorded on the launch stream)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c3")
    ap.add_argument("--alpha", type=float, default=None, help="entmax alpha instead of the workload's own (1.5)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-c4", action="store_true", help="skip the n=32768 forward-only measurement")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode-shape (Nq = 1 and 8, Nk = 32768) measurement")
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

    data, cfg, t = upload(args.workload)
    B, H, n, d, alpha = cfg["B"], cfg["H"], cfg["n"], cfg["d"], cfg["alpha"]
    if args.alpha is not None:
        alpha = args.alpha
    do_bwd = bool(cfg["bwd"])
    kw = dict(alpha=alpha, beta=t["beta"], gamma=t["gamma"], delta=data["delta"], causal=True, logn_mode=0)
    prm = binding.make_params(t["Q"], t["K"], alpha, data["delta"], True, t["beta"], 0)
    ws = torch.empty(max(binding.workspace_bytes(prm, 0), binding.workspace_bytes(prm, 1)), dtype=torch.uint8,
                     device=dev)
    out = torch.empty_like(t["Q"])
    tau = torch.empty(B, H, n, dtype=torch.float32, device=dev)
    # what a training step keeps between forward and backward: O, tau and the rows' candidate lists
    saved = binding.new_saved(prm, dev) if do_bwd else None

    def step(fwd_ev=None, bwd_ev=None, stats=None):
        binding.entmax_attn_fwd(t["Q"], t["K"], t["V"], out=out, tau=tau, workspace=ws, stats=stats,
                                phase_events=fwd_ev, saved=saved, **kw)
        if do_bwd:
            return binding.entmax_attn_bwd(t["Q"], t["K"], t["V"], out, t["dO"], tau, workspace=ws, stats=stats,
                                           phase_events=bwd_ev, saved=saved, **kw)
        return None

    # tile counters (one untimed step): executed work and tile-skip rate
    st = binding.new_stats(dev)
    step(stats=st)
    torch.cuda.synchronize()
    sd = binding.stats_dict(st)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # the timed region: exactly K steps, no events inside
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # per-kernel durations: the same K steps again with hipEvents between the phases (on the launch stream)
    hev = HipEvents()
    fwd_sets = [hev.make(binding.FWD_NUM_PHASES + 1) for _ in range(args.steps)]
    bwd_sets = [hev.make(binding.BWD_NUM_PHASES + 1) for _ in range(args.steps)] if do_bwd else [None] * args.steps
    torch.cuda.synchronize()
    for k in range(args.steps):
        step(fwd_sets[k], bwd_sets[k])
    torch.cuda.synchronize()

    def phase_ms(sets, names):
        res = {}
        for pi, nm in enumerate(names):
            res[nm] = float(np.mean([hev.elapsed_ms(s[pi], s[pi + 1]) for s in sets]))
        return res

    fwd_ms = phase_ms(fwd_sets, binding.FWD_PHASES)
    bwd_ms = phase_ms(bwd_sets, binding.BWD_PHASES) if do_bwd else {}
    fwd_total = float(np.mean([hev.elapsed_ms(s[0], s[-1]) for s in fwd_sets]))
    bwd_total = float(np.mean([hev.elapsed_ms(s[0], s[-1]) for s in bwd_sets])) if do_bwd else 0.0

    F = tile_flops(d)
    # algorithmic flops per launch: 2*32*32*D per 32x32 score tile, times the tiles the kernel's own counters report.
    # The list kernels' finish / row / key kernels are gathers over a few entries per row: no tile work.
    algo = {
        "fwd_lists": F * sd["fwd_list_qk"],
        "fwd_finish": 0.0,
        "fwd_tiled": F * (sd["fwd_qk_max"] + sd["fwd_qk_solve"] + sd["fwd_qk_pv"] + sd["fwd_pv_tiles"]),
        "bwd_lists": F * sd["bwd_list_qk"],
        "bwd_rows": 0.0,
        "bwd_keys": 0.0,
        "bwd_mask": F * sd["bwd_qk_mask"],
        "bwd_dq": F * 4 * sd["bwd_dq_tiles"],
        "bwd_dkv": F * 4 * sd["bwd_dkv_tiles"],
    }
    kernel_ms = {"fwd_lists": fwd_ms["lists"], "fwd_finish": fwd_ms["finish"], "fwd_tiled": fwd_ms["tiled"]}
    if do_bwd:
        kernel_ms.update(bwd_lists=bwd_ms["lists"], bwd_rows=bwd_ms["rows"], bwd_keys=bwd_ms["keys"],
                         bwd_mask=bwd_ms["mask"], bwd_dq=bwd_ms["dq"], bwd_dkv=bwd_ms["dkv"])
    # the roofline object describes the longest kernel among those that do tile (MFMA) work
    dominant = max((k for k in kernel_ms if algo[k] > 0), key=kernel_ms.get, default=max(kernel_ms, key=kernel_ms.get))
    achieved = algo[dominant] / (kernel_ms[dominant] * 1e-3) / 1e12
    total_exec = sum(algo[k] for k in kernel_ms)

    dense_flops = synth.dense_equiv_flops(B, H, n, d, True, False) + (
        synth.dense_equiv_flops(B, H, n, d, True, True) if do_bwd else 0.0)
    value = dense_flops / (ms_per_step * 1e-3) / 1e12
    vis = max(sd["fwd_tiles_visible"], 1)

    result = {
        "metric": "entmax attention fwd+bwd dense-equivalent TFLOP/s at n=4096 (tokens/s and fwd at n=32768 alongside)",
        "value": value,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if cfg["dtype"] == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": "%s: B=%d H=%d n=%d d=%d %s causal alpha=%g ASEntmax per-head scale, %g%% planted keys, %s"
                               % (args.workload, B, H, n, d, cfg["dtype"], alpha, 100 * cfg["planted"],
                                  "fwd+bwd" if do_bwd else "fwd"),
                   "B": B, "H": H, "n": n, "d": d, "alpha": alpha, "tile": "32x32"},
        "tokens_per_s": B * n / (ms_per_step * 1e-3),
        "fwd_ms": fwd_total,
        "bwd_ms": bwd_total,
        "kernel_ms": kernel_ms,
        "phase_ms": {"fwd": fwd_ms, "bwd": bwd_ms},
        "executed_tflops": total_exec / (sum(kernel_ms.values()) * 1e-3) / 1e12,
        "frac_bf16_mfma_peak_executed": total_exec / (sum(kernel_ms.values()) * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        # tiles that can hold a non-zero probability: candidate tiles of the list kernel (an upper bound of the
        # non-zero tiles) plus the P.V tiles the tiled kernel executed
        "tile_skip_rate_fwd": 1.0 - (sd["fwd_cand_tiles"] + sd["fwd_pv_tiles"]) / vis,
        "list_blocks_fraction": sd["fwd_sparse_blocks"] / max(B * H * ((n + 127) // 128), 1),
        "support_per_row": sd["fwd_support"] / max(B * H * n, 1),
        "candidates_per_row": sd["fwd_candidates"] / max(B * H * n, 1),
        "solve_sweeps_per_tiled_block": sd["fwd_solve_sweeps"] / max(sd["fwd_blocks"], 1),
        "tile_stats": sd,
        "roofline": {"bound": "mfma", "kernel": dominant, "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                     "traffic": MEASURED_HBM_BYTES_C3.get(dominant) if args.workload == "c3" else None},
    }

    if not args.no_c4 and args.workload == "c3":
        # forward only at 8x the training length (n = 32768), same counters
        del ws
        data4, cfg4, t4 = upload("c4", want_dO=False)
        kw4 = dict(alpha=cfg4["alpha"], beta=t4["beta"], gamma=t4["gamma"], delta=data4["delta"], causal=True)
        prm4 = binding.make_params(t4["Q"], t4["K"], cfg4["alpha"], data4["delta"], True, t4["beta"], 0)
        ws4 = torch.empty(binding.workspace_bytes(prm4, 0), dtype=torch.uint8, device=dev)
        out4 = torch.empty_like(t4["Q"])
        tau4 = torch.empty(cfg4["B"], cfg4["H"], cfg4["n"], dtype=torch.float32, device=dev)
        st4 = binding.new_stats(dev)
        binding.entmax_attn_fwd(t4["Q"], t4["K"], t4["V"], out=out4, tau=tau4, workspace=ws4, stats=st4, **kw4)
        torch.cuda.synchronize()
        sd4 = binding.stats_dict(st4)
        k4 = max(3, args.steps // 4)
        ev4 = [hev.make(binding.FWD_NUM_PHASES + 1) for _ in range(k4)]
        torch.cuda.synchronize()
        ta = time.perf_counter()
        for k in range(k4):
            binding.entmax_attn_fwd(t4["Q"], t4["K"], t4["V"], out=out4, tau=tau4, workspace=ws4,
                                    phase_events=ev4[k], **kw4)
        torch.cuda.synchronize()
        tb = time.perf_counter()
        ms4 = (tb - ta) * 1e3 / k4
        main4 = float(np.mean([hev.elapsed_ms(s[0], s[binding.FWD_NUM_PHASES]) for s in ev4]))
        F4 = tile_flops(cfg4["d"])
        algo4 = F4 * (sd4["fwd_list_qk"] + sd4["fwd_qk_max"] + sd4["fwd_qk_solve"] + sd4["fwd_qk_pv"] + sd4["fwd_pv_tiles"])
        dense4 = synth.dense_equiv_flops(cfg4["B"], cfg4["H"], cfg4["n"], cfg4["d"], True, False)
        result["fwd_n32768"] = {
            "workload": "c4: B=1 H=12 n=32768 d=64 bf16 causal alpha=1.5 ASEntmax scale, 5% planted keys, fwd",
            "steps": k4, "ms": ms4, "dense_equiv_tflops": dense4 / (ms4 * 1e-3) / 1e12,
            "tokens_per_s": cfg4["B"] * cfg4["n"] / (ms4 * 1e-3),
            "kernels_ms": main4, "executed_tflops": algo4 / (main4 * 1e-3) / 1e12,
            "frac_bf16_mfma_peak_executed": algo4 / (main4 * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "tile_skip_rate": 1.0 - (sd4["fwd_cand_tiles"] + sd4["fwd_pv_tiles"]) / max(sd4["fwd_tiles_visible"], 1),
            "list_blocks_fraction": sd4["fwd_sparse_blocks"] / max(cfg4["B"] * cfg4["H"] * ((cfg4["n"] + 127) // 128), 1),
            "support_per_row": sd4["fwd_support"] / max(cfg4["B"] * cfg4["H"] * cfg4["n"], 1),
            "candidates_per_row": sd4["fwd_candidates"] / max(cfg4["B"] * cfg4["H"] * cfg4["n"], 1),
            "tile_stats": {k: v for k, v in sd4.items() if k.startswith("fwd")},
        }
    if not args.no_decode and args.workload == "c3":
        # decode shapes: a few new query rows against a 32768-key cache; bound by one read of K from HBM
        result["decode_nk32768"] = {}
        for nq in (1, 8):
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
                "roofline": {"bound": "hbm", "kernel": "decode_scores", "achieved": algo_bytes / (scores_ms * 1e-3) / 1e9,
                             "peak": 8000.0, "unit": "GB/s", "frac": algo_bytes / (scores_ms * 1e-3) / 1e9 / 8000.0},
            }
            del td, wsd, kcopies
    hev.close()

    if not args.no_cpu_baseline:
        # the fp64 oracle as it stands, on a bounded sample of the same workload (first batches only)
        from oracle import oracle
        bs = min(B, 2)
        sub = {k: data[k][:bs] for k in ("Q", "K", "V", "dO")}
        okw = dict(beta=data["beta"], gamma=data["gamma"], delta=data["delta"], causal=True)
        c0 = time.perf_counter()
        oracle.attn_fwd(sub["Q"], sub["K"], sub["V"], alpha, **okw)
        if do_bwd:
            oracle.attn_bwd(sub["Q"], sub["K"], sub["V"], sub["dO"], alpha, **okw)
        c1 = time.perf_counter()
        sample_flops = dense_flops * bs / B
        result["cpu_baseline"] = {
            "value": sample_flops / (c1 - c0) / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": "fp64 oracle %s on the first %d of %d batches (%d heads, n=%d), %.1f s wall"
                      % ("fwd+bwd" if do_bwd else "fwd", bs, B, bs * H, n, c1 - c0),
            "tokens_per_s": bs * n / (c1 - c0),
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
