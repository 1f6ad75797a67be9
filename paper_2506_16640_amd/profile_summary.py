"""Turns rocprofv3 output of a bench.py run into the short summaries kept under profiles/.

  python -m paper_2506_16640_amd.profile_summary trace  <kernel_stats.csv> <bench.json> <out.md> --title T --command C
  python -m paper_2506_16640_amd.profile_summary pmc    <stats.csv> <out.md> --counters DIR [DIR ...]
                                                       [--traffic-out profiles/hbm_traffic_<workload>.txt] --title T --command C

`trace` tabulates the per-kernel durations of a `rocprofv3 --kernel-trace --stats` run next to bench.py's own
event-based figures of the same run.  `pmc` averages the counters of `rocprofv3 --pmc ...` runs per kernel
(one directory per counter set), derives matrix-core utilisation and instruction mix, and -- when FETCH_SIZE
and WRITE_SIZE were collected -- HBM bytes per launch, calibrated on torch's fp32 -> bf16 conversion kernel of
known size that bench.py's upload of the inputs runs; `--traffic-out` writes those bytes as the table
bench.py reads for `roofline.traffic`.
"""
import argparse
import collections
import csv
import glob
import json
import os

# bench.py's name of each kernel
BENCH_NAMES = collections.OrderedDict([
    ("fwd_lists_kernel", "fwd_lists"), ("fwd_lists_pair_kernel", "fwd_lists"), ("fwd_finish_kernel", "fwd_finish"), ("fwd_kernel", "fwd_tiled"),
    ("bwd_lists_kernel", "bwd_lists"), ("bwd_rows_kernel", "bwd_rows"), ("bwd_keys_kernel", "bwd_keys"),
    ("bwd_dq_kernel", "bwd_dq"), ("bwd_dkv_kernel", "bwd_dkv"),
    ("key_offsets_kernel", "key_offsets"), ("decode_scores_kernel", "decode_scores"),
    ("decode_scores_mfma_kernel", "decode_scores_mfma"), ("scale_proj_fwd_kernel", "scale_proj_fwd"),
    ("scale_proj_bwd_kernel", "scale_proj_bwd"), ("scale_proj_reduce_kernel", "scale_proj_reduce"),
    ("decode_solve_kernel", "decode_solve"),
])
CALIBRATION_KERNEL = "bfloat16_copy_kernel"


def short(name):
    return name.replace("(anonymous namespace)::", "").split("(")[0].replace("void ", "")


def ours(kernel):
    return "entmax::" in kernel or "scale_proj_" in kernel


def bench_name(kernel):
    for k, v in BENCH_NAMES.items():
        if "::" + k + "<" in kernel or kernel.endswith("::" + k):
            return v
    return None


def read_stats(path):
    rows = []
    for r in csv.DictReader(open(path)):
        rows.append(dict(name=short(r["Name"]), calls=int(r["Calls"]), avg_us=float(r["AverageNs"]) / 1e3,
                         min_us=float(r["MinNs"]) / 1e3, max_us=float(r["MaxNs"]) / 1e3, pct=r["Percentage"]))
    return rows


def collect_counters(dirs):
    """Mean counter values per kernel, and for the calibration kernel (torch's fp32 -> bf16 conversion: a thread
    converts eight elements) the totals of counter value and element count per counter."""
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    cal = collections.defaultdict(lambda: [0.0, 0.0])
    for d in dirs:
        for f in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
            for row in csv.DictReader(open(f)):
                name = short(row["Kernel_Name"])
                acc[name][row["Counter_Name"]].append(float(row["Counter_Value"]))
                if CALIBRATION_KERNEL in name:
                    cal[row["Counter_Name"]][0] += float(row["Counter_Value"])
                    cal[row["Counter_Name"]][1] += 8.0 * float(row["Grid_Size"])
    return {k: {c: sum(v) / len(v) for c, v in cs.items()} for k, cs in acc.items()}, cal


def cmd_trace(a):
    rows = read_stats(a.stats)
    b = json.load(open(a.bench))
    with open(a.out, "w") as f:
        f.write("# rocprofv3 kernel-trace summary: %s\n\n" % a.title)
        f.write("Command (repository root, one MI355X, `export TMPDIR=/tmp`):\n\n    %s\n\n" % a.command)
        f.write("Workload: " + b["config"]["workload"] + "\n\n")
        f.write("| kernel | calls | avg us | min us | max us | % |\n|---|---|---|---|---|---|\n")
        for r in rows:
            if ours(r["name"]):
                f.write("| `%s` | %d | %.1f | %.1f | %.1f | %s |\n" % (r["name"], r["calls"], r["avg_us"], r["min_us"],
                                                                     r["max_us"], r["pct"]))
        f.write("\nbench.py's own figures in the same (profiled) run, from hipEvents recorded between the phases:\n\n")
        f.write("    ms_per_step = %.4f, tokens/s = %.4g\n" % (b["ms_per_step"], b["value"]))
        f.write("    kernel_ms = " + json.dumps(b["kernel_ms"]) + "\n")
        f.write("    roofline = " + json.dumps(b["roofline"]) + "\n")
        f.write("    mfma_peak_measured_tflops = %.1f\n" % b.get("mfma_peak_measured_tflops", float("nan")))
        f.write("    tile_stats = " + json.dumps(b["tile_stats"]) + "\n")
        for key in ("other_workloads", "decode_nk32768", "scale_projection"):
            if key in b:
                f.write("    %s = %s\n" % (key, json.dumps(b[key])))


def cmd_pmc(a):
    dur = {r["name"]: r["avg_us"] for r in read_stats(a.stats)}
    ctr, calsum = collect_counters(a.counters)
    with open(a.out, "w") as f:
        f.write("# rocprofv3 counter summary: %s\n\n" % a.title)
        f.write("Commands (repository root, one MI355X, `export TMPDIR=/tmp`), one counter set per run:\n\n")
        for line in a.command:
            f.write("    %s\n" % line)
        f.write("\nValues are means per dispatch.  Kernel durations are those of the kernel-trace run of the same build.\n\n")
        f.write("## Matrix-core utilisation and instruction mix\n\n")
        f.write("`mfma util` = SQ_VALU_MFMA_BUSY_CYCLES / (duration x 2.4 GHz x 1024 SIMDs).  SQ_WAVE_CYCLES, SQ_WAIT_* and "
                "SQ_ACTIVE_* count in units of four cycles.\n\n")
        f.write("| kernel | avg us | MFMA insts | mfma util | VALU/MFMA | SALU/MFMA | LDS insts | VMEM insts | wait any / wave "
                "cycles | active / wave cycles | LDS bank conflicts |\n|---|---|---|---|---|---|---|---|---|---|---|\n")
        for k in sorted(ctr, key=lambda k: -dur.get(k, 0)):
            c = ctr[k]
            if not ours(k) or k not in dur or "SQ_WAVE_CYCLES" not in c:
                continue
            m = c.get("SQ_INSTS_MFMA", 0)
            util = c.get("SQ_VALU_MFMA_BUSY_CYCLES", 0) / (dur[k] * 1e-6 * 2.4e9 * 1024)
            wc = max(c.get("SQ_WAVE_CYCLES", 1), 1)
            f.write("| `%s` | %.1f | %.3g | %.3f | %.1f | %.1f | %.3g | %.3g | %.2f | %.2f | %.0f |\n" % (
                k, dur[k], m, util, c.get("SQ_INSTS_VALU", 0) / m if m else 0, c.get("SQ_INSTS_SALU", 0) / m if m else 0,
                c.get("SQ_INSTS_LDS", 0), c.get("SQ_INSTS_VMEM", 0), c.get("SQ_WAIT_ANY", 0) / wc,
                c.get("SQ_ACTIVE_INST_ANY", 0) / wc, c.get("SQ_LDS_BANK_CONFLICT", 0)))
        if calsum.get("FETCH_SIZE", [0, 0])[0] > 0 and calsum.get("WRITE_SIZE", [0, 0])[0] > 0:
            ff = calsum["FETCH_SIZE"][1] * 4 / 1024.0 / calsum["FETCH_SIZE"][0]
            wf = calsum["WRITE_SIZE"][1] * 2 / 1024.0 / calsum["WRITE_SIZE"][0]
            f.write("\n## HBM traffic per launch\n\n")
            f.write("Calibration: the same runs contain bench.py's upload conversions (`at::native::bfloat16_copy_kernel_cuda`, "
                    "fp32 -> bf16, eight elements per thread of its grid: 4 bytes read and 2 written per element).  Over all of "
                    "them FETCH_SIZE reads %.0f for %.0f KiB (factor %.3f), WRITE_SIZE %.0f for %.0f KiB (factor %.3f).\n\n"
                    % (calsum["FETCH_SIZE"][0], calsum["FETCH_SIZE"][1] * 4 / 1024.0, ff, calsum["WRITE_SIZE"][0],
                       calsum["WRITE_SIZE"][1] * 2 / 1024.0, wf))
            f.write("| kernel | FETCH_SIZE | WRITE_SIZE | read MB | written MB | total MB | avg us | HBM GB/s |\n"
                    "|---|---|---|---|---|---|---|---|\n")
            table = []
            for k in sorted(ctr, key=lambda k: -dur.get(k, 0)):
                c = ctr[k]
                if not ours(k) or k not in dur or "FETCH_SIZE" not in c or "WRITE_SIZE" not in c:
                    continue
                rd = c["FETCH_SIZE"] * ff * 1024 / 1e6
                wr = c["WRITE_SIZE"] * wf * 1024 / 1e6
                f.write("| `%s` | %.1f | %.1f | %.1f | %.1f | %.1f | %.1f | %.0f |\n" % (
                    k, c["FETCH_SIZE"], c["WRITE_SIZE"], rd, wr, rd + wr, dur[k], (rd + wr) / dur[k] * 1e3))
                if bench_name(k):
                    table.append((bench_name(k), (rd + wr) * 1e6, k))
            if a.traffic_out:
                with open(a.traffic_out, "w") as t:
                    t.write("# HBM bytes per launch (calibrated FETCH_SIZE + WRITE_SIZE), written by\n"
                            "# python -m paper_2506_16640_amd.profile_summary pmc; see %s\n" % os.path.basename(a.out))
                    t.write("# bench.py name   bytes   kernel\n")
                    for nm, by, k in table:
                        t.write("%s %.0f %s\n" % (nm, by, k.replace(" ", "")))


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    t = sub.add_parser("trace")
    t.add_argument("stats")
    t.add_argument("bench")
    t.add_argument("out")
    t.add_argument("--title", required=True)
    t.add_argument("--command", required=True)
    p = sub.add_parser("pmc")
    p.add_argument("stats")
    p.add_argument("out")
    p.add_argument("--counters", nargs="+", required=True)
    p.add_argument("--traffic-out", default=None)
    p.add_argument("--title", required=True)
    p.add_argument("--command", action="append", default=[])
    a = ap.parse_args()
    (cmd_trace if a.cmd == "trace" else cmd_pmc)(a)


if __name__ == "__main__":
    main()
