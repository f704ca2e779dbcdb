"""Turns the rocprofv3 output of the benchmark's profiling runs into the short text summaries kept under profiles/.

The runs themselves (on the GPU machine, from the repo root, after `cd /tmp && export TMPDIR=/tmp && cd <repo>`), for config N:

    rocprofv3 --kernel-trace --stats --output-format csv -d OUT/stats -o bench -- python3 bench.py --config N --steps 5 --warmup 2 --no-cpu-baseline > OUT/stats.log
    rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d OUT/fetch -o b -- python3 bench.py --config N --steps 2 --warmup 1 --no-cpu-baseline --calibrate-copy
    rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d OUT/write -o b -- python3 bench.py --config N --steps 2 --warmup 1 --no-cpu-baseline --calibrate-copy
    rocprofv3 --pmc <unit counters> --kernel-trace --output-format csv -d OUT/units -o b -- python3 bench.py --config N --steps 2 --warmup 1 --no-cpu-baseline

and then `python3 -m paper_2505_20524_amd.profile_summary --config N --dir OUT --out profiles`.
Only argument parsing, CSV reading and text formatting happen here; no figure is invented: everything printed is a
sum, an average or a ratio of what the profiler wrote.  bench.py reads the dominant kernel's traffic per launch back from
the traffic summary (`read_gemm_traffic`), so that the benchmark line never carries a typed-in constant.
"""
import argparse
import collections
import csv
import glob
import json
import os
import re

UNIT_COUNTERS = ("TCP_TCC_READ_REQ_sum TCP_TOTAL_CACHE_ACCESSES_sum TCP_PENDING_STALL_CYCLES_sum TCP_TCC_READ_REQ_LATENCY_sum "
                 "TA_TA_BUSY_sum TA_BUFFER_TOTAL_CYCLES_sum SQ_VALU_MFMA_BUSY_CYCLES SQ_WAVE_CYCLES SQ_WAIT_ANY SQ_ACTIVE_INST_VALU "
                 "SQ_BUSY_CYCLES GRBM_GUI_ACTIVE")
KERNELS = ("fp8_gemm_kernel", "gemm_split_reduce_kernel", "amax_batch_kernel", "quantize_batch_kernel", "amax_kernel", "quantize_transpose_kernel",
           "quantize_rows_kernel", "attn_fwd_kernel", "attn_bwd_dkdv_kernel", "attn_bwd_dq_kernel", "kurtosis_kernel", "qknorm_rows_kernel",
           "copyBuffer")
TRAFFIC_LINE = re.compile(r"= ([0-9.]+e[+-]?[0-9]+) bytes per launch")


def traffic_file(out_dir, cid):
    return os.path.join(out_dir, "bench_config%d_hbm_traffic.md" % cid)


def read_gemm_traffic(out_dir, cid):
    """Bytes per fp8_gemm_kernel launch as measured and written by `traffic_summary`, or None when there is no such summary."""
    try:
        m = TRAFFIC_LINE.search(open(traffic_file(out_dir, cid)).read())
    except OSError:
        return None
    return float(m.group(1)) if m else None


def _find(directory, name):
    hits = glob.glob(os.path.join(directory, "**", name), recursive=True)
    if not hits:
        raise FileNotFoundError("%s under %s" % (name, directory))
    return hits[0]


def _pmc(path):
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(path)):
        acc[r["Kernel_Name"]][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return acc


def _key(name):
    for s in KERNELS:
        if s in name:
            return s
    return None


def _fold(acc, counter):
    out = collections.defaultdict(list)
    for k, v in acc.items():
        if _key(k) and counter in v:
            out[_key(k)] += v[counter]
    return out


def stats_summary(cid, d, out_dir, bench_line):
    rows = list(csv.DictReader(open(_find(os.path.join(d, "stats"), "bench_kernel_stats.csv"))))
    o = ["# rocprofv3 kernel stats: bench.py, config %d\n" % cid,
         "Command (on the GPU box, from the repo root, after `cd /tmp && export TMPDIR=/tmp && cd $GRAFT_REPO_ROOT`):\n",
         "    rocprofv3 --kernel-trace --stats --output-format csv -d OUT/stats -o bench -- python3 bench.py --config %d --steps 5 --warmup 2 --no-cpu-baseline\n" % cid,
         "24 passes of the block: 12 under just-in-time scaling (2 warm-up + 5 timed + 5 with every kernel class bracketed by events) and 12 under "
         "delayed scaling (2 + 5 + 5; `fog_quantize_delayed_batch`, one launch per layer's casts: `quantize_delayed_batch_kernel`), then the side "
         "figures (kurtosis monitor, fused cast + transpose, fused producers); `bench_kernel_stats.csv`:\n",
         "| kernel | calls | total ms | avg us | % |\n|---|---|---|---|---|"]
    per = {}
    for r in rows:
        n = r["Name"].replace("(anonymous namespace)::", "").replace("void ", "")
        per[n] = (int(r["Calls"]), float(r["TotalDurationNs"]))
        if float(r["Percentage"]) < 0.05:
            continue
        o.append("| `%s` | %s | %.3f | %.1f | %.1f |" % (n[:80] + ("..." if len(n) > 80 else ""), r["Calls"], float(r["TotalDurationNs"]) / 1e6,
                                                        float(r["AverageNs"]) / 1e3, float(r["Percentage"])))

    def grp(pred):
        return sum(v[0] for k, v in per.items() if pred(k)), sum(v[1] for k, v in per.items() if pred(k))
    c, t = grp(lambda k: "fp8_gemm_kernel" in k)
    o.append("")
    if c:
        o.append("All `fp8_gemm_kernel` instantiations together: %d launches, average %.1f us per launch (kernel trace)." % (c, t / c / 1e3))
    if bench_line:
        r = bench_line["roofline"]
        o.append("bench.py's own HIP-event figure in the same run: %d launches per step, average %.1f us per launch, %.0f TFLOP/s (%.1f %% of the "
                 "%.0f TFLOP/s dense-FP8 peak); whole step %.2f ms, %.0f TFLOP/s under the profiler." % (
                     r["launches_per_step"], r["avg_launch_ms"] * 1e3, r["achieved"], r["frac"] * 100, r["peak"], bench_line["ms_per_step"], bench_line["value"]))
    o.append("")
    parts = []
    for name, pred, div in (("GEMM (split reduce included)", lambda k: "fp8_gemm_kernel" in k or "gemm_split_reduce" in k, 24),
                            ("attention forward", lambda k: "attn_fwd_kernel" in k, 24),
                            ("attention backward (row constants, dV, dK, dQ)", lambda k: "attn_bwd" in k, 24),
                            ("abs-max pass (just-in-time passes only)", lambda k: "amax_batch_kernel" in k or "amax_kernel" in k, 12),
                            ("cast pass, just-in-time", lambda k: "quantize_batch_kernel" in k or ("quantize_rows_kernel" in k and "false>" in k.split("(")[0]), 12),
                            ("cast pass with abs-max output, delayed", lambda k: "quantize_delayed_batch_kernel" in k or ("quantize_rows_kernel" in k and "true>" in k.split("(")[0]), 12)):
        c, t = grp(pred)
        if c:
            parts.append("%s %.3f ms" % (name, t / div / 1e6))
    o.append("Per pass of the block (kernel time / passes that run the kernel): " + "; ".join(parts) + ".")
    open(os.path.join(out_dir, "bench_config%d_kernel_stats.md" % cid), "w").write("\n".join(o) + "\n")


def traffic_summary(cid, d, out_dir, bench_line):
    F = _fold(_pmc(_find(os.path.join(d, "fetch"), "b_counter_collection.csv")), "FETCH_SIZE")
    W = _fold(_pmc(_find(os.path.join(d, "write"), "b_counter_collection.csv")), "WRITE_SIZE")
    cf, cw = F["copyBuffer"][0], W["copyBuffer"][0]
    sf, sw = 1048576.0 / cf, 1048576.0 / cw
    o = ["# HBM traffic per launch (rocprofv3 --pmc), bench.py config %d\n" % cid,
         "Commands (two separate runs, counters only with the kernel trace):\n",
         "    rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d OUT/fetch -o b -- python3 bench.py --config %d --steps 2 --warmup 1 --no-cpu-baseline --calibrate-copy" % cid,
         "    rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d OUT/write -o b -- python3 bench.py --config %d --steps 2 --warmup 1 --no-cpu-baseline --calibrate-copy\n" % cid,
         "`--calibrate-copy` adds one plain 1 GiB device-to-device copy (`__amd_rocclr_copyBuffer`): FETCH_SIZE read %.1f and WRITE_SIZE %.1f for 1048576 KiB "
         "moved each way, so readings are scaled by %.3f (fetch) and %.3f (write).\n" % (cf, cw, sf, sw),
         "| kernel | launches | FETCH_SIZE avg (raw) | WRITE_SIZE avg (raw) | read MB | written MB |\n|---|---|---|---|---|---|"]
    for k in KERNELS[:-1]:
        if not F[k] or not W[k]:
            continue
        fa, wa = sum(F[k]) / len(F[k]), sum(W[k]) / len(W[k])
        o.append("| `%s` | %d | %.0f | %.0f | %.1f | %.1f |" % (k, len(F[k]), fa, wa, fa * sf * 1024 / 1e6, wa * sw * 1024 / 1e6))
    if F["fp8_gemm_kernel"]:
        rd = sum(F["fp8_gemm_kernel"]) / len(F["fp8_gemm_kernel"]) * sf * 1024
        wr = sum(W["fp8_gemm_kernel"]) / len(W["fp8_gemm_kernel"]) * sw * 1024
        o.append("")
        o.append("Dominant kernel (`fp8_gemm_kernel`): %.0f MB read + %.0f MB written = %.3e bytes per launch on average." % (rd / 1e6, wr / 1e6, rd + wr))
        if bench_line:
            alg = bench_line.get("gemm_algorithmic_bytes_per_launch")
            if alg:
                o.append("The algorithmic minimum (each operand read once, C written once) averages %.1f MB per launch over the step's products: the "
                         "measured traffic is %.1fx that." % (alg / 1e6, (rd + wr) / alg))
        o.append("The counter sits between L2 and the fabric: what the memory-side cache serves is counted too, so this is an upper bound on HBM traffic.")
    open(traffic_file(out_dir, cid), "w").write("\n".join(o) + "\n")


def units_summary(cid, d, out_dir):
    acc = _pmc(_find(os.path.join(d, "units"), "b_counter_collection.csv"))
    kn = ("fp8_gemm_kernel", "attn_fwd_kernel", "dkdv_kernel<true, 1>", "dkdv_kernel<true, 2>", "dkdv_kernel<true, 0>", "attn_bwd_dq_kernel")
    disp = {"fp8_gemm_kernel": "fp8_gemm_kernel", "attn_fwd_kernel": "attn_fwd_kernel", "dkdv_kernel<true, 1>": "attn_bwd_dkdv (dV)",
            "dkdv_kernel<true, 2>": "attn_bwd_dkdv (dK)", "dkdv_kernel<true, 0>": "attn_bwd_dkdv (dK + dV)", "attn_bwd_dq_kernel": "attn_bwd_dq_kernel"}
    A = collections.defaultdict(lambda: collections.defaultdict(list))
    for k, v in acc.items():
        for n in kn:
            if n in k and "split_reduce" not in k:
                for c, vals in v.items():
                    A[n][c] += vals
    kn = [n for n in kn if A[n]]
    avg = lambda n, c: sum(A[n][c]) / len(A[n][c])
    cs = UNIT_COUNTERS.split()
    o = ["# Execution-unit counters per launch (rocprofv3 --pmc), bench.py config %d\n" % cid,
         "Command (one run; 8 SQ / 4 TCP / 2 TA / 2 GRBM counters per run is the hardware limit):\n",
         "    rocprofv3 --pmc %s --kernel-trace --output-format csv -d OUT/units -o b -- python3 bench.py --config %d --steps 2 --warmup 1 --no-cpu-baseline\n" % (UNIT_COUNTERS, cid),
         "Averages per launch over the run's launches of each kernel (sums over the chip's 8 XCDs / 256 CUs / 1024 SIMDs):\n",
         "| counter | " + " | ".join("`%s`" % disp[n] for n in kn) + " |", "|---|" + "---|" * len(kn)]
    for c in cs:
        o.append("| %s | " % c + " | ".join("%.4g" % avg(n, c) for n in kn) + " |")
    o.append("")
    o.append("Derived (GRBM_GUI_ACTIVE counts every XCD: / 8 gives shader cycles per launch; SQ_VALU_MFMA_BUSY_CYCLES / 1024 gives busy cycles per SIMD; "
             "the launch durations come from the kernel trace of the same run):\n")
    trace = list(csv.DictReader(open(_find(os.path.join(d, "units"), "b_kernel_trace.csv"))))
    dur = collections.defaultdict(list)
    for r in trace:
        for n in kn:
            if n in r["Kernel_Name"] and "split_reduce" not in r["Kernel_Name"]:
                dur[n].append(float(r["End_Timestamp"]) - float(r["Start_Timestamp"]))
    o.append("| | " + " | ".join("`%s`" % disp[n] for n in kn) + " |")
    o.append("|---|" + "---|" * len(kn))
    o.append("| launch duration under the counters, us | " + " | ".join("%.1f" % (sum(dur[n]) / len(dur[n]) / 1e3) for n in kn) + " |")
    o.append("| shader clock = cycles / duration, GHz | " + " | ".join("%.2f" % (avg(n, "GRBM_GUI_ACTIVE") / 8 / (sum(dur[n]) / len(dur[n]))) for n in kn) + " |")
    o.append("| matrix-core busy fraction of those cycles | " + " | ".join("%.1f %%" % (100 * avg(n, "SQ_VALU_MFMA_BUSY_CYCLES") / 1024 / (avg(n, "GRBM_GUI_ACTIVE") / 8)) for n in kn) + " |")
    o.append("| wave time waiting on s_waitcnt (SQ_WAIT_ANY / SQ_WAVE_CYCLES) | " + " | ".join("%.0f %%" % (100 * avg(n, "SQ_WAIT_ANY") / avg(n, "SQ_WAVE_CYCLES")) for n in kn) + " |")
    o.append("| wave time issuing vector ALU incl. matrix instructions (SQ_ACTIVE_INST_VALU / SQ_WAVE_CYCLES) | " + " | ".join("%.0f %%" % (100 * avg(n, "SQ_ACTIVE_INST_VALU") / avg(n, "SQ_WAVE_CYCLES")) for n in kn) + " |")
    o.append("| resident waves per SIMD (4 SQ_WAVE_CYCLES / (1024 x cycles)) | " + " | ".join("%.2f" % (4 * avg(n, "SQ_WAVE_CYCLES") / (1024 * avg(n, "GRBM_GUI_ACTIVE") / 8)) for n in kn) + " |")
    o.append("| bytes per L2 read request (16 B x 64 lanes x TA wavefronts / requests) | " + " | ".join("%.0f" % (avg(n, "TA_BUFFER_TOTAL_CYCLES_sum") / 16 * 1024 / avg(n, "TCP_TCC_READ_REQ_sum")) for n in kn) + " |")
    o.append("| mean L2 read latency seen by the vector cache, cycles | " + " | ".join("%.0f" % (avg(n, "TCP_TCC_READ_REQ_LATENCY_sum") / avg(n, "TCP_TCC_READ_REQ_sum")) for n in kn) + " |")
    open(os.path.join(out_dir, "bench_config%d_unit_counters.md" % cid), "w").write("\n".join(o) + "\n")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=5)
    ap.add_argument("--dir", required=True, help="directory with the stats / fetch / write / units sub-directories the profiler wrote")
    ap.add_argument("--out", default="profiles")
    args = ap.parse_args()
    bench_line = None
    log = os.path.join(args.dir, "stats.log")
    if os.path.exists(log):
        m = re.search(r'\{"metric.*', open(log).read())
        if m:
            bench_line = json.loads(m.group(0))
    for sub, fn in (("stats", lambda: stats_summary(args.config, args.dir, args.out, bench_line)),
                    ("fetch", lambda: traffic_summary(args.config, args.dir, args.out, bench_line)),
                    ("units", lambda: units_summary(args.config, args.dir, args.out))):
        if os.path.isdir(os.path.join(args.dir, sub)):
            fn()
            print("wrote the %s summary of config %d" % (sub, args.config))


if __name__ == "__main__":
    main()
