"""Writes the text summaries under profiles/ from raw rocprofv3 output.

The raw output (CSV files of `rocprofv3 --kernel-trace --stats` and `--pmc` runs of bench.py) is
produced on the GPU machine by the commands that each summary quotes; this script only reads those
files and the JSON line bench.py printed in the same run.  Usage, from the repository root:

    python -m paper_2108_09413_amd.profile_report --raw <directory>

where the directory holds what the quoted commands wrote: stats/ fetch/ write/ mfma/ fp_stats/
(rocprofv3 -d targets) and the *.log files with bench.py's output (stats.log, fp_stats.log).
Missing parts are skipped.  The summaries quote the commands with the directory as given here.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import hashlib
import json
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PRE = "cd /tmp && export TMPDIR=/tmp && cd <repo> && "
BENCH_STATS = "python bench.py --steps 2 --warmup 1 --no-cpu-baseline --no-other-configs --no-comparison-systems"
BENCH_PMC = ("python bench.py --steps 1 --warmup 0 --n 1236 --no-cpu-baseline --no-other-configs --no-comparison-systems "
             "--profile-every 0")
BENCH_FP = "python bench.py --system fp --steps 1"
MODES = {"0": "head", "1": "block", "2": "block + projection"}


def sources_sha256() -> str:
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(ROOT, "paper_2108_09413_amd", "csrc", "*.*"))):
        if path.endswith((".hip", ".h", ".cpp")):
            h.update(os.path.basename(path).encode())
            h.update(open(path, "rb").read())
    return h.hexdigest()


def library_name(profiler_name: str) -> str:
    """The name the library's timing report uses for a kernel as the profiler prints it."""
    n = profiler_name.replace("void ", "").replace("isr::", "").replace("(anonymous namespace)::", "")
    n = re.sub(r"\(.*\)$", "", n)
    m = re.match(r"conv_dma_kernel<(\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (?:true|false), (\d+), (\d+)(?:, (?:true|false))?>", n)
    if m:
        return "conv_dma_kernel<%s, %s, %s, %s, %s, %s, %sx%s>" % m.groups()
    m = re.match(r"conv_patch_kernel<(\d+), (\d+), \d+, (?:true|false), (?:true|false)>", n)
    if m:
        return "conv_patch_kernel<%s, 256, %s>" % m.groups()      # channels x pixels of the tile, K bytes per step
    if re.match(r"proj_expand_reduce_kernel<(?:true|false)>", n):
        return "proj_expand_reduce_kernel<256, 128, 512, 128>"     # block input, middle, block and next middle channels
    if re.match(r"expand_reduce1024_kernel<(?:true|false)>", n):
        return "expand_reduce_kernel<256, 1024, 256>"
    if re.match(r"expand_reduce256_kernel<(?:true|false)>", n):
        return "expand_reduce_kernel<128, 512, 256>"
    if re.match(r"expand_reduce_kernel<(?:true|false)>", n):
        return "expand_reduce_kernel<128, 512, 128>"               # middle, block and next middle channels
    m = re.match(r"bottleneck_kernel<(\d), (true|false)>", n)
    if m:
        return "bottleneck_kernel<%s, %s>" % (MODES[m.group(1)], m.group(2))
    m = re.match(r"fconv_kernel<(\d), (\d), (\d), (\d)>", n)
    if m:
        mt, nt, wm, wn = map(int, m.groups())
        return "fconv_kernel<%d x %d>" % (32 * mt * wm, 32 * nt * wn)
    if n == "stem_pool_kernel":
        return "stem_pool_kernel (+noise)"      # the default plan of the 224 x 224 workload draws the noise in this kernel
    return n


def is_conv(name: str) -> bool:
    return name.startswith(("conv_dma_kernel", "conv_patch_kernel", "expand_reduce_kernel", "proj_expand_reduce_kernel", "bottleneck_kernel", "stem_pool_kernel", "fconv_kernel"))


def last_json(path):
    try:
        lines = [l for l in open(path) if l.startswith("{")]
        return json.loads(lines[-1]) if lines else None
    except OSError:
        return None


def find(dirname, suffix):
    hits = glob.glob(os.path.join(dirname, "**", "*" + suffix), recursive=True)
    return hits[0] if hits else None


RAW = "<raw>"   # the raw-output directory as named on the command line; quoted in the commands of each summary


def kernel_stats(raw, sub, out_name, title, command, bench_log, peak, unit):
    path = find(os.path.join(raw, sub), "_kernel_stats.csv")
    if not path:
        return
    rows = list(csv.DictReader(open(path)))
    bench = last_json(os.path.join(raw, bench_log))
    lines = ["# " + title, "", "Command (on the MI355X box, from the repository root):", "",
             "    " + PRE + command, "", "sources_sha256: " + sources_sha256(), "",
             "| kernel (profiler name) | name in the library's timing report | calls | total ms | avg us | % |", "|---|---|---|---|---|---|"]
    for r in rows:
        if float(r["Percentage"]) < 0.05:
            continue
        short = r["Name"].replace("void ", "").replace("isr::", "").replace("(anonymous namespace)::", "")
        lines.append("| `%s` | `%s` | %s | %.1f | %.2f | %s |" % (re.sub(r"\(.*\)$", "", short), library_name(r["Name"]), r["Calls"],
                                                                    int(r["TotalDurationNs"]) / 1e6, float(r["AverageNs"]) / 1e3, r["Percentage"]))
    conv = [r for r in rows if is_conv(library_name(r["Name"]))]
    tot = sum(int(r["TotalDurationNs"]) for r in conv)
    calls = sum(int(r["Calls"]) for r in conv)
    allk = sum(int(r["TotalDurationNs"]) for r in rows if "isr::" in r["Name"])
    lines += ["", "Convolution kernels together: %d launches, %.1f ms (%.1f %% of the library's kernel time), average %.2f us per launch."
              % (calls, tot / 1e6, 100.0 * tot / max(allk, 1), tot / max(calls, 1) / 1e3)]
    if bench and bench.get("roofline"):
        rf = bench["roofline"]
        prow = [r for r in rows if library_name(r["Name"]) == rf["kernel"]]
        pavg = sum(int(r["TotalDurationNs"]) for r in prow) / max(sum(int(r["Calls"]) for r in prow), 1) / 1e3
        lines += ["", "The same run of bench.py printed (HIP events on the library's stream around every launch of each timed chunk):",
                  "dominant kernel `%s`: %d timed launches, average %.2f us, %.1f %s algorithmic = %.1f %% of the %s %s peak; "
                  "the profiler's average over all launches of that instance (ragged last chunks included): %.2f us."
                  % (rf["kernel"], rf["launches_timed"], rf["avg_launch_us"], rf["achieved"], unit, 100 * rf["frac"], peak, unit, pavg),
                  "Whole path in that run: %.0f inferences/s." % bench["value"], "",
                  "Per kernel instance, from that run's JSON line (`per_kernel`):", "",
                  "| kernel instance | timed launches | avg us | %s | time share |" % unit, "|---|---|---|---|---|"]
        for r in bench.get("per_kernel") or []:
            lines.append("| `%s` | %d | %.2f | %s | %.4f |" % (r["name"], r["launches"], r["avg_us"],
                                                              "-" if r.get("TOP/s") is None else "%.1f" % r["TOP/s"], r["time_share"]))
    lines.append("")
    open(os.path.join(ROOT, "profiles", out_name), "w").write("\n".join(lines))
    print("wrote", out_name)


def counter_table(path, counter):
    """{library kernel name: [dispatch values]} of one counter."""
    out = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] == counter:
            out[library_name(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return out


def hbm_traffic(raw, chunk=668, n=1236, n0=100):
    fpath = find(os.path.join(raw, "fetch"), "_counter_collection.csv")
    wpath = find(os.path.join(raw, "write"), "_counter_collection.csv")
    if not (fpath and wpath):
        return
    f, w = counter_table(fpath, "FETCH_SIZE"), counter_table(wpath, "WRITE_SIZE")
    cmd = BENCH_PMC + " --copy-calibration-mib 2048"
    ninf = n + n0 + 8
    lines = ["# HBM traffic of the ResNet-50 int8 certification path (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)", "",
             "Commands (two runs, one counter each):", "",
             "    " + PRE + "rocprofv3 --pmc FETCH_SIZE -d " + RAW + "/fetch -o f --output-format csv -- " + cmd,
             "    " + PRE + "rocprofv3 --pmc WRITE_SIZE -d " + RAW + "/write -o w --output-format csv -- " + cmd, "",
             "sources_sha256: " + sources_sha256(), "",
             "Workload: one certification with n0=%d, n=%d (%d noisy inferences = two full chunks of %d) plus the 8 one-sample "
             "warm-up calls that upload the noise tables." % (n0, n, n + n0, chunk),
             "Counter unit: KiB per dispatch, summed here over all dispatches of a kernel instance (names as in the library's timing report).", "",
             "| kernel | dispatches | FETCH_SIZE KiB | WRITE_SIZE KiB |", "|---|---|---|---|"]
    names = sorted(set(f) | set(w), key=lambda k: -(sum(f[k]) + sum(w[k])))
    for k in names:
        if sum(f[k]) + sum(w[k]) >= 1000:
            lines.append("| `%s` | %d | %.0f | %.0f |" % (k[:70], max(len(f[k]), len(w[k])), sum(f[k]), sum(w[k])))
    kib = 2048 * 1024.0
    cal_f = sum(v for k in f if "copyBuffer" in k for v in f[k])
    cal_w = sum(v for k in w if "copyBuffer" in k for v in w[k])
    ff, fw = cal_f / kib, cal_w / kib
    sf = ff if 0.3 < ff < 1.5 else 1.0
    sw = fw if 0.3 < fw < 1.5 else 1.0
    lines += ["", "Calibration: the plain 2048 MiB device-to-device copy (`__amd_rocclr_copyBuffer`, all its dispatches; random source, "
              "evicted from the caches first) reads %.0f KiB and writes %.0f KiB by these counters for %.0f KiB each way:" % (cal_f, cal_w, kib),
              "factors FETCH_SIZE %.3f, WRITE_SIZE %.3f (counter / true bytes); the byte figures below are the raw counters divided by these." % (ff, fw), ""]
    cf = sum(sum(v) for k, v in f.items() if is_conv(k)) / sf
    cw = sum(sum(v) for k, v in w.items() if is_conv(k)) / sw
    cn = sum(len(v) for k, v in w.items() if is_conv(k))
    lines += ["Convolution kernels (all instances): %d dispatches, %.0f KiB fetched, %.0f KiB written = %.2f MB read and %.2f MB written "
              "per noisy inference (%d inferences)." % (cn, cf, cw, cf * 1024 / ninf / 1e6, cw * 1024 / ninf / 1e6, ninf), "",
              "conv_hbm_bytes_per_inference: fetch=%.0f write=%.0f" % (cf * 1024 / ninf, cw * 1024 / ninf), "",
              "Bytes of one full-chunk launch of each instance (the largest dispatches of the runs above: a full chunk of %d copies; "
              "instances that serve several layers are averaged over those of at least half the largest):" % chunk, ""]
    for k in names:
        if not is_conv(k) and not k.startswith(("gap", "fc_", "noise")):
            continue
        big_f = [v for v in f[k] if v >= 0.5 * max(f[k])] if f[k] else [0.0]
        big_w = [v for v in w[k] if v >= 0.5 * max(w[k])] if w[k] else [0.0]
        lines.append("kernel_bytes_per_full_chunk_launch: `%s` dispatches=%d fetch=%.0f write=%.0f"
                     % (k, min(len(big_f), len(big_w)), sum(big_f) / len(big_f) / sf * 1024, sum(big_w) / len(big_w) / sw * 1024))
    lines.append("")
    open(os.path.join(ROOT, "profiles", "resnet50_certify_hbm_traffic.md"), "w").write("\n".join(lines))
    print("wrote resnet50_certify_hbm_traffic.md")


def mfma_utilisation(raw, chunk=668):
    path = find(os.path.join(raw, "mfma"), "_counter_collection.csv")
    if not path:
        return
    disp = collections.defaultdict(lambda: collections.defaultdict(float))
    for r in csv.DictReader(open(path)):
        disp[(library_name(r["Kernel_Name"]), r["Dispatch_Id"])][r["Counter_Name"]] += float(r["Counter_Value"])
    agg = collections.defaultdict(lambda: collections.defaultdict(float))
    cnt = collections.Counter()
    for (k, _), c in disp.items():
        cnt[k] += 1
        for name, v in c.items():
            agg[k][name] += v
    lines = ["# int8 MFMA utilisation of the convolution kernels (rocprofv3 --pmc)", "", "Command:", "",
             "    " + PRE + "rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES SQ_INSTS_VALU_MFMA_MOPS_I8 SQ_ACTIVE_INST_VALU "
             "GRBM_GUI_ACTIVE -d " + RAW + "/mfma -o m --output-format csv -- " + BENCH_PMC, "",
             "sources_sha256: " + sources_sha256(), "",
             "Workload: one certification with n0=100, n=1236 (two full chunks of %d noisy ResNet-50/224 inferences) plus 8 one-sample "
             "calls; small dispatches are included; a kernel instance covers all layers that use it." % chunk,
             "GRBM_GUI_ACTIVE is summed over the 8 XCDs, the SQ counters over all CUs.  MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / "
             "(GRBM_GUI_ACTIVE / 8 x 256 CUs x 4 SIMDs): the share of SIMD cycles in which the matrix pipe executes, i.e. the fraction "
             "of the int8 MFMA peak at the clock the chip actually ran.  int8 ops = SQ_INSTS_VALU_MFMA_MOPS_I8 x 512.", "",
             "| kernel | dispatches | GUI active cycles / 8 | MFMA busy SIMD-cycles | MFMA busy % | VALU active % | int8 Tops issued |",
             "|---|---|---|---|---|---|---|"]
    tb = tg = 0.0
    for k, c in sorted(agg.items(), key=lambda kv: -kv[1]["GRBM_GUI_ACTIVE"]):
        if not is_conv(k):
            continue
        g, b = c["GRBM_GUI_ACTIVE"] / 8, c["SQ_VALU_MFMA_BUSY_CYCLES"]
        tb += b
        tg += g
        lines.append("| `%s` | %d | %.0f | %.0f | %.1f | %.1f | %.3f |" % (k, cnt[k], g, b, 100 * b / (g * 1024),
                                                                          100 * c["SQ_ACTIVE_INST_VALU"] / (g * 1024),
                                                                          c["SQ_INSTS_VALU_MFMA_MOPS_I8"] * 512 / 1e12))
    lines += ["", "All convolution dispatches together: MFMA busy %.1f %% of the SIMD cycles of their kernels." % (100 * tb / max(tg * 1024, 1)), ""]
    open(os.path.join(ROOT, "profiles", "conv_resnet50_certify_mfma_utilisation.md"), "w").write("\n".join(lines))
    print("wrote conv_resnet50_certify_mfma_utilisation.md")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--raw", required=True, help="directory with the raw rocprofv3 output and bench.py logs")
    args = ap.parse_args()
    global RAW
    RAW = os.path.relpath(args.raw, ROOT) if os.path.isabs(args.raw) else args.raw.rstrip("/")
    kernel_stats(args.raw, "stats", "conv_resnet50_certify_kernel_stats.md",
                 "rocprofv3 kernel statistics: ResNet-50 int8 certification (bench.py headline workload)",
                 "rocprofv3 --kernel-trace --stats -d " + RAW + "/stats -o r50 --output-format csv -- " + BENCH_STATS,
                 "stats.log", 5000, "TOP/s")
    kernel_stats(args.raw, "fp_stats", "fconv_resnet50_floatrs_fp_kernel_stats.md",
                 "rocprofv3 kernel statistics: ResNet-50 FloatRS-fp comparison system (fp32 network on the fp32 MFMA)",
                 "rocprofv3 --kernel-trace --stats -d " + RAW + "/fp_stats -o fp --output-format csv -- " + BENCH_FP,
                 "fp_stats.log", 157.3, "TFLOP/s")
    hbm_traffic(args.raw)
    mfma_utilisation(args.raw)


if __name__ == "__main__":
    main()
