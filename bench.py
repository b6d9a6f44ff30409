#!/usr/bin/env python3
"""Benchmark of the integer randomized smoothing hot path on one MI355X.

A step is one certification (Alg. 1 of the paper: n0 selection + n estimation
noisy inferences, votes, decision) of one (image, sigma) pair of the headline
workload: the ResNet-50 int8 network on a 3x224x224 image with n = 100000.
Images, weights and tables are resident in HBM before the timed region.

Prints one JSON line: whole-job noisy inferences/s; the roofline record of the
dominant kernel instance (the convolution kernel instance with the largest share
of the timed kernel time, timed with HIP events on the library's stream inside
the timed region) next to the aggregate over all convolution kernels and the
per-instance table; short runs of the other workload configurations; and the
CPU oracle timed on the host cores on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import glob
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0   # MI355X dense int8, published
HBM_PEAK_GBS = 8000.0

WORKLOADS = {
    # name: (config number, default chunk, oracle samples for the CPU baseline)
    # 668 samples x 14x14 pixels = 512 output tiles of 256 pixels: the deep layers fill the 256 CUs twice
    "resnet50": (4, 668, 48),
    "resnet20": (1, 8192, 2048),
    "resnet110": (2, 4096, 512),
    "tiny": (0, 1024, 1100),
}
# short runs reported next to the headline: (config, chunk, steps); a step is one certification at the config's own n0, n
OTHER_CONFIGS = ((0, 1024, 8), (1, 8192, 3), (2, 4096, 2), (3, 668, 3))


def kernel_sources_sha256() -> str:
    """Checksum of the kernel and host sources: an offline counter summary applies only to the code it was taken on."""
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(ROOT, "paper_2108_09413_amd", "csrc", "*.*"))):
        if path.endswith((".hip", ".h", ".cpp")):
            h.update(os.path.basename(path).encode())
            h.update(open(path, "rb").read())
    return h.hexdigest()


def host_cpu_info() -> dict:
    model, physical = "unknown", set()
    try:
        phys_id = None
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name") and model == "unknown":
                model = line.split(":", 1)[1].strip()
            elif line.startswith("physical id"):
                phys_id = line.split(":", 1)[1].strip()
            elif line.startswith("core id"):
                physical.add((phys_id, line.split(":", 1)[1].strip()))
    except OSError:
        pass
    return {"nproc": os.cpu_count(), "physical_cores": len(physical) or None, "model": model}


def kernel_table(stats, all_ms):
    rows = []
    for s in sorted(stats, key=lambda s: -s["total_ms"]):
        tops = s["alg_ops"] / (s["total_ms"] * 1e-3) / 1e12 if s["alg_ops"] and s["total_ms"] > 0 else None
        rows.append({"name": s["name"], "conv": s["is_conv"], "launches": s["launches"],
                     "avg_us": round(s["total_ms"] * 1e3 / s["launches"], 2),
                     "TOP/s": round(tops, 2) if tops is not None else None,
                     "frac_of_int8_peak": round(tops / INT8_MFMA_PEAK_TOPS, 4) if tops is not None else None,
                     "GB/s": round(s["alg_bytes"] / (s["total_ms"] * 1e-3) / 1e9, 1) if s["total_ms"] > 0 else None,
                     "time_share": round(s["total_ms"] / all_ms, 4) if all_ms else None})
    return rows


def conv_aggregate(stats):
    conv = [s for s in stats if s["is_conv"]]
    ms = sum(s["total_ms"] for s in conv)
    ops = sum(s["alg_ops"] for s in conv)
    launches = sum(s["launches"] for s in conv)
    return conv, ms, ops, launches


def offline_traffic():
    """Per-kernel HBM bytes per launch from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summary, or
    (None, reason) when the summary was taken on other sources than the ones in the tree."""
    path = os.path.join(ROOT, "profiles", "resnet50_certify_hbm_traffic.md")
    try:
        txt = open(path).read()
    except OSError:
        return None, "no counter summary committed"
    m = re.search(r"sources_sha256: ([0-9a-f]{64})", txt)
    if not m:
        return None, "counter summary carries no source checksum"
    if m.group(1) != kernel_sources_sha256():
        return None, "counter summary was taken on other kernel sources than this tree's (re-run the counter passes)"
    per_kernel = {}
    for name, n, fetch, write in re.findall(r"^kernel_bytes_per_full_chunk_launch: `([^`]+)` dispatches=(\d+) fetch=(\d+) write=(\d+)$", txt, re.M):
        per_kernel[name] = {"dispatches": int(n), "fetch": int(fetch), "write": int(write)}
    mt = re.search(r"conv_hbm_bytes_per_inference: fetch=(\d+) write=(\d+)", txt)
    if not per_kernel or not mt:
        return None, "counter summary has no per-kernel byte lines"
    return {"per_kernel": per_kernel, "conv_per_inference": int(mt.group(1)) + int(mt.group(2))}, os.path.relpath(path, ROOT)


def run_config(isr, synth, torch, cfg_id, chunk, steps, profile_every, n_override=0, mode="certify", batch=1, warmup=1):
    """Loads a workload, runs `warmup` + `steps` steps and returns (seconds, inferences, kernel stats, last result, context)."""
    cfg = synth.CONFIGS[cfg_id]
    n0, n = cfg["n0"], (n_override or cfg["n"])
    alpha = 0.001
    blob = synth.build_model(cfg_id)
    model = isr.isr_load_model(blob)
    isr.isr_set_workspace(model, chunk)
    n_img = min(cfg["images"], 10)
    images = [torch.from_numpy(synth.make_image(cfg_id, i + 1)).cuda() for i in range(n_img)]
    pairs = [(i, s) for i in range(n_img) for s in cfg["sigmas"]]
    for s in cfg["sigmas"]:   # noise tables for every sigma are built and uploaded before the timed region
        isr.isr_certify(model, images[0], s, 1, 1, alpha, want_counts=False)
    if mode == "predict":
        n0 = 0
    image_array = torch.stack(images)

    def step(k):
        if batch > 1:
            items = [(pairs[j % len(pairs)][0], pairs[j % len(pairs)][1], pairs[j % len(pairs)][0] + 1)
                     for j in range(k * batch, (k + 1) * batch)]
            if mode == "predict":
                return isr.isr_predict_batch(model, image_array, items, n, alpha, seed=0)[0][-1]
            return isr.isr_certify_batch(model, image_array, items, n0, n, alpha, seed=0)[0][-1]
        i, s = pairs[k % len(pairs)]
        if mode == "predict":
            return isr.isr_predict(model, images[i], s, n, alpha, seed=0, image_id=i + 1)[0]
        return isr.isr_certify(model, images[i], s, n0, n, alpha, seed=0, image_id=i + 1, want_counts=False)[0]

    for k in range(warmup):
        step(k)
    isr.isr_profile(model, profile_every)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    results = [step(warmup + k) for k in range(steps)]
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    stats = isr.isr_profile_read(model) if profile_every else []
    isr.isr_profile(model, 0)
    ctx = dict(cfg=cfg, n0=n0, n=n, n_img=n_img, alpha=alpha, blob=blob, macs=synth.model_macs(cfg_id))
    model.close()
    return dt, steps * batch * (n0 + n), stats, results[-1], ctx


FP32_MFMA_PEAK_TFLOPS = 157.3   # MI355X dense fp32 matrix peak


def run_float_system(isr, synth, torch, cfg_id, chunk, system, n, steps, profile_every=4):
    """The paper's floating-point comparison systems on the same workload: Alg. 1 with continuous
    Gaussian noise, FloatRS-quant (int8 network on the rounded input) or FloatRS-fp (fp32 network).
    One warm-up step with a short run, then `steps` timed steps of n0 + n inferences."""
    cfg = synth.CONFIGS[cfg_id]
    n0, alpha = cfg["n0"], 0.001
    model = isr.isr_load_model(synth.build_model(cfg_id))
    # fp32 tensors take four times the bytes of a chunk's int8 tensors: a four times larger workspace keeps the copies per chunk
    isr.isr_set_workspace(model, chunk * (4 if system == isr.FLOATRS_FP else 1), float_fp=(system == isr.FLOATRS_FP))
    n_img = min(cfg["images"], 10)
    images = [torch.from_numpy(synth.make_image(cfg_id, i + 1)).cuda() for i in range(n_img)]
    pairs = [(i, s) for i in range(n_img) for s in cfg["sigmas"]]
    isr.isr_float_certify(model, images[0], float(pairs[0][1]), n0, 2 * chunk, alpha, system)      # warm-up (fp32 weights are built here)
    isr.isr_profile(model, profile_every)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        i, sg = pairs[k % len(pairs)]
        last = isr.isr_float_certify(model, images[i], float(sg), n0, n, alpha, system, seed=0, image_id=i + 1)[0]
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    stats = isr.isr_profile_read(model) if profile_every else []
    isr.isr_profile(model, 0)
    fchunk = isr.isr_float_chunk(model, system)
    model.close()
    inferences = steps * (n0 + n)
    all_ms = sum(st["total_ms"] for st in stats)
    out = {"system": "FloatRS-quant" if system == isr.FLOATRS_QUANT else "FloatRS-fp", "config": cfg_id, "arch": cfg["arch"],
           "n0": n0, "n": n, "steps": steps, "chunk_samples": fchunk,
           "inferences_per_s": round(inferences / dt, 1), "ms_per_step": round(dt / steps * 1e3, 2),
           "dtype": "int8" if system == isr.FLOATRS_QUANT else "f32",
           "last_result": {"cls": last.cls, "radius": last.radius, "n_top": last.n_top}}
    if system == isr.FLOATRS_FP and all_ms > 0:
        conv = [st for st in stats if st["is_conv"]]
        dom = max(conv, key=lambda st: st["total_ms"])
        tf = dom["alg_ops"] / (dom["total_ms"] * 1e-3) / 1e12
        ops, ms = sum(st["alg_ops"] for st in conv), sum(st["total_ms"] for st in conv)
        out["roofline"] = {"bound": "mfma", "kernel": dom["name"], "achieved": round(tf, 2), "peak": FP32_MFMA_PEAK_TFLOPS,
                           "unit": "TFLOP/s", "frac": round(tf / FP32_MFMA_PEAK_TFLOPS, 4), "traffic": None,
                           "launches_timed": dom["launches"], "avg_launch_us": round(dom["total_ms"] * 1e3 / dom["launches"], 2),
                           "time_share_of_all_kernels": round(dom["total_ms"] / all_ms, 4)}
        out["all_conv_TFLOP/s"] = round(ops / (ms * 1e-3) / 1e12, 2)
        out["all_conv_frac_of_fp32_peak"] = round(ops / (ms * 1e-3) / 1e12 / FP32_MFMA_PEAK_TFLOPS, 4)
        out["per_kernel"] = kernel_table(stats, all_ms)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="resnet50", choices=sorted(WORKLOADS) + ["noisebank"])
    ap.add_argument("--chunk", type=int, default=0, help="noisy copies per device chunk (0 = default)")
    ap.add_argument("--n", type=int, default=0, help="override estimation samples per step")
    ap.add_argument("--mode", default="certify", choices=["certify", "predict"],
                    help="procedure a step runs: Alg. 1 (n0 + n samples) or Alg. 2 (n samples)")
    ap.add_argument("--batch", type=int, default=1,
                    help="(image, sigma) pairs per step; above 1 a step is one batched call over that many pairs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the short runs of the other workload configurations")
    ap.add_argument("--no-comparison-systems", action="store_true",
                    help="skip the short runs of the paper's floating-point comparison systems (FloatRS-quant, FloatRS-fp)")
    ap.add_argument("--system", default="int", choices=["int", "quant", "fp"],
                    help="int: the integer path (the headline metric); quant / fp: run only that comparison system on the workload")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (reference for HBM byte counters)")
    ap.add_argument("--profile-every", type=int, default=16,
                    help="time every kernel of each k-th chunk with HIP events (0 = off)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus above 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2108_09413_amd as isr
    import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.workload == "noisebank":
        return bench_noise_bank(args, isr, torch)
    cfg_id, chunk, oracle_samples = WORKLOADS[args.workload]
    chunk = args.chunk or chunk
    if args.system != "int":
        system = isr.FLOATRS_QUANT if args.system == "quant" else isr.FLOATRS_FP
        n = args.n or (synth.CONFIGS[cfg_id]["n"] if system == isr.FLOATRS_QUANT else 20000)
        # a step of the fp32 system is about 30 chunks: time every 4th so that full chunks outweigh the short selection chunk
        r = run_float_system(isr, synth, torch, cfg_id, chunk, system, n, args.steps, min(args.profile_every, 4))
        print(json.dumps({"metric": f"noisy {r['dtype']} inferences/sec ({r['system']})", "value": r["inferences_per_s"],
                          "unit": "inferences/s", "n_gpus": 1, "steps": args.steps, "warmup": 1, "ms_per_step": r["ms_per_step"],
                          "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": r["dtype"],
                          "data": "synthetic", "config": {"workload": f"config {cfg_id}: {r['arch']}, {r['system']}, n0={r['n0']}, n={r['n']}",
                                                          "chunk_samples": r["chunk_samples"]},
                          "roofline": r.get("roofline"), "all_conv_TFLOP/s": r.get("all_conv_TFLOP/s"),
                          "per_kernel": r.get("per_kernel"), "cpu_baseline": None, "last_result": r["last_result"]}))
        return

    if args.copy_calibration_mib:
        # random (non-zero) source far larger than the caches, evicted from them by a second buffer first
        src = torch.empty(args.copy_calibration_mib << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        flush = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst, flush

    dt, inferences, stats, last, ctx = run_config(isr, synth, torch, cfg_id, chunk, args.steps, args.profile_every,
                                                  n_override=args.n, mode=args.mode, batch=args.batch, warmup=args.warmup)
    cfg, n0, n, macs = ctx["cfg"], ctx["n0"], ctx["n"], ctx["macs"]
    value = inferences / dt
    all_ms = sum(s["total_ms"] for s in stats)
    conv, conv_ms, conv_ops, conv_launches = conv_aggregate(stats)
    table = kernel_table(stats, all_ms)
    roofline = roofline_all = roofline_hbm = None
    traffic, traffic_src = offline_traffic() if args.workload == "resnet50" else (None, "counter summary covers the resnet50 workload only")
    if conv_ms > 0:
        dom = max(conv, key=lambda s: s["total_ms"])          # the dominant kernel: largest share of the timed kernel time
        dom_tops = dom["alg_ops"] / (dom["total_ms"] * 1e-3) / 1e12
        dom_traffic = None
        if traffic and dom["name"] in traffic["per_kernel"] and chunk == 668:
            t = traffic["per_kernel"][dom["name"]]
            dom_traffic = t["fetch"] + t["write"]
        roofline = {
            "bound": "mfma", "kernel": dom["name"],
            "achieved": round(dom_tops, 2), "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
            "frac": round(dom_tops / INT8_MFMA_PEAK_TOPS, 4), "traffic": dom_traffic,
            "traffic_source": traffic_src if dom_traffic is not None else f"null: {traffic_src}",
            "launches_timed": dom["launches"], "avg_launch_us": round(dom["total_ms"] * 1e3 / dom["launches"], 2),
            "alg_ops_per_launch": round(dom["alg_ops"] / dom["launches"]),
            "alg_bytes_per_launch": round(dom["alg_bytes"] / dom["launches"]),
            "time_share_of_all_kernels": round(dom["total_ms"] / all_ms, 4),
            "note": "dominant = the convolution kernel instance with the largest total time over the timed launches; "
                    "traffic = HBM bytes of one full-chunk launch of that instance (offline rocprofv3 FETCH_SIZE + WRITE_SIZE "
                    "runs, scaled by the copy calibration), null when the committed summary is not of these sources",
        }
        achieved = conv_ops / (conv_ms * 1e-3) / 1e12
        roofline_all = {
            "bound": "mfma", "kernel": "all convolution kernel instances (see per_kernel)",
            "achieved": round(achieved, 2), "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
            "frac": round(achieved / INT8_MFMA_PEAK_TOPS, 4),
            # HBM bytes of an average conv launch: bytes per inference x copies per chunk / conv launches per chunk
            # (timed chunks = launches of a kernel that runs once per chunk)
            "traffic": round(traffic["conv_per_inference"] * chunk /
                             (conv_launches / max(max((s["launches"] for s in stats if s["name"].startswith("gap_kernel")), default=1), 1)))
            if traffic and chunk == 668 else None,
            "launches_timed": conv_launches, "avg_launch_us": round(conv_ms * 1e3 / max(conv_launches, 1), 2),
            "alg_ops_per_launch": round(conv_ops / max(conv_launches, 1)),
            "conv_share_of_kernel_time": round(conv_ms / all_ms, 4) if all_ms else None,
        }
        if roofline_all["traffic"]:
            hbm_gbs = roofline_all["traffic"] * conv_launches / (conv_ms * 1e-3) / 1e9
            roofline_hbm = {"bound": "hbm", "kernel": roofline_all["kernel"], "achieved": round(hbm_gbs, 1),
                            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(hbm_gbs / HBM_PEAK_GBS, 4),
                            "traffic": roofline_all["traffic"]}

    others = None
    if not args.no_other_configs and args.workload == "resnet50" and args.mode == "certify" and args.batch == 1:
        others = []
        for oc, ochunk, osteps in OTHER_CONFIGS:
            odt, oinf, ostats, olast, octx = run_config(isr, synth, torch, oc, ochunk, osteps, 4)
            _, oms, oops, _ = conv_aggregate(ostats)
            otops = oops / (oms * 1e-3) / 1e12 if oms > 0 else None
            others.append({"config": oc, "name": octx["cfg"]["name"], "arch": octx["cfg"]["arch"], "chunk_samples": ochunk,
                           "steps": osteps, "n0": octx["n0"], "n": octx["n"],
                           "inferences_per_s": round(oinf / odt, 1), "certified_images_per_s": round(osteps / odt, 3),
                           "ms_per_step": round(odt / osteps * 1e3, 3),
                           "conv_TOP/s": round(otops, 2) if otops else None,
                           "conv_frac_of_int8_peak": round(otops / INT8_MFMA_PEAK_TOPS, 4) if otops else None,
                           "last_result": {"cls": olast.cls, "radius": olast.radius, "n_top": olast.n_top}})

    systems = None
    if not args.no_comparison_systems and args.mode == "certify" and args.batch == 1:
        # the paper's efficiency comparison (int8 against float inference, section "Efficiency Evaluation"), same GPU, same workload
        systems = [run_float_system(isr, synth, torch, cfg_id, chunk, isr.FLOATRS_QUANT, n, 1, 0),
                   run_float_system(isr, synth, torch, cfg_id, chunk, isr.FLOATRS_FP, min(n, 20000), 1, 4)]
        for r in systems:
            r["int8_path_speedup_over_it"] = round(value / r["inferences_per_s"], 3)

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        om = oracle.Model(ctx["blob"])
        info = host_cpu_info()
        # every hardware thread the job may use: the box's OMP_NUM_THREADS share when set, else all of them
        threads = int(os.environ.get("OMP_NUM_THREADS") or 0) or (os.cpu_count() or 1)
        threads = max(1, min(threads, os.cpu_count() or 1, oracle_samples))
        x = synth.make_image(cfg_id, 1)
        t1 = time.perf_counter()
        om.mc(x, cfg["sigmas"][0], 0, 1, 1, 0, oracle_samples, threads=threads, want_logits=False)
        cdt = time.perf_counter() - t1
        cpu = {"value": round(oracle_samples / cdt, 3), "unit": "inferences/s", "cores": threads, "kind": "oracle",
               "sample": f"{oracle_samples} noisy inferences of image 1, sigma {cfg['sigmas'][0]}, phase 1 "
                         f"({cdt:.1f} s on {threads} OpenMP threads)",
               "host": info,
               "extrapolated_certified_images_per_s": round(oracle_samples / cdt / (n0 + n), 8)}

    out = {
        "metric": "noisy int8 inferences/sec", "value": round(value, 1), "unit": "inferences/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(dt / args.steps * 1e3, 2), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"config {cfg_id} ({cfg['name']}): {cfg['arch']} int8, input "
                               f"{'x'.join(map(str, cfg['shape']))}, {cfg['classes']} classes; one step = {args.mode} "
                               f"{args.batch if args.batch > 1 else 'one'} (image, sigma) pair{'s in one batched call' if args.batch > 1 else ''} "
                               f"with n0={n0}, n={n}, alpha={ctx['alpha']}; pairs cycle over "
                               f"{ctx['n_img']} images x sigma {list(cfg['sigmas'])}",
                   "chunk_samples": chunk, "macs_per_inference": macs},
        "certified_images_per_s": round(args.steps * args.batch / dt, 4),
        "whole_path_int8_tops": round(2.0 * macs * value / 1e12, 2),
        "whole_path_frac_of_int8_peak": round(2.0 * macs * value / 1e12 / INT8_MFMA_PEAK_TOPS, 4),
        "roofline": roofline,
        "roofline_all_conv": roofline_all,
        "roofline_hbm": roofline_hbm,
        "per_kernel": table,
        "other_configs": others,
        "comparison_systems": systems,
        "cpu_baseline": cpu,
        "paper_context": "int8 over fp32 on a desktop CPU: 3.5x (ResNet-20, 55.8 s vs 194.4 s per image at N = 100000) to "
                         "5.4x (ResNet-50): other hardware, not a target",
        "last_result": {"cls": last.cls, "radius": last.radius, "n_top": last.n_top,
                        "radius_int": last.radius_int, "radius_sq_int": last.radius_sq_int},
    }
    print(json.dumps(out))


def bench_noise_bank(args, isr, torch):
    """Stored training noise: one step = a bank of --n (default 50000) tensors of 3x32x32
    discrete-Gaussian draws (int16) at sigma 32, written to HBM."""
    count, d, sigma = args.n or 50000, 3 * 32 * 32, 32
    out = torch.empty((count, d), dtype=torch.int16, device="cuda")
    for k in range(args.warmup):
        isr.isr_noise_bank(sigma, 0, k, 0, count, d, out=out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        isr.isr_noise_bank(sigma, 0, 100 + k, 0, count, d, out=out)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    values = args.steps * count * d
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        sample = 2000
        t1 = time.perf_counter()
        oracle.noise_bank(sigma, 0, 100, 0, sample, d)
        cdt = time.perf_counter() - t1
        cpu = {"value": round(sample * d / cdt, 1), "unit": "draws/s", "cores": 1, "kind": "oracle",
               "sample": f"{sample} tensors of {d} draws ({cdt:.1f} s, one thread)", "host": host_cpu_info()}
    # executed VALU instructions per 4 draws of one lane, from the committed rocprofv3 counter run
    # (SQ_INSTS_VALU / (draws / 4 / 64), profiles/noise_bank_kernel.md); peak = 256 CUs x 64 lanes x 2.4 GHz
    valu_per_group, alu_peak = 137.0, 256 * 64 * 2.4e9 / 1e12
    tops = values / 4 * valu_per_group / dt / 1e12
    print(json.dumps({
        "metric": "stored discrete-Gaussian noise draws/sec", "value": round(values / dt, 1), "unit": "draws/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(dt / args.steps * 1e3, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int16", "data": "synthetic",
        "config": {"workload": f"noise bank: {count} tensors x {d} draws (3x32x32), sigma {sigma}, int16, whole call "
                               f"(table build + upload + kernel + synchronisation)"},
        "roofline": {"bound": "alu", "kernel": "noise_bank_kernel", "achieved": round(tops, 2), "peak": round(alu_peak, 2),
                     "unit": "T lane-instructions/s", "frac": round(tops / alu_peak, 4), "traffic": None,
                     "note": "137 executed VALU instructions per lane per 4 draws (rocprofv3 SQ_INSTS_VALU) over the "
                             "whole-call time; the 2 bytes written per draw are "
                             f"{values * 2 / dt / 1e9:.0f} GB/s"},
        "cpu_baseline": cpu}))


if __name__ == "__main__":
    main()
