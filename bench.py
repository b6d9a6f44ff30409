#!/usr/bin/env python3
"""Benchmark of the integer randomized smoothing hot path on one MI355X.

A step is one certification (Alg. 1 of the paper: n0 selection + n estimation
noisy inferences, votes, decision) of one (image, sigma) pair of the headline
workload: the ResNet-50 int8 network on a 3x224x224 image with n = 100000.
Images, weights and tables are resident in HBM before the timed region.

Prints one JSON line: whole-job noisy inferences/s, the roofline record of the
dominant kernel (int8 MFMA implicit-GEMM convolution, timed with HIP events on
the library's stream inside the timed region) and the CPU oracle timed on the
host cores on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
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
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (reference for HBM byte counters)")
    ap.add_argument("--profile-every", type=int, default=16,
                    help="time every kernel of each k-th chunk with HIP events (0 = off)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus above 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2108_09413_amd as isr
    import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.workload == "noisebank":
        return bench_noise_bank(args, isr, torch)
    cfg_id, chunk, oracle_samples = WORKLOADS[args.workload]
    cfg = synth.CONFIGS[cfg_id]
    chunk = args.chunk or chunk
    n0, n = cfg["n0"], (args.n or cfg["n"])
    alpha = 0.001
    blob = synth.build_model(cfg_id)
    macs = synth.model_macs(cfg_id)
    model = isr.isr_load_model(blob)
    isr.isr_set_workspace(model, chunk)
    n_img = min(cfg["images"], 10)
    images = [torch.from_numpy(synth.make_image(cfg_id, i + 1)).cuda() for i in range(n_img)]
    pairs = [(i, s) for i in range(n_img) for s in cfg["sigmas"]]
    # noise tables for every sigma are built and uploaded before the timed region
    for s in cfg["sigmas"]:
        isr.isr_certify(model, images[0], s, 1, 1, alpha, want_counts=False)

    if args.mode == "predict":
        n0 = 0
    image_array = torch.stack(images)

    def step(k):
        if args.batch > 1:
            items = [(pairs[j % len(pairs)][0], pairs[j % len(pairs)][1], pairs[j % len(pairs)][0] + 1)
                     for j in range(k * args.batch, (k + 1) * args.batch)]
            if args.mode == "predict":
                return isr.isr_predict_batch(model, image_array, items, n, alpha, seed=0)[0][-1]
            return isr.isr_certify_batch(model, image_array, items, n0, n, alpha, seed=0)[0][-1]
        i, s = pairs[k % len(pairs)]
        if args.mode == "predict":
            return isr.isr_predict(model, images[i], s, n, alpha, seed=0, image_id=i + 1)[0]
        return isr.isr_certify(model, images[i], s, n0, n, alpha, seed=0, image_id=i + 1, want_counts=False)[0]

    if args.copy_calibration_mib:
        # random (non-zero) source far larger than the caches, evicted from them by a second buffer first
        src = torch.empty(args.copy_calibration_mib << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        flush = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst, flush
    for k in range(args.warmup):
        step(k)
    isr.isr_profile(model, args.profile_every)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    results = [step(args.warmup + k) for k in range(args.steps)]
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    stats = isr.isr_profile_read(model)
    isr.isr_profile(model, 0)

    inferences = args.steps * args.batch * (n0 + n)
    value = inferences / dt
    conv = [s for s in stats if s["name"].startswith("conv")]
    conv_ms = sum(s["total_ms"] for s in conv)
    conv_ops = sum(s["alg_ops"] for s in conv)
    conv_launches = sum(s["launches"] for s in conv)
    all_ms = sum(s["total_ms"] for s in stats)
    roofline = roofline_hbm = None
    if conv_ms > 0:
        achieved = conv_ops / (conv_ms * 1e-3) / 1e12
        roofline = {
            "bound": "mfma", "kernel": "all convolution kernels: conv_dma_kernel (all tiles), bottleneck_kernel, stem_pool_kernel",
            "achieved": round(achieved, 2), "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
            "frac": round(achieved / INT8_MFMA_PEAK_TOPS, 4), "traffic": None,
            "launches_timed": conv_launches,
            "avg_launch_us": round(conv_ms * 1e3 / max(conv_launches, 1), 2),
            "alg_ops_per_launch": round(conv_ops / max(conv_launches, 1)),
            "conv_share_of_kernel_time": round(conv_ms / all_ms, 4) if all_ms else None,
            "per_kernel": [
                {"name": s["name"], "launches": s["launches"],
                 "avg_us": round(s["total_ms"] * 1e3 / s["launches"], 2),
                 "TOP/s": round(s["alg_ops"] / (s["total_ms"] * 1e-3) / 1e12, 2) if s["alg_ops"] else None,
                 "GB/s": round(s["alg_bytes"] / (s["total_ms"] * 1e-3) / 1e9, 1),
                 "time_share": round(s["total_ms"] / all_ms, 4)} for s in stats],
        }

    # HBM bytes per conv launch from the committed rocprofv3 counter summary (measured offline,
    # per noisy inference; scaled to the launches of one chunk)
    if roofline is not None and args.workload == "resnet50":
        try:
            import re
            txt = open(os.path.join(ROOT, "profiles", "resnet50_certify_hbm_traffic.md")).read()
            mt = re.search(r"conv_hbm_bytes_per_inference: fetch=(\d+) write=(\d+)", txt)
            launches_per_inference = conv_launches / max(sum(s["launches"] for s in stats if s["name"] == "noise"), 1) / chunk
            roofline["traffic"] = round((int(mt.group(1)) + int(mt.group(2))) / launches_per_inference)
            roofline["traffic_note"] = ("HBM bytes per conv launch: rocprofv3 FETCH_SIZE+WRITE_SIZE per inference "
                                        "(scaled by the copy calibration) x inferences per launch")
            roofline["alg_bytes_per_launch"] = round(sum(s["alg_bytes"] for s in conv) / max(conv_launches, 1))
            hbm_gbs = roofline["traffic"] * conv_launches / (conv_ms * 1e-3) / 1e9
            roofline_hbm = {"bound": "hbm", "kernel": roofline["kernel"], "achieved": round(hbm_gbs, 1),
                            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(hbm_gbs / HBM_PEAK_GBS, 4),
                            "traffic": roofline["traffic"]}
        except Exception:
            pass

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        om = oracle.Model(blob)
        threads = min(os.cpu_count() or 1, 16)
        x = synth.make_image(cfg_id, 1)
        t1 = time.perf_counter()
        om.mc(x, cfg["sigmas"][0], 0, 1, 1, 0, oracle_samples, threads=threads, want_logits=False)
        cdt = time.perf_counter() - t1
        cpu = {"value": round(oracle_samples / cdt, 3), "unit": "inferences/s", "cores": threads, "kind": "oracle",
               "sample": f"{oracle_samples} noisy inferences of image 1, sigma {cfg['sigmas'][0]}, phase 1 "
                         f"({cdt:.1f} s on {threads} OpenMP threads)"}

    out = {
        "metric": "noisy int8 inferences/sec", "value": round(value, 1), "unit": "inferences/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(dt / args.steps * 1e3, 2), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"config {cfg_id} ({cfg['name']}): {cfg['arch']} int8, input "
                               f"{'x'.join(map(str, cfg['shape']))}, {cfg['classes']} classes; one step = {args.mode} "
                               f"{args.batch if args.batch > 1 else 'one'} (image, sigma) pair{'s in one batched call' if args.batch > 1 else ''} "
                               f"with n0={n0}, n={n}, alpha={alpha}; pairs cycle over "
                               f"{n_img} images x sigma {list(cfg['sigmas'])}",
                   "chunk_samples": chunk, "macs_per_inference": macs},
        "certified_images_per_s": round(args.steps * args.batch / dt, 4),
        "whole_path_int8_tops": round(2.0 * macs * value / 1e12, 2),
        "whole_path_frac_of_int8_peak": round(2.0 * macs * value / 1e12 / INT8_MFMA_PEAK_TOPS, 4),
        "roofline": roofline,
        "roofline_hbm": roofline_hbm,
        "cpu_baseline": cpu,
        "last_result": {"cls": results[-1].cls, "radius": results[-1].radius, "n_top": results[-1].n_top},
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
               "sample": f"{sample} tensors of {d} draws ({cdt:.1f} s, one thread)"}
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
