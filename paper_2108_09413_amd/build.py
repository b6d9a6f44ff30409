"""Builds libisr.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libisr.so")
SOURCES = ["api.cpp", "plan.cpp", "model_parse.cpp", "noise_table.cpp", "host_stats.cpp", "kernels.hip", "conv_igemm.hip", "stem_pool.hip", "basic_block.hip", "bottleneck.hip", "bottleneck128.hip", "stem16.hip", "trans_block.hip", "noise_bank_static.hip", "conv_deep.hip", "conv_patch.hip", "expand_reduce.hip", "float_api.cpp", "float_path.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON = ["-O3", "-std=c++17", "-fPIC", "-I", os.path.join(ROOT, "include"), "-I", CSRC]
# kernels: gfx950 only; packed-FP32 instruction selection is switched off; MFMA results go to
# ordinary VGPRs (no accumulator-register copies in front of the epilogue arithmetic)
HIP_FLAGS = ["--offload-arch=gfx950", "-x", "hip", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wno-unknown-attributes"]
VGPR_FORM = ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]
# kernels whose accumulators exceed the ordinary VGPRs keep the default (accumulation registers)
ACC_REGISTER_SOURCES = {"conv_deep.hip"}
# host-only sources: plain C++ against the HIP runtime headers
HOST_FLAGS = ["-x", "c++", "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include"]


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    flags = HOST_FLAGS
    if src.endswith(".hip"):
        flags = HIP_FLAGS + ([] if src in ACC_REGISTER_SOURCES else VGPR_FORM)
    proc = subprocess.run([HIPCC, *COMMON, *flags, "-c", os.path.join(CSRC, src), "-o", obj],
                          stderr=subprocess.PIPE, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in proc.stderr.splitlines() if noise not in l)
    if err.strip():
        print(err)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}")
    return obj


def build_library(verbose: bool = False) -> str:
    with ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.check_call([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs])
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build_library(verbose=True)
