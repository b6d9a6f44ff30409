"""Host code and oracle under AddressSanitizer + UndefinedBehaviorSanitizer: tests/sanitize_host.cpp
(library parser, planner, table builder, statistics; oracle parser and forward pass) is built once
with the sanitizers and run over the workload blobs and over thousands of damaged copies of them.
Any out-of-bounds access, overflow or leak in the paths a malformed model can reach fails the run."""
import os
import shutil
import subprocess

import numpy as np
import pytest

import synth
from synth.models import NetBuilder

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2108_09413_amd", "csrc")
CLANGXX = "/opt/rocm/lib/llvm/bin/clang++"
CLANG = "/opt/rocm/lib/llvm/bin/clang"
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


def _odd_net():
    """Every op type, channel counts off the 16-grid, strides, a projection shortcut, two adds."""
    b = NetBuilder(rng=np.random.default_rng(12), in_shape=(3, 20, 12), num_classes=7)
    t0 = b.tensor(3, 20, 12, 0, 74.0)
    t1 = b.conv(t0, 5, 5, 1, 2, True)
    t2 = b.conv(t1, 40, 3, 2, 1, False, zp_out=9)
    t3 = b.conv(t2, 40, 1, 1, 0, True, zp_out=-100)
    t4 = b.add(t2, t3, False, ma=-600000, mb=900000, sh=20, zp_out=-5)
    t5 = b.maxpool(t4, 3, 2, 1)
    t6 = b.conv(t5, 64, 1, 1, 0, True)
    t7 = b.conv(t6, 64, 3, 1, 1, True)
    t8 = b.conv(t7, 64, 1, 1, 0, False)
    t9 = b.add(t6, t8, True)
    b.fc(b.gap(t9), 7)
    return b.blob()


@pytest.fixture(scope="module")
def sanitized_binary(tmp_path_factory):
    if not (os.path.exists(CLANGXX) and os.path.exists(CLANG)):
        pytest.skip("no clang to build the sanitizer harness")
    out = tmp_path_factory.mktemp("san")
    exe = str(out / "sanitize_host")
    oracle_obj = str(out / "isr_oracle.o")
    subprocess.check_call([CLANG, *SAN, "-std=c11", "-c", os.path.join(ROOT, "oracle", "isr_oracle.c"), "-o", oracle_obj])
    srcs = [os.path.join(ROOT, "tests", "sanitize_host.cpp")] + [os.path.join(CSRC, f) for f in
                                                                 ("model_parse.cpp", "plan.cpp", "noise_table.cpp", "host_stats.cpp")]
    subprocess.check_call([CLANGXX, *SAN, "-std=c++17", "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include", "-I", os.path.join(ROOT, "include"),
                           "-I", CSRC, *srcs, oracle_obj, "-o", exe, "-lm"])
    return exe, out


def test_host_paths_are_clean_under_sanitizers(sanitized_binary):
    exe, out = sanitized_binary
    paths = []
    for name, blob in (("tiny", synth.build_model(0)), ("resnet20", synth.build_model(1)), ("odd", _odd_net()),
                       ("resnet50_64", synth.build_model(3, size=64))):
        path = str(out / f"{name}.isrm")
        open(path, "wb").write(blob)
        paths.append(path)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:allocator_may_return_null=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    # the small blobs get the full damage sweep; the large one (23 MB of weights at 64x64) is parsed and planned once
    proc = subprocess.run([exe, *paths[:3]], capture_output=True, text=True, env=env, timeout=600)
    assert proc.returncode == 0, proc.stdout[-2000:] + proc.stderr[-4000:]
    assert "status 0" in proc.stdout and "ERROR" not in proc.stderr, proc.stderr[-4000:]
    accepted, rejected = [int(w.strip(",")) for w in proc.stdout.split() if w.strip(",").isdigit()][:2]
    assert rejected > 1000 and accepted >= 3, proc.stdout
