"""The library's host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).

Host passes of api.cpp, scheduler.cpp, kd_host.cpp and section.hip (the executor: validation, workspace plan, kernel
sequencing) are compiled with the sanitizers, linked with stand-in kernels that touch every buffer over its full
documented extent (tests/host_sanitizer/fake_backend.cpp), and driven through the C ABI on exact-size heap buffers
(tests/host_sanitizer/driver.cpp).  A sanitizer report or a failed check ends the driver with a non-zero status."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2605_10501_amd", "csrc")
HERE = os.path.join(ROOT, "tests", "host_sanitizer")
OUT = os.path.join(ROOT, "_build", "host_sanitizer")
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"]
CLANG = "/opt/rocm/lib/llvm/bin/clang++"


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    assert r.returncode == 0, " ".join(cmd) + "\n" + r.stdout + err
    return r.stdout


@pytest.mark.skipif(shutil.which("hipcc") is None or not os.path.exists(CLANG), reason="needs the ROCm compilers")
def test_host_code_under_address_and_ub_sanitizers():
    os.makedirs(OUT, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    objs = []
    for src in ["api.cpp", "scheduler.cpp", "kd_host.cpp", "section.hip"]:
        obj = os.path.join(OUT, src + ".o")
        # host pass only (no device code is generated or embedded); each -fsanitize= directly after -Xarch_host
        cmd = ["hipcc", "--offload-arch=gfx950", "--cuda-host-only", "-O1", "-g", "-std=c++17", "-x", "hip", "-Wno-unused-value"]
        for f in SAN:
            cmd += ["-Xarch_host", f]
        _run(cmd + inc + ["-c", os.path.join(CSRC, src), "-o", obj])
        objs.append(obj)
    exe = os.path.join(OUT, "driver")
    _run([CLANG, "-std=c++17", "-O1", "-g", *SAN, *inc, os.path.join(HERE, "driver.cpp"), os.path.join(HERE, "fake_backend.cpp"),
          *objs, "-o", exe])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)
    r = subprocess.run([exe], capture_output=True, text=True, env=env)
    assert r.returncode == 0 and "host sanitizer driver: OK" in r.stdout, r.stdout + r.stderr
