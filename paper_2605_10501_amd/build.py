"""Build the HIP section-compute library for gfx950 (in tree: libmaestro_section.so)."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libmaestro_section.so")
BUILD = os.path.join(ROOT, "_build")
SOURCES = ["api.cpp", "profile.cpp", "scheduler.cpp", "kd_host.cpp", "elementwise.hip", "gemm.hip", "attention.hip", "attention_mfma.hip", "kd.hip",
           "section.hip", "merger.hip", "probes.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Wno-unused-value"]


def _compile(src):
    obj = os.path.join(BUILD, src + ".o")
    cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose=True):
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    import ctypes
    ctypes.CDLL(OUT)   # an unresolved symbol must fail the build, not the first caller
    if verbose:
        print("built", OUT)
    return OUT


if __name__ == "__main__":
    build()
