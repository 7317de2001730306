"""Builds libecf8.so (host encoder + gfx950 HIP kernels) in-tree with hipcc.

Every source is compiled to an object of its own, the sources in parallel, then linked.
build() compiles everything every time; build(incremental=True) keeps the objects whose
source and headers have not changed (a development shortcut, never used by the entry points).
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libecf8.so")
CSRC = os.path.join(PKG, "csrc")
OBJ_DIR = os.path.join(PKG, "_build")
SOURCES = ["ecf8_host.cpp", "ecf8_jit.cpp", "ecfw_host.cpp", "ecf8_decode.hip", "ecf8_gemm.hip", "ecf8_gemm_exact.hip",
           "ecf8_encode.hip", "ecfw_decode.hip", "ecfw_encode.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-pthread",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument", "-I", os.path.join(ROOT, "include")]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd))
    r = subprocess.run(cmd, capture_output=True, text=True)
    out = (r.stdout + r.stderr).strip()
    # the host pass does not know the gfx-only target feature; that one warning is expected
    out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
    if out and (verbose or r.returncode):
        print(out, file=sys.stderr)
    return r.returncode


def _newest_header():
    dirs = [CSRC, os.path.join(ROOT, "include")]
    return max(os.path.getmtime(os.path.join(d, f)) for d in dirs for f in os.listdir(d) if f.endswith(".h"))


def build(verbose=False, extra=(), incremental=False):
    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = [s for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]
    hdr_time = _newest_header() if incremental else 0.0
    jobs = []
    for s in srcs:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJ_DIR, s + ".o")
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), hdr_time):
            continue
        jobs.append([HIPCC] + FLAGS + list(extra) + ["-c", src, "-o", obj])
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        codes = list(pool.map(lambda c: _run(c, verbose), jobs))
    if any(codes):
        raise RuntimeError("hipcc failed compiling libecf8.so")
    objs = [os.path.join(OBJ_DIR, s + ".o") for s in srcs]
    if _run([HIPCC] + FLAGS + ["-shared"] + objs + ["-o", LIB], verbose):
        raise RuntimeError("hipcc failed linking libecf8.so")
    return LIB


if __name__ == "__main__":
    build(verbose=True, incremental="--incremental" in sys.argv)
