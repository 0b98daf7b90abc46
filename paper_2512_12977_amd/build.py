"""Builds libvlcache.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from typing import Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libvlcache.so")
SOURCES = ["api.cpp", "planner.cpp", "layer.cpp", "stream_kernels.hip", "gemm.hip", "attention.hip", "moe.hip", "noalloc.hip", "probe.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc() -> str:
    for c in ("/opt/rocm/bin/hipcc", "hipcc"):
        if os.path.sep not in c or os.path.exists(c):
            return c
    raise RuntimeError("hipcc not found")


def build(verbose: bool = True, tag: str = "", defines: Sequence[str] = ()) -> str:
    """Compile every source and link the shared library; returns its path.  With a tag the result is
    libvlcache_<tag>.so (beside the product library, which is left alone) built with the given -D macros:
    the measurement variants of the kernels (see the VLC_ABLATE_* macros in csrc/attention.hip)."""
    hipcc = _hipcc()
    objdir = os.path.join(HERE, "_build", tag) if tag else os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    lib = os.path.join(HERE, "libvlcache_%s.so" % tag) if tag else LIB
    if defines and not tag:
        raise ValueError("macros change what the kernels compute: give the variant a tag")
    extra = ["-D" + d for d in defines]

    def compile_one(src: str) -> str:
        obj = os.path.join(objdir, src + ".o")
        cmd = [hipcc, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, err))
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", lib)
    return lib


def build_host_check(verbose: bool = False) -> str:
    """The library's sources and tests/sanitize/host_check.cpp as one executable whose HOST code is instrumented with
    AddressSanitizer and UndefinedBehaviorSanitizer (device code is compiled as always and never runs: the program
    only calls the planner and the argument checks).  Returns the path of the executable."""
    hipcc = _hipcc()
    objdir = os.path.join(HERE, "_build", "asan")
    os.makedirs(objdir, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    flags = [f for f in FLAGS if f != "-O3"] + ["-O1", "-g"] + san
    srcs = [os.path.join(CSRC, s) for s in SOURCES] + [os.path.join(ROOT, "tests", "sanitize", "host_check.cpp")]

    def compile_one(src: str) -> str:
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        r = subprocess.run([hipcc, *flags, "-c", src, "-o", obj], capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc (sanitizers) failed on %s:\n%s" % (src, r.stderr))
        return obj

    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(compile_one, srcs))
    exe = os.path.join(objdir, "host_check")
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
                        "-o", exe, *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link (sanitizers) failed:\n" + r.stderr)
    if verbose:
        print("built", exe)
    return exe


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("--tag", default="", help="build libvlcache_<tag>.so instead of the product library")
    ap.add_argument("--define", action="append", default=[], help="-D macro for a tagged measurement variant")
    a = ap.parse_args()
    build(tag=a.tag, defines=a.define)
