"""Builds libdpipe.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdpipe.so")
SOURCES = ["gemm.hip", "attention.hip", "elementwise.hip", "stage.hip", "ktime.hip", "partition.hip", "bubbles.hip", "noalloc.hip", "conv.hip", "image_encoder.hip", "search.hip", "errors.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose: bool = True, jobs: int = 4) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs, procs = [], []
    bdir = os.path.join(HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    for src in SOURCES:
        obj = os.path.join(bdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        if len(procs) >= jobs:
            _wait(procs, verbose)
    _wait(procs, verbose)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


def _wait(procs, verbose):
    while procs:
        src, p = procs.pop(0)
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "is not a recognized feature for this target" not in l)
        if p.returncode != 0:
            sys.stderr.write(out + "\n")
            raise RuntimeError(f"hipcc failed on {src}")
        if verbose and out.strip():
            print(out)


# The sources that make no GPU call (partitioner, bubble filler, schedule search, error message): they also
# compile as plain C++, which is how the sanitizer build of the tests takes them.
HOST_ONLY_SOURCES = ["partition.hip", "bubbles.hip", "search.hip", "errors.hip"]


def build_host_sanitized(driver_cpp: str, out_path: str) -> str:
    """Builds `driver_cpp` together with the host-only sources as one executable under AddressSanitizer and
    UndefinedBehaviorSanitizer (g++; no GPU code is involved)."""
    cxx = os.environ.get("CXX", "g++")
    cmd = [cxx, "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-Wall", driver_cpp]
    for src in HOST_ONLY_SOURCES:
        cmd += ["-x", "c++", os.path.join(CSRC, src)]
    cmd += ["-o", out_path]
    subprocess.run(cmd, check=True)
    return out_path


if __name__ == "__main__":
    build()
