"""Compile the hch shared library for gfx950 with hipcc (in-tree, next to the sources)."""
from __future__ import annotations

import hashlib
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhch.so")
SOURCES = ["hch_api.hip", "psh_build.cpp"]
HEADERS = ["kernels.hip.hpp", "direct.hip.hpp", "gemm_bf16.hip.hpp", "psh_device.hip.hpp", "psh_build.hpp", "profile.hpp", os.path.join("..", "..", "include", "hch.h")]


def hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def source_digest():
    """First 16 hex digits of a sha256 over the library's sources (csrc/ and the public header):
    names the code a measurement was taken on (the summaries under profiles/ carry it, bench.py
    compares it with the sources it runs)."""
    h = hashlib.sha256()
    paths = [os.path.join(CSRC, n) for n in sorted(os.listdir(CSRC))]
    paths.append(os.path.join(HERE, "..", "include", "hch.h"))
    for p in paths:
        with open(p, "rb") as f:
            h.update(os.path.basename(p).encode())
            h.update(f.read())
    return h.hexdigest()[:16]


def build_library(force=True, verbose=False):
    """Build libhch.so.  With force=False an up-to-date library is kept."""
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS]
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps):
        return LIB
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           # keep the compiler from forming packed-fp32 instructions
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           # accumulators of the matrix instructions in ordinary VGPRs, updated in place: with the
           # default (AGPR) form the compiler copies every accumulator through VGPRs once per loop
           # iteration, which costs the bf16 kernels more issue slots than their matrix instructions
           "-mllvm", "-amdgpu-mfma-vgpr-form",
           "-Wall", "-Wno-unused-function", "-pthread",
           "-o", LIB] + os.environ.get("HCH_EXTRA_HIPCC_FLAGS", "").split() + [os.path.join(CSRC, f) for f in SOURCES]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
