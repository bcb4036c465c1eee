"""Builds liblfmmi.so (HIP kernels + C ABI) for gfx950, in-tree."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblfmmi.so")
SOURCES = ["kernels.hip", "api.cpp", "pack.cpp"]
HEADERS = ["kernels.h", "pack.h", "microbench.hip", os.path.join("..", "..", "include", "lfmmi.h")]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # scalar fp32 only: no packed-fp32 instructions from the auto-vectoriser
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # private arrays stay out of LDS: kernels here address LDS by absolute offsets
    "-mllvm", "-disable-promote-alloca-to-lds",
    "-Wall", "-Wno-unused-command-line-argument",
]


def is_stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES + HEADERS] + [os.path.abspath(__file__)]
    return any(os.path.getmtime(d) > t for d in deps)


MICROBENCH = os.path.join(HERE, "lfmmi_microbench")


def microbench_command(hipcc):
    flags = [f for f in FLAGS if f not in ("-fPIC", "-shared")]
    return [hipcc] + flags + ["-o", MICROBENCH, os.path.join(CSRC, "microbench.hip")]


def build(force=True, extra_flags=()):
    """Compile with hipcc (cross-compiles without a GPU): the library, and the
    microbenchmark program behind the roofline peaks."""
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + list(extra_flags) + ["-o", LIB] + \
          [os.path.join(CSRC, s) for s in SOURCES]
    jobs = [subprocess.Popen(cmd), subprocess.Popen(microbench_command(hipcc))]
    codes = [j.wait() for j in jobs]
    if any(codes):
        raise subprocess.CalledProcessError(max(codes), cmd)
    return LIB


if __name__ == "__main__":
    print(build())
