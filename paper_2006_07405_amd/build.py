"""Builds liba2sgd.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc.  No GPU is needed to compile."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "liba2sgd.so")
SOURCES = [os.path.join(HERE, "csrc", "a2sgd_kernels.hip"), os.path.join(HERE, "csrc", "a2sgd_segments.hip"),
           os.path.join(HERE, "csrc", "a2sgd_api.cpp")]

# Denormals are kept (a flushed tiny negative would change sign group); packed-fp32 instructions are disabled.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-flush-denormals-to-zero",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wextra",
         "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(HERE, "csrc")]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + ["-x", "hip"] + SOURCES + ["-o", LIB]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "is not a recognized feature" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out, file=sys.stderr)
    return LIB


STREAMS_LIB = os.path.join(HERE, "libhbm_streams.so")
STREAMS_SRC = os.path.join(HERE, "csrc", "hbm_streams.hip")


def build_streams() -> str:
    """The plain streaming kernels that bench.py times for its measured bandwidth ceilings (csrc/hbm_streams.hip)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Xclang", "-target-feature",
           "-Xclang", "-packed-fp32-ops", "-Wall", "-Wextra", "-x", "hip", STREAMS_SRC, "-o", STREAMS_LIB]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed on the streaming kernels:\n" + proc.stdout)
    return STREAMS_LIB


CLIENT_SRC = os.path.join(ROOT, "tests", "c_client", "client.cpp")
CLIENT = os.path.join(ROOT, "tests", "c_client", "client")


def build_client() -> str:
    """The test program that calls the C ABI without Python or torch (tests/c_client): host code only, linked
    against the library next to this file."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-O2", "-std=c++17", "-Wall", "-Wextra", "-I" + os.path.join(ROOT, "include"), CLIENT_SRC, "-o", CLIENT,
           "-L" + HERE, "-la2sgd", "-Wl,-rpath,$ORIGIN/../../paper_2006_07405_amd"]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed on the client:\n" + proc.stdout)
    return CLIENT


if __name__ == "__main__":
    print(build(verbose=True))
