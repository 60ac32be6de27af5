"""Builds libr2ccl.so for gfx950 with hipcc (cross-compiles; no GPU needed)."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = [os.path.join(HERE, "csrc", f) for f in ("partition.hip", "ring.hip", "rails.hip", "split.hip", "recursive.hip", "streams.hip", "rerank.cpp")]
HEADERS = sorted(glob.glob(os.path.join(HERE, "csrc", "*.h"))) + sorted(glob.glob(os.path.join(ROOT, "include", "*.h")))
LIB = os.path.join(HERE, "libr2ccl.so")
PROBE_SRC = os.path.join(HERE, "csrc", "stream_probe.hip")
PROBE_LIB = os.path.join(HERE, "libr2probe.so")
EXAMPLE_SRC = os.path.join(HERE, "examples", "ring_allreduce.c")
EXAMPLE = os.path.join(HERE, "examples", "ring_allreduce")

# Packed-fp32 instructions are switched off for all device code.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wall", "-Wextra"]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(HERE, "csrc"),
           "-o", LIB, *SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    noise = "is not a recognized feature for this target"  # host pass does not know the device flag
    out = "\n".join(l for l in res.stdout.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    build_example(verbose)
    build_probe(verbose)
    return LIB


def build_probe(verbose: bool = False) -> str:
    """The bare-kernel memory probe `bench.py --stream-mix` times beside the product: a library of its own,
    so that nothing of it is in libr2ccl.so."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-o", PROBE_LIB, PROBE_SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed on the stream probe:\n" + res.stdout)
    return PROBE_LIB


def build_example(verbose: bool = False) -> str:
    """The plain-C caller of the ABI: compiled with gcc against the header and the library just built."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-O2", "-std=c11", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I" + os.path.join(rocm, "include"),
           "-I" + os.path.join(ROOT, "include"), EXAMPLE_SRC, "-L" + HERE, "-lr2ccl",
           "-L" + os.path.join(rocm, "lib"), "-lamdhip64", "-lm", "-Wl,-rpath,$ORIGIN/..",
           "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", EXAMPLE]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("gcc failed on the C example:\n" + res.stdout)
    return EXAMPLE


if __name__ == "__main__":
    build(verbose=True)
    sys.exit(0)
