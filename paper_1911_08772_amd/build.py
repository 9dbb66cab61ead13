"""Compile the native parts in-tree.

libsparsify.so  -- the HIP kernels and their C ABI (hipcc, gfx950 only)
libsynth.so     -- the seeded input generator (plain C, host)
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB_SPARSIFY = os.path.join(HERE, "libsparsify.so")
LIB_SYNTH = os.path.join(HERE, "libsynth.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
             "-ffp-contract=off", "-fno-fast-math", "-fno-gpu-flush-denormals-to-zero",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wall", "-Wno-unused-command-line-argument"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)


def build_sparsify(verbose: bool = False) -> str:
    srcs = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))
    _run([HIPCC, *HIP_FLAGS, "-I", INCLUDE, "-I", CSRC, *srcs, "-o", LIB_SPARSIFY], verbose)
    return LIB_SPARSIFY


def build_synth(verbose: bool = False) -> str:
    _run(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", os.path.join(CSRC, "synth.c"),
          "-o", LIB_SYNTH, "-lm"], verbose)
    return LIB_SYNTH


def build_all(verbose: bool = False) -> None:
    build_synth(verbose)
    build_sparsify(verbose)


def _stale(lib, srcs):
    return (not os.path.exists(lib)) or any(os.path.getmtime(s) > os.path.getmtime(lib)
                                            for s in srcs)


def _sparsify_sources():
    return ([os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".h"))] +
            [os.path.join(INCLUDE, f) for f in os.listdir(INCLUDE) if f.endswith(".h")])


def ensure_synth() -> str:
    """Path of the built generator; (re)builds it when it is missing or older than its source."""
    if _stale(LIB_SYNTH, [os.path.join(CSRC, "synth.c")]):
        build_synth()
    return LIB_SYNTH


def ensure_sparsify() -> str:
    """Path of the built HIP library; (re)builds it when it is missing or older than any of its
    sources, so that a test run never silently exercises the binary of an earlier edit."""
    other = os.environ.get("SPARSIFY_LIBRARY")  # another build of the same sources (a debug build, say)
    if other:
        return other
    if _stale(LIB_SPARSIFY, _sparsify_sources()):
        build_sparsify()
    return LIB_SPARSIFY


if __name__ == "__main__":
    build_all(verbose=True)
