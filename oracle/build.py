"""Compile the CPU oracle into oracle/liboracle.so (g++, no fast-math, no contraction)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "liboracle.so")


def build(verbose: bool = False, src: str = None, out: str = None) -> str:
    """Compiles oracle.cpp (or another source file with the same interface) into a library."""
    out = out or LIB
    cmd = ["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
           "-I", HERE, "-shared", "-fPIC", src or os.path.join(HERE, "oracle.cpp"), "-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return out


def ensure_built() -> str:
    src = os.path.join(HERE, "oracle.cpp")
    hdr = os.path.join(HERE, "oracle.h")
    if (not os.path.exists(LIB) or os.path.getmtime(LIB) < max(os.path.getmtime(src),
                                                              os.path.getmtime(hdr))):
        build()
    return LIB


if __name__ == "__main__":
    build(verbose=True)
