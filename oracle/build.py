"""Compiles the CPU oracle (plain C++17, no HIP) into oracle/liboracle.so.

TEST INFRASTRUCTURE ONLY: nothing in the product path builds, loads or calls it.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = ["philox.cpp", "shard.cpp", "fill.cpp", "capi.cpp"]
LIB = os.path.join(HERE, "liboracle.so")


def build(verbose: bool = False) -> str:
    # -ffp-contract=off: every fp32 operation of the definition rounds on its own.
    cmd = ["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-pthread",
           "-Wall", "-Wextra", "-o", LIB] + [os.path.join(HERE, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(HERE, f)) > t
               for f in os.listdir(HERE) if f.endswith((".cpp", ".hpp")))


if __name__ == "__main__":
    build(verbose=True)
