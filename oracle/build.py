"""Compiles the CPU oracle (plain C++17, no HIP) into oracle/liboracle.so.

TEST INFRASTRUCTURE ONLY: nothing in the product path builds, loads or calls it.

The library carries the SHA-256 of the sources and flags it was built from
("ORACLE_BUILD_ID=<hex>"); ensure() rebuilds a library that is missing or stale, so that a
test never runs against an oracle older than its sources.
"""
import hashlib
import os
import re
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = ["philox.cpp", "shard.cpp", "fill.cpp", "capi.cpp"]
LIB = os.path.join(HERE, "liboracle.so")
# -ffp-contract=off: every fp32 operation of the definition rounds on its own.
FLAGS = ["-std=c++17", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-pthread", "-Wall", "-Wextra"]


def source_id() -> str:
    h = hashlib.sha256()
    h.update("\0".join(FLAGS + SOURCES).encode())
    for name in SOURCES + sorted(f for f in os.listdir(HERE) if f.endswith(".hpp")):
        with open(os.path.join(HERE, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read() + b"\0")
    return h.hexdigest()


def built_id():
    try:
        with open(LIB, "rb") as f:
            m = re.search(rb"ORACLE_BUILD_ID=([0-9a-f]{64})", f.read())
    except OSError:
        return None
    return m.group(1).decode() if m else None


def is_current() -> bool:
    return built_id() == source_id()


def build(verbose: bool = False) -> str:
    cmd = ["g++"] + FLAGS + ['-DORACLE_BUILD_ID="%s"' % source_id(), "-o", LIB] + [os.path.join(HERE, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


def ensure() -> str:
    if not is_current():
        build()
    return LIB


if __name__ == "__main__":
    build(verbose=True)
