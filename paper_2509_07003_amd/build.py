"""Builds the package's shared libraries in-tree with hipcc, for gfx950 only.

  libvesrng.so          the product: HIP kernels + the C ABI of include/vesrng.h
  libvesrng_bench.so    measurement aids of include/vesrng_bench.h (bench.py and its test only)
  libvesrng_variant_*   the product sources with ONE design choice flipped, so that the benchmark
                        can time a choice against its alternative (bench.py --design-choices only)

Every library carries the SHA-256 of what it was built from (sources, headers, flags) as a
"VESRNG_BUILD_ID=<hex>" string; a loader compares it with the sources it finds and rebuilds a
library that is missing or stale, so that an old binary is never tested or timed by accident.
"""
import hashlib
import os
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# -ffp-contract=off: every fp32 operation in the value definitions rounds on its own
# (fused multiply-adds are written out explicitly where they are meant).
# packed-fp32-ops is switched off for all device code.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
         "-fvisibility=hidden", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wextra", "-Wno-unused-command-line-argument"]

PRODUCT_SOURCES = ["kernels.hip", "geometry.cpp", "host_api.cpp", "vesrng.cpp"]
TARGETS = {
    "vesrng": {"lib": "libvesrng.so", "sources": PRODUCT_SOURCES, "defines": []},
    "bench": {"lib": "libvesrng_bench.so", "sources": ["probes.hip"], "defines": []},
    # The kernels without the argument-fetch pinning (early exit, no live-at-entry parameters).
    "variant_nopin": {"lib": "libvesrng_variant_nopin.so", "sources": PRODUCT_SOURCES,
                      "defines": ["VESRNG_VARIANT_TAG=nopin", "VESRNG_PIN_ARGUMENT_FETCH=0"]},
    # Whole units leave through the compiler's plain non-temporal store instead of sc1 nt.
    "variant_ntstore": {"lib": "libvesrng_variant_ntstore.so", "sources": PRODUCT_SOURCES,
                        "defines": ["VESRNG_VARIANT_TAG=ntstore", "VESRNG_STREAM_STORE_SC1=0"]},
    # Three-way XORs of the generator as two v_xor_b32.
    "variant_twoxor": {"lib": "libvesrng_variant_twoxor.so", "sources": PRODUCT_SOURCES,
                       "defines": ["VESRNG_VARIANT_TAG=twoxor", "VESRNG_PHILOX_BITOP3=0"]},
    # Aligned kernels with the run arithmetic per lane even where runs are whole wavefronts long.
    "variant_lanerun": {"lib": "libvesrng_variant_lanerun.so", "sources": PRODUCT_SOURCES,
                        "defines": ["VESRNG_VARIANT_TAG=lanerun", "VESRNG_WAVE_UNIFORM_RUNS=0"]},
    # The staging kernel with its tile map worked out once per wavefront in scalar registers (runs of 64 blocks and more).
    "variant_wavetile": {"lib": "libvesrng_variant_wavetile.so", "sources": PRODUCT_SOURCES,
                         "defines": ["VESRNG_VARIANT_TAG=wavetile", "VESRNG_TILE_WAVE_MAP=1"]},
    # The staging kernel with the general form of its tile map also where the short form applies.
    "variant_longmap": {"lib": "libvesrng_variant_longmap.so", "sources": PRODUCT_SOURCES,
                        "defines": ["VESRNG_VARIANT_TAG=longmap", "VESRNG_TILE_SAME_PHASE=0"]},
    # Fused dropout that writes a mask at the hardware's full eight resident waves per SIMD (no cap at seven).
    "variant_nocap": {"lib": "libvesrng_variant_nocap.so", "sources": PRODUCT_SOURCES,
                      "defines": ["VESRNG_VARIANT_TAG=nocap", "VESRNG_CAP_MASKED_DROPOUT_WAVES=0"]},
    # Shards of 2^30 elements and more through the 64-bit index kernels as a whole instead of piece by piece.
    "variant_widekernels": {"lib": "libvesrng_variant_widekernels.so", "sources": PRODUCT_SOURCES,
                            "defines": ["VESRNG_VARIANT_TAG=widekernels", "VESRNG_WIDE_SHARDS_IN_PIECES=0"]},
    # Two and three axes of runs through the loop over any number of axes instead of the written-out forms.
    "variant_loopaxes": {"lib": "libvesrng_variant_loopaxes.so", "sources": PRODUCT_SOURCES,
                         "defines": ["VESRNG_VARIANT_TAG=loopaxes", "VESRNG_EXACT_RUN_AXES=1"]},
    # Aligned randint with one thread per generator block, halves traded between neighbouring lanes, two stores per thread.
    "variant_pairint": {"lib": "libvesrng_variant_pairint.so", "sources": PRODUCT_SOURCES,
                        "defines": ["VESRNG_VARIANT_TAG=pairint", "VESRNG_RANDINT_HALF_BLOCKS=0"]},
    # Ragged shards: never staged through LDS, whole blocks stored element-aligned / realigned across lanes.
    "variant_ragged": {"lib": "libvesrng_variant_ragged.so", "sources": PRODUCT_SOURCES,
                       "defines": ["VESRNG_VARIANT_TAG=ragged", "VESRNG_TILING=0"]},
    "variant_realign": {"lib": "libvesrng_variant_realign.so", "sources": PRODUCT_SOURCES,
                        "defines": ["VESRNG_VARIANT_TAG=realign", "VESRNG_TILING=0", "VESRNG_RAGGED_DPP_REALIGN=1"]},
    # Ragged shards: every operator staged, always with the small tile / with the large tile where there is one.
    "variant_smalltile": {"lib": "libvesrng_variant_smalltile.so", "sources": PRODUCT_SOURCES,
                          "defines": ["VESRNG_VARIANT_TAG=smalltile", "VESRNG_TILING=1", "VESRNG_BIG_TILE_MIN_ELEMS=(1ull<<62)"]},
    "variant_bigtile": {"lib": "libvesrng_variant_bigtile.so", "sources": PRODUCT_SOURCES,
                        "defines": ["VESRNG_VARIANT_TAG=bigtile", "VESRNG_TILING=2", "VESRNG_BIG_TILE_MIN_ELEMS=0ull"]},
}
LIB = os.path.join(HERE, TARGETS["vesrng"]["lib"])


def lib_path(target: str = "vesrng") -> str:
    return os.path.join(HERE, TARGETS[target]["lib"])


def source_id(target: str = "vesrng") -> str:
    """SHA-256 over the flags, the target's defines and sources, and every header it can include."""
    t = TARGETS[target]
    h = hashlib.sha256()
    h.update(("\0".join(FLAGS + t["defines"] + t["sources"])).encode())
    files = [os.path.join(CSRC, s) for s in t["sources"]]
    files += sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".h", ".hpp")))
    files += sorted(os.path.join(INCLUDE, f) for f in os.listdir(INCLUDE) if f.endswith(".h"))
    for path in files:
        with open(path, "rb") as f:
            h.update(os.path.basename(path).encode() + b"\0" + f.read() + b"\0")
    return h.hexdigest()


def built_id(target: str = "vesrng"):
    """The build id embedded in the library file, or None if there is no such library."""
    try:
        with open(lib_path(target), "rb") as f:
            m = re.search(rb"VESRNG_BUILD_ID=([0-9a-f]{64})", f.read())
    except OSError:
        return None
    return m.group(1).decode() if m else None


def is_current(target: str = "vesrng") -> bool:
    return built_id(target) == source_id(target)


def build(target: str = "vesrng", verbose: bool = False) -> str:
    t = TARGETS[target]
    lib = lib_path(target)
    defines = ["-D" + d for d in t["defines"]] + ['-DVESRNG_BUILD_ID="%s"' % source_id(target)]
    cmd = [HIPCC] + FLAGS + defines + ["-x", "hip"] + [os.path.join(CSRC, s) for s in t["sources"]] + ["-o", lib]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # hipcc's host pass does not know the device-only feature flag; that warning is harmless.
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if verbose or res.returncode != 0:
        print(out, flush=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building " + t["lib"])
    return lib


def build_all(verbose: bool = False, jobs: int = min(8, os.cpu_count() or 1)):
    """Compiles every target, a few at a time (each hipcc run is single-threaded)."""
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        return list(pool.map(lambda name: build(name, verbose), TARGETS))


def ensure(target: str = "vesrng") -> str:
    """Path of an up-to-date library: rebuilt first when it is missing or was built from other
    sources.  Raises when that build fails - there is nothing to fall back to."""
    try:
        current = is_current(target)
    except OSError as e:
        raise RuntimeError("cannot check %s against its sources: %s" % (TARGETS[target]["lib"], e))
    if not current:
        build(target)
    return lib_path(target)


if __name__ == "__main__":
    build_all(verbose=True)
