"""Host-side checks of the library (no GPU): the shared object loads and exports what
include/vesrng.h declares, its closed-form shard geometry and kernel decode plan agree
with the oracle's simulated index lists, and every error path returns its status."""
import ctypes
import itertools
import os
import re

import numpy as np
import pytest

import oracle
import paper_2509_07003_amd as v
from helpers import all_placements, mesh_coords
from paper_2509_07003_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(header_name):
    header = open(os.path.join(ROOT, "include", header_name)).read()
    return sorted(set(re.findall(r"\b(vesrng_[a-z0-9_]+)\s*\(", header)))


def _exported(path):
    """Names in the dynamic symbol table of a shared library that it defines itself (hipcc's own
    one-byte compilation-unit markers, __hip_cuid_<hash>, aside)."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", path], check=True, stdout=subprocess.PIPE, text=True).stdout
    names = [line.split()[-1] for line in out.splitlines() if line.split()[1] in "TDBRWV"]
    return sorted(n for n in names if not n.startswith("__hip_cuid_"))


def test_library_exports_exactly_the_declared_symbols():
    """libvesrng.so exports the entry points include/vesrng.h declares - the method's operators, the
    host-side geometry / offset calls and the two host test hooks - and nothing else: no measurement
    aid, no stray C++ symbol."""
    declared = _declared("vesrng.h")
    assert declared == ["vesrng_advance_offset", "vesrng_dropout", "vesrng_dropout_add", "vesrng_global_index",
                        "vesrng_global_index_general", "vesrng_local_shape", "vesrng_normal", "vesrng_randint",
                        "vesrng_raw_u32", "vesrng_status_string", "vesrng_uniform"]
    assert _exported(v.library_path()) == declared
    assert declared == binding.EXPORTS
    lib = ctypes.CDLL(v.library_path())
    for name in declared:
        assert hasattr(lib, name), name


def test_bench_library_exports_exactly_its_header_and_is_separate():
    """The measurement aids live in their own header and library, which the product binding never loads."""
    from paper_2509_07003_amd import bench_binding
    declared = _declared("vesrng_bench.h")
    assert declared == bench_binding.EXPORTS
    assert _exported(bench_binding.library_path()) == declared
    assert bench_binding.library_path() != v.library_path()
    src = open(os.path.join(ROOT, "paper_2509_07003_amd", "binding.py")).read()
    assert "bench" not in src and "probe" not in src


def test_loaders_rebuild_a_stale_library(tmp_path):
    """A library built from other sources than the ones present is not loaded as it is: the build
    identity embedded in the binary must match the hash of the sources, for the product and the oracle."""
    from paper_2509_07003_amd import build as lib_build
    from oracle import build as oracle_build
    for t in lib_build.TARGETS:
        assert lib_build.is_current(t), t
    assert oracle_build.is_current()
    assert lib_build.built_id("vesrng") == lib_build.source_id("vesrng") != lib_build.source_id("bench")
    # The same check fails on a tree whose sources differ from the binary's (one byte appended).
    import shutil
    import subprocess
    import sys
    pkg = tmp_path / "paper_2509_07003_amd"
    shutil.copytree(os.path.join(ROOT, "paper_2509_07003_amd"), pkg, ignore=shutil.ignore_patterns("__pycache__", "*variant*"))
    shutil.copytree(os.path.join(ROOT, "include"), tmp_path / "include")
    with open(pkg / "csrc" / "plan.h", "a") as f:
        f.write("\n")
    assert (pkg / "libvesrng.so").exists()
    env = dict(os.environ, HIPCC="/bin/false", PYTHONPATH=str(tmp_path))
    res = subprocess.run([sys.executable, "-c", "import paper_2509_07003_amd"], env=env, cwd=str(tmp_path),
                         stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
    # The binary is there, but stale: the loader tries to rebuild it and, unable to, refuses to load it.
    assert res.returncode != 0 and "hipcc failed building libvesrng.so" in res.stderr


def test_status_strings():
    for st in range(13):
        assert v.vesrng_status_string(st) and "unknown" not in v.vesrng_status_string(st)
    assert "unknown" in v.vesrng_status_string(99)


SHAPES = [[1], [7], [12], [2, 6], [6, 4], [5, 3], [3, 4, 2], [4, 6, 3], [2, 3, 2, 4], [1, 6, 1, 3]]
MESHES = [[1], [2], [3], [4], [2, 2], [2, 3], [3, 2], [4, 2], [2, 2, 2]]


def test_geometry_and_decode_plan_match_the_oracle_brute_force():
    """Every rank of every mesh / placement assignment: local shape and the i -> j map of the
    kernels' decode plan (box form where the shard is a box, else the placement chain) and of
    the general route alone, against the oracle's simulated index lists."""
    checked = 0
    for shape in SHAPES:
        for mesh in MESHES:
            for pls in all_placements(len(shape), len(mesh)):
                for c in mesh_coords(mesh):
                    try:
                        want_shape, want_n = oracle.local_shape(shape, mesh, list(pls), list(c))
                    except oracle.OracleError:
                        with pytest.raises(v.VesrngError) as e:
                            v.vesrng_local_shape(v.Sharding(shape, mesh, pls, c))
                        assert e.value.status == 5
                        continue
                    sh = v.Sharding(shape, mesh, pls, c)
                    assert v.vesrng_local_shape(sh) == (want_shape, want_n), (shape, mesh, pls, c)
                    checked += 1
                    if want_n:
                        want_j = list(oracle.global_indices(shape, mesh, list(pls), list(c)).reshape(-1))
                        assert v.vesrng_global_index(sh, range(want_n)) == want_j, (shape, mesh, pls, c)
                        assert v.vesrng_global_index_general(sh, range(want_n)) == want_j, (shape, mesh, pls, c)
    assert checked > 29000


def test_shards_that_are_not_boxes_take_the_general_route():
    # 12 entries in 2 groups, cut in 2, then the 6 survivors cut in 3: rank (1,1) holds {5, 9}.
    sh = v.Sharding([12], [2, 3], [("IS", 0, 2), ("S", 0)], [1, 1])
    assert v.vesrng_local_shape(sh) == ([2], 2)
    assert v.vesrng_global_index(sh, [0, 1]) == [5, 9]
    # Interleave on an already interleaved dimension whose groups do not nest.
    args = ([4, 36], [3, 2, 2], [("IS", 1, 4), ("IS", 1, 3), ("S", 1)], [2, 1, 0])
    sh = v.Sharding(*args)
    n = v.vesrng_local_shape(sh)[1]
    assert n == oracle.local_shape(*args)[1] and n > 0
    assert v.vesrng_global_index(sh, range(n)) == list(oracle.global_indices(*args).reshape(-1))


def test_plain_shard_and_replicate_are_always_supported():
    rng = np.random.default_rng(17)
    for _ in range(300):
        nd = int(rng.integers(1, 6))
        shape = [int(x) for x in rng.integers(1, 12, size=nd)]
        md = int(rng.integers(1, 4))
        mesh = [int(x) for x in rng.integers(1, 6, size=md)]
        pls = [("S", int(rng.integers(0, nd))) if rng.random() < 0.75 else ("R",) for _ in range(md)]
        c = [int(rng.integers(0, p)) for p in mesh]
        sh = v.Sharding(shape, mesh, pls, c)
        want_shape, want_n = oracle.local_shape(shape, mesh, pls, c)
        assert v.vesrng_local_shape(sh) == (want_shape, want_n)
        if want_n:
            want_j = oracle.global_indices(shape, mesh, pls, c).reshape(-1)
            assert v.vesrng_global_index(sh, range(want_n)) == list(want_j)


def test_global_stride_is_honoured():
    shape, stride = [3, 4, 5], [1, 3, 12]      # a permuted (column-major) global view
    for c in range(2):
        sh = v.Sharding(shape, [2], [("S", 1)], [c], global_stride=stride)
        n = v.vesrng_local_shape(sh)[1]
        want = oracle.global_indices(shape, [2], [("S", 1)], [c], global_stride=stride).reshape(-1)
        assert v.vesrng_global_index(sh, range(n)) == list(want)


def test_wide_index_path_on_a_tensor_beyond_32_bits():
    # 2^34 elements, column-sharded so that runs do not merge; indices need 64 bits.
    shape, mesh, pls, c = [1 << 14, 1 << 20], [4, 2], [("S", 1), ("S", 0)], [3, 1]
    sh = v.Sharding(shape, mesh, pls, c)
    lshape, n = v.vesrng_local_shape(sh)
    assert lshape == [1 << 13, 1 << 18] and n == 1 << 31
    rows = oracle.index_list(shape, mesh, pls, c, 0)
    cols = oracle.index_list(shape, mesh, pls, c, 1)
    rng = np.random.default_rng(1)
    idx = [0, n - 1, (1 << 18) - 1, 1 << 18] + [int(x) for x in rng.integers(0, n, size=200)]
    want = [int(rows[i >> 18]) * (1 << 20) + int(cols[i & ((1 << 18) - 1)]) for i in idx]
    assert v.vesrng_global_index(sh, idx) == want
    assert max(want) >= 1 << 33


def test_config_shards():
    assert v.vesrng_local_shape(v.Sharding([4096, 4096], [3], [("S", 1)], [2])) == ([4096, 1364], 4096 * 1364)
    assert v.vesrng_local_shape(v.Sharding([8, 32, 4096, 4096], [4, 2], [("S", 1), ("S", 1)], [3, 1])) == \
        ([8, 4, 4096, 4096], 1 << 29)
    sh = v.Sharding([8, 32, 4096, 4096], [4, 2], [("S", 1), ("S", 1)], [3, 1])
    assert v.vesrng_global_index(sh, [0, (1 << 26) - 1, 1 << 26]) == \
        [28 << 24, (32 << 24) - 1, (32 << 24) + (28 << 24)]
    assert v.vesrng_local_shape(v.Sharding([3, 5], [4], [("S", 0)], [3])) == ([0, 5], 0)   # empty shard
    assert v.vesrng_local_shape(v.Sharding([], [2], [("R",)], [1])) == ([], 1)             # 0-d tensor


def test_advance_offset():
    for shape, off in (([4096, 4096], 0), ([5], 8), ([8], 8), ([3, 3], 0), ([], 4), ([0, 9], 4), ([1 << 20, 1 << 14], 1 << 40)):
        sh = v.Sharding(shape, [2], [("S", 0)] if shape else [("R",)], [1])
        assert v.vesrng_advance_offset(sh, off) == oracle.advance_offset(shape, off)
    # The same for every rank, whatever the placement.
    a = v.vesrng_advance_offset(v.Sharding([10, 10], [4], [("S", 1)], [0]), 16)
    b = v.vesrng_advance_offset(v.Sharding([10, 10], [2, 2], [("R",), ("S", 0)], [1, 1]), 16)
    assert a == b == 116
    # Virtual-thread layout: ceil(N / theta) steps per thread.
    for theta in (1, 5, 60, 1 << 40):
        assert v.vesrng_advance_offset(v.Sharding([6, 10], virtual_threads=theta), 16) == \
            oracle.advance_offset([6, 10], 16, None, theta)
    with pytest.raises(v.VesrngError) as e:
        v.vesrng_advance_offset(v.Sharding([10]), 3)
    assert e.value.status == 6
    with pytest.raises(v.VesrngError) as e:
        v.vesrng_advance_offset(v.Sharding([1 << 40]), (1 << 64) - 8)
    assert e.value.status == 10


def _status(fn, *args):
    with pytest.raises(v.VesrngError) as e:
        fn(*args)
    return e.value.status


def test_error_paths_return_their_status_without_touching_the_gpu():
    ok = v.Sharding([8, 8], [2], [("S", 0)], [0])
    buf = 1 << 20   # a fake, 16-byte aligned device address: never dereferenced on an error path
    assert _status(v.vesrng_local_shape, v.Sharding([4, -1])) == 2
    assert _status(v.vesrng_local_shape, v.Sharding([2] * 9)) == 2
    assert _status(v.vesrng_local_shape, v.Sharding([1 << 40, 1 << 40])) == 2
    assert _status(v.vesrng_local_shape, v.Sharding([4], [0], [("S", 0)], [0])) == 3
    assert _status(v.vesrng_local_shape, v.Sharding([4], [2], [("S", 0)], [2])) == 4
    assert _status(v.vesrng_local_shape, v.Sharding([4], [2], [("S", 0)], [-1])) == 4
    assert _status(v.vesrng_local_shape, v.Sharding([4], [2], [("P",)], [0])) == 5
    assert _status(v.vesrng_local_shape, v.Sharding([4], [2], [("S", 1)], [0])) == 5
    assert _status(v.vesrng_local_shape, v.Sharding([6], [2], [("IS", 0, 4)], [0])) == 5
    assert _status(v.vesrng_local_shape, v.Sharding([6], [2], [("IS", 0, 0)], [0])) == 5
    assert _status(v.vesrng_local_shape, v.Sharding([4, 4], global_stride=[4, 0])) == 10
    assert _status(v.vesrng_uniform, ok, v.F32, 0.0, 1.0, 1, 2, buf) == 6
    assert _status(v.vesrng_uniform, ok, v.F32, 2.0, 1.0, 1, 0, buf) == 7
    assert _status(v.vesrng_uniform, ok, v.F32, 0.0, float("inf"), 1, 0, buf) == 7
    assert _status(v.vesrng_uniform, ok, v.F32, float("nan"), 1.0, 1, 0, buf) == 7
    assert _status(v.vesrng_uniform, ok, 7, 0.0, 1.0, 1, 0, buf) == 8
    assert _status(v.vesrng_uniform, ok, v.F32, 0.0, 1.0, 1, 0, None) == 1
    assert _status(v.vesrng_uniform, ok, v.F32, 0.0, 1.0, 1, 0, buf + 4) == 12
    assert _status(v.vesrng_uniform, ok, v.F32, 0.0, 1.0, 1, (1 << 64) - 16, buf) == 10
    assert _status(v.vesrng_normal, ok, v.F32, 0.0, -1.0, 1, 0, buf) == 7
    assert _status(v.vesrng_normal, ok, v.BF16, float("nan"), 1.0, 1, 0, buf) == 7
    assert _status(v.vesrng_normal, ok, 3, 0.0, 1.0, 1, 0, buf) == 8
    assert _status(v.vesrng_dropout, ok, v.BF16, 1.5, 1, 0, buf, buf, None) == 7
    assert _status(v.vesrng_dropout, ok, v.BF16, -0.1, 1, 0, buf, buf, None) == 7
    assert _status(v.vesrng_dropout, ok, v.BF16, 0.1, 1, 0, None, buf, None) == 1
    assert _status(v.vesrng_dropout, ok, v.BF16, 0.1, 1, 0, buf, buf, buf + 1) == 12
    assert _status(v.vesrng_dropout, ok, v.BF16, 0.1, 1, 1, buf, buf, None) == 6
    assert _status(v.vesrng_randint, ok, 5, 5, 1, 0, buf) == 7
    assert _status(v.vesrng_randint, ok, 0, (1 << 32) + 1, 1, 0, buf) == 7
    assert _status(v.vesrng_raw_u32, ok, 1, 0, None) == 1
    assert _status(v.vesrng_raw_u32, v.Sharding([4], [2], [("P",)], [0]), 1, 0, buf) == 5
    from paper_2509_07003_amd import bench_binding as b
    assert _status(b.vesrng_bench_probe, b.PROBE_COPY, 16, None, buf) == 1
    assert _status(b.vesrng_bench_probe, b.PROBE_DROPOUT_TRAFFIC, 16, buf, buf, None) == 1
    assert _status(b.vesrng_bench_probe, b.PROBE_STORE, 16, None, buf + 8) == 12
    assert _status(b.vesrng_bench_probe, 99, 16, buf, buf, buf) == 7
    assert _status(b.vesrng_bench_alu, 99, 16, 16, buf) == 7
    assert _status(b.vesrng_bench_alu, 0, 16, 16, None) == 1
    assert _status(b.vesrng_bench_clock, 16, None) == 1
    b.vesrng_bench_probe(b.PROBE_STORE, 0, None, None)
    # Empty shard: fine, nothing to launch, pointers not needed.
    v.vesrng_uniform(v.Sharding([3, 5], [4], [("S", 0)], [3]), v.F32, 0.0, 1.0, 1, 0, None)
    v.vesrng_dropout(v.Sharding([0]), v.BF16, 0.1, 1, 0, None, None, None)


def _random_description(rng, max_extent=9, allow_stride=True):
    nd = int(rng.integers(1, 6))
    shape = [int(x) for x in rng.integers(1, max_extent + 1, size=nd)]
    md = int(rng.integers(1, 4))
    mesh = [int(x) for x in rng.integers(1, 5, size=md)]
    pls = []
    for _ in range(md):
        r = rng.random()
        d = int(rng.integers(0, nd))
        if r < 0.2:
            pls.append(("R",))
        elif r < 0.75:
            pls.append(("S", d))
        else:
            pls.append(("IS", d, int(rng.integers(1, 5))))
    coord = [int(rng.integers(0, p)) for p in mesh]
    stride = None
    if allow_stride and rng.random() < 0.3:
        # A permuted, padded global layout: strides of a random dimension order with gaps.
        order = list(rng.permutation(nd))
        stride, acc = [0] * nd, 1
        for d in order:
            stride[d] = acc
            acc *= shape[d] + int(rng.integers(0, 3))
    return shape, mesh, pls, coord, stride


def test_random_descriptions_against_the_oracle():
    rng = np.random.default_rng(20240607)
    ok = 0
    for _ in range(1500):
        shape, mesh, pls, coord, stride = _random_description(rng)
        try:
            want_shape, want_n = oracle.local_shape(shape, mesh, pls, coord)
        except oracle.OracleError:
            with pytest.raises(v.VesrngError):
                v.vesrng_local_shape(v.Sharding(shape, mesh, pls, coord, stride))
            continue
        sh = v.Sharding(shape, mesh, pls, coord, stride)
        assert v.vesrng_local_shape(sh) == (want_shape, want_n)
        if want_n:
            want_j = list(oracle.global_indices(shape, mesh, pls, coord, stride).reshape(-1))
            assert v.vesrng_global_index(sh, range(want_n)) == want_j, (shape, mesh, pls, coord, stride)
            assert v.vesrng_global_index_general(sh, range(want_n)) == want_j, (shape, mesh, pls, coord, stride)
        ok += 1
    assert ok > 1000


def test_header_is_plain_c_and_links_from_c(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 and a C program can call the
    host-only entry points of the shared library."""
    import subprocess
    src = tmp_path / "abi.c"
    src.write_text(r'''
#include <stdio.h>
#include "vesrng.h"
int main(void) {
  int64_t shape[2] = {4096, 4096};
  int32_t mesh[1] = {3}, coord[1] = {2};
  vesrng_placement pl[1] = {{VESRNG_SHARD, 1, 0}};
  vesrng_sharding s = {2, shape, 0, 1, mesh, pl, coord, 0};
  int64_t local[2], n;
  uint64_t next;
  if (vesrng_local_shape(&s, local, &n) != VESRNG_OK) return 1;
  if (vesrng_advance_offset(&s, 0, &next) != VESRNG_OK) return 2;
  printf("%lld %lld %lld %llu %s\n", (long long)local[0], (long long)local[1], (long long)n,
         (unsigned long long)next, vesrng_status_string(VESRNG_ERR_OFFSET_ALIGN));
  return vesrng_uniform(&s, VESRNG_F32, 0.0, 1.0, 1, 2, (void*)16, 0) == VESRNG_ERR_OFFSET_ALIGN ? 0 : 3;
}
''')
    exe = tmp_path / "abi"
    lib = v.library_path()
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"), str(src),
                    "-o", str(exe), lib, "-Wl,-rpath," + os.path.dirname(lib)], check=True)
    out = subprocess.run([str(exe)], check=True, stdout=subprocess.PIPE, text=True).stdout.split(None, 4)
    assert out[:4] == ["4096", "1364", str(4096 * 1364), "16777216"]
    assert "multiple of 4" in out[4]


def test_import_fails_loudly_without_the_native_library(tmp_path):
    """No CPU fallback: a copy of the package without libvesrng.so and without a working hipcc
    must refuse to import rather than compute anything some other way."""
    import shutil
    import subprocess
    import sys
    pkg = tmp_path / "paper_2509_07003_amd"
    pkg.mkdir()
    for name in ("__init__.py", "binding.py", "build.py", "workloads.py"):
        shutil.copy(os.path.join(ROOT, "paper_2509_07003_amd", name), pkg / name)
    env = dict(os.environ, HIPCC="/bin/false", PYTHONPATH=str(tmp_path))
    res = subprocess.run([sys.executable, "-c", "import paper_2509_07003_amd"], env=env, cwd=str(tmp_path),
                         stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
    assert res.returncode != 0
    assert "hipcc failed" in res.stderr or "libvesrng" in res.stderr


def test_generator_state_advances_by_the_global_tensor_on_every_rank():
    """The caller-side (seed, offset) bookkeeping: the offset moves by what the operator consumes on
    the GLOBAL tensor (the oracle's rule), identically for every rank and placement."""
    tensors = [([1024, 1024], None), ([5], None), ([3, 3], None), ([4096, 4096], None), ([7, 9], [20, 2]), ([], None)]
    want = 64
    track = [want]
    for shape, stride in tensors:
        want = oracle.advance_offset(shape, want, stride)
        track.append(want)
    for mesh, pls_of, coords in (([1], lambda d: [("R",)], [(0,)]), ([4], lambda d: [("S", 0)] if d else [("R",)], [(0,), (3,)]),
                                 ([2, 2], lambda d: [("S", d - 1), ("R",)] if d else [("R",), ("R",)], [(0, 1), (1, 0)])):
        for coord in coords:
            g = v.Generator(seed=9, offset=64)
            seen = [g.offset]
            for shape, stride in tensors:
                g._advance(v.Sharding(shape, mesh, pls_of(len(shape)), list(coord), stride))
                seen.append(g.offset)
            assert seen == track, (mesh, coord)
    g = v.Generator(1, 8)
    g.set_state((5, 16))
    assert g.get_state() == (5, 16)
    with pytest.raises(ValueError):
        v.Generator(1, 6)
    with pytest.raises(ValueError):
        g.set_state((1, 2))


def test_library_carries_gfx950_device_code_only():
    """The in-tree library is built for MI355X: its device code object names gfx950 and no other GPU."""
    import re
    with open(v.library_path(), "rb") as f:
        blob = f.read()
    targets = set(re.findall(rb"amdgcn-amd-amdhsa--(gfx[0-9a-f]+)", blob))
    assert targets == {b"gfx950"}, targets


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it exits with a message instead of a number."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in (r.stderr + r.stdout) and "{" not in r.stdout
