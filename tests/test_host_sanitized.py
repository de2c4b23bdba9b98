"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU):
tests/host_check.cpp is built with g++ -fsanitize=address,undefined from the library's own
geometry.cpp and host_api.cpp and fed the brute-force grid of rank descriptions, random
descriptions with strides, descriptions at and beyond the fixed capacities, and tile-map requests
for shards too large to generate.  A sanitizer report aborts the program, which fails the test."""
import os
import subprocess

import numpy as np
import pytest

import oracle
from helpers import all_placements, mesh_coords

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2509_07003_amd", "csrc")
KIND = {"R": 0, "S": 1, "IS": 2, "P": 3}


@pytest.fixture(scope="module")
def host_check(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("host_check") / "host_check")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-Wall", "-Wextra", os.path.join(ROOT, "tests", "host_check.cpp"), os.path.join(CSRC, "geometry.cpp"),
           os.path.join(CSRC, "host_api.cpp"), "-o", exe]
    subprocess.run(cmd, check=True)

    def run(lines):
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=1", UBSAN_OPTIONS="halt_on_error=1")
        env.pop("LD_PRELOAD", None)   # the sanitizer runtime must come first in the program's library list
        res = subprocess.run([exe], input="\n".join(lines) + "\n", stdout=subprocess.PIPE, stderr=subprocess.PIPE,
                             text=True, env=env)
        assert res.returncode == 0, "sanitizer report or crash:\n" + res.stderr[-4000:]
        out = res.stdout.splitlines()
        assert len(out) == len(lines)
        return out

    return run


def sharding_words(shape, mesh, pls, coord, stride=None, theta=0):
    w = [len(shape)] + list(shape) + ([1] + list(stride) if stride is not None else [0])
    w += [len(mesh)] + list(mesh)
    for p in pls:
        w += [KIND[p[0]], p[1] if len(p) > 1 else 0, p[2] if len(p) > 2 else 1]
    return " ".join(str(int(x)) for x in w + list(coord) + [theta])


def parse_g(line):
    t = line.split()
    assert t[0] == "G"
    status, nd = int(t[1]), int(t[2])
    res = {"status": status}
    k = 3
    if status == 0:
        res["shape"] = [int(x) for x in t[k:k + nd]]
        res["numel"] = int(t[k + nd])
        k += nd + 1
        if t[k] == "J":
            n = res["numel"]
            res["J_status"], res["J"] = int(t[k + 1]), [int(x) for x in t[k + 2:k + 2 + n]]
            k += 2 + n
            assert t[k] == "K"
            res["K_status"], res["K"] = int(t[k + 1]), [int(x) for x in t[k + 2:k + 2 + n]]
            k += 2 + n
    assert t[k] == "A"
    res["A_status"], res["next"] = int(t[k + 1]), int(t[k + 2])
    return res


SHAPES = [[1], [7], [12], [2, 6], [6, 4], [5, 3], [3, 4, 2], [4, 6, 3], [2, 3, 2, 4], [1, 6, 1, 3]]
MESHES = [[1], [2], [3], [4], [2, 2], [2, 3], [3, 2], [4, 2], [2, 2, 2]]


def test_brute_force_grid_under_the_sanitizers(host_check):
    """Every rank of every mesh / placement assignment of the grid: local shape, the i -> j map of the
    kernels' decode plan and of the general route, and the offset advance, against the oracle."""
    cases, lines = [], []
    for shape in SHAPES:
        for mesh in MESHES:
            for pls in all_placements(len(shape), len(mesh)):
                for c in mesh_coords(mesh):
                    cases.append((shape, mesh, list(pls), list(c)))
                    lines.append("G " + sharding_words(shape, mesh, pls, c) + " 100000")
    out = host_check(lines)
    checked = 0
    for (shape, mesh, pls, c), line in zip(cases, out):
        got = parse_g(line)
        try:
            want_shape, want_n = oracle.local_shape(shape, mesh, pls, c)
        except oracle.OracleError:
            assert got["status"] == 5, (shape, mesh, pls, c)
            continue
        assert got["status"] == 0 and got["shape"] == want_shape and got["numel"] == want_n, (shape, mesh, pls, c)
        assert got["A_status"] == 0 and got["next"] == oracle.advance_offset(shape, 0)
        if want_n:
            want_j = [int(x) for x in oracle.global_indices(shape, mesh, pls, c).reshape(-1)]
            assert got["J_status"] == 0 and got["J"] == want_j, (shape, mesh, pls, c)
            assert got["K_status"] == 0 and got["K"] == want_j, (shape, mesh, pls, c)
        checked += 1
    assert checked > 29000


def test_random_descriptions_with_strides_under_the_sanitizers(host_check):
    from test_host_abi import _random_description
    rng = np.random.default_rng(20240607)
    cases = [_random_description(rng) for _ in range(1500)]
    out = host_check(["G " + sharding_words(*c) + " 100000" for c in cases])
    ok = 0
    for (shape, mesh, pls, coord, stride), line in zip(cases, out):
        got = parse_g(line)
        try:
            want_shape, want_n = oracle.local_shape(shape, mesh, pls, coord)
        except oracle.OracleError:
            assert got["status"] != 0
            continue
        assert got["status"] == 0 and got["shape"] == want_shape and got["numel"] == want_n
        assert got["next"] == oracle.advance_offset(shape, 0, stride)
        if want_n:
            want_j = [int(x) for x in oracle.global_indices(shape, mesh, pls, coord, stride).reshape(-1)]
            assert got["J"] == want_j and got["K"] == want_j, (shape, mesh, pls, coord, stride)
        ok += 1
    assert ok > 1000


def test_descriptions_at_and_beyond_the_fixed_capacities(host_check):
    """The geometry keeps its lists in fixed-size arrays (8 dimensions, 8 placements per dimension, 12
    axes per dimension): what fits is answered, what does not is refused with a status - never an
    overrun (the sanitizers watch)."""
    lines, want = [], []

    def add(words, status):
        lines.append("G " + words + " 5000")
        want.append(status)

    # Eight placements on ONE dimension: the capacity.  All interleaved, so every one adds an axis.
    shape = [2 ** 16]
    for kinds in ([("IS", 0, 2)] * 8, [("S", 0)] * 8, [("IS", 0, 4), ("S", 0)] * 4, [("IS", 0, 2), ("IS", 0, 8)] * 4):
        for coord in ([0] * 8, [1] * 8, [1, 0] * 4):
            add(sharding_words(shape, [2] * 8, kinds, coord), None)
    # Eight dimensions, every one interleaved by its own mesh dimension.
    add(sharding_words([4] * 8, [2] * 8, [("IS", d, 2) for d in range(8)], [1] * 8), None)
    # Beyond the capacities: refused by status.
    add(sharding_words([2] * 9, [1], [("R",)], [0]), 2)                       # nine tensor dimensions
    add(sharding_words([64], [2] * 9, [("S", 0)] * 9, [0] * 9), 3)            # nine mesh dimensions
    add(sharding_words([64], [2], [("S", 3)], [0]), 5)                        # dimension out of range
    add(sharding_words([64], [2], [("S", -1)], [0]), 5)
    add(sharding_words([64], [2], [("IS", 0, 0)], [0]), 5)
    add(sharding_words([64], [2], [("IS", 0, -4)], [0]), 5)
    add(sharding_words([64], [2], [("S", 0)], [2]), 4)
    add(sharding_words([64, -1], [2], [("S", 0)], [1]), 2)
    add(sharding_words([2 ** 40, 2 ** 40], [1], [("R",)], [0]), 2)            # element count beyond 2^62
    add(sharding_words([2 ** 31, 2 ** 30], [2], [("S", 0)], [1], stride=[2 ** 62, 1]), 10)   # stride overflow
    add(sharding_words([4, 4], [1], [("R",)], [0], stride=[4, 0]), 10)
    out = host_check(lines)
    for line, st in zip(out, want):
        got = parse_g(line)
        if st is not None:
            assert got["status"] == st, line[:80]
            continue
        assert got["status"] in (0, 9), line[:80]          # answered, or "unsupported": nothing in between
        if got["status"] == 0 and "J" in got:
            assert got["J"] == got["K"]                       # the two routes agree where both exist
    # The capacity cases against the oracle (its lists have no capacity).
    for kinds in ([("IS", 0, 2)] * 8, [("IS", 0, 4), ("S", 0)] * 4):
        for coord in ([0] * 8, [1, 0] * 4):
            got = parse_g(host_check(["G " + sharding_words(shape, [2] * 8, kinds, coord) + " 5000"])[0])
            want_shape, want_n = oracle.local_shape(shape, [2] * 8, kinds, coord)
            assert got["status"] == 0 and got["shape"] == want_shape
            assert got["K"] == [int(x) for x in oracle.global_indices(shape, [2] * 8, kinds, coord).reshape(-1)]
            assert got["J"] == got["K"]


# ------------------------------------------------------------------ tile map ----
def parse_t(line):
    head, *tiles = line.split(" | ")
    t = head.split()
    assert t[0] == "T" and t[1] == "0", line[:200]
    res = {"flavour": int(t[2]), "wide": int(t[3]), "units_per_run": int(t[4]), "tile_units": int(t[5]),
           "n_tiles": int(t[6]), "short": (t[7] == "short=1") if len(t) > 7 else False, "tiles": []}
    for tile in tiles:
        w = tile.split()
        assert w[0] != "OUT-OF-TILE", "the kernel would write outside its LDS tile: " + tile[:100]
        i0, lim, count, dummy = int(w[0]), int(w[1]), int(w[2]), int(w[3])
        res["tiles"].append({"i0": i0, "lim": lim, "count": count, "dummy": dummy, "pos": [int(x) for x in w[4:]]})
    return res


TILED, TILED_BIG = 1, 2


def tile_request(words, offset, unit_elems, tileable, big, big_min, whole, tiles, limits=(0, 0, 16)):
    """limits: the staging kernels serve element counts in [limits[0], limits[1]) (0 = no upper limit) with runs of
    at least limits[2] elements."""
    return "T %s %d %d %d %d %d %d %d %d %d %d %s" % ((words, offset, unit_elems, tileable, big, big_min, whole) + tuple(limits)
                                                      + (len(tiles), " ".join(str(t) for t in tiles)))


def check_tiles(host_check, words, offset, unit_elems, big, position_of, local_numel, probe_elements, threads_units=256):
    """Asks for the tiles that hold the given local elements (plus the first and last two) and checks
    every slot: written exactly once, by the stream position of its local element."""
    first = parse_t(host_check([tile_request(words, offset, unit_elems, 1, big, 0, 0, [])])[0])
    assert first["flavour"] == (TILED_BIG if big else TILED)
    per = first["tile_units"] * unit_elems
    assert first["n_tiles"] == -(-local_numel // per)
    assert 32 <= first["tile_units"] <= threads_units * (4 if big else 1) and first["tile_units"] % 8 == 0
    want = sorted({0, 1, first["n_tiles"] - 2, first["n_tiles"] - 1} | {e // per for e in probe_elements}
                  | {e // per + 1 for e in probe_elements} | {max(0, e // per - 1) for e in probe_elements})
    want = [t for t in want if 0 <= t < first["n_tiles"]]
    got = parse_t(host_check([tile_request(words, offset, unit_elems, 1, big, 0, 0, want)])[0])
    assert len(got["tiles"]) == len(want)
    passes = (unit_elems // 4) * (4 if big else 1)
    for t, tile in zip(want, got["tiles"]):
        assert tile["i0"] == t * per and tile["lim"] == min(per, local_numel - t * per)
        assert tile["count"] <= passes * 256, "more generator blocks than the workgroup's passes cover"
        i = np.arange(tile["i0"], tile["i0"] + tile["lim"], dtype=np.uint64)
        assert tile["pos"] == [int(p) for p in position_of(i)], ("tile", t)
    return first, got


@pytest.mark.parametrize("run_len", [2 ** 31 + 1, 2 ** 32 + 1, 2 ** 32 + 2 ** 31 + 3, 2 ** 20 + 1])
def test_tile_map_of_a_single_misaligned_run_beyond_32_bits(host_check, run_len):
    """One contiguous shard that starts off a generator-block boundary takes the staging kernel with a
    single run.  For runs of 2^31 elements and more the tile map has to clamp the run's bounds to the
    tile BEFORE narrowing them: every slot of the first, last and 2^31 / 2^32-crossing tiles is written
    exactly once, with the position of its own element."""
    n = 2 * run_len                       # two ranks, chunk = run_len; rank 1 starts at run_len (odd: phase 1 or 3)
    words = sharding_words([n], [2], [("S", 0)], [1])
    offset = 1 << 36
    probes = [e for e in (2 ** 31 - 1, 2 ** 31, 2 ** 32 - 1, 2 ** 32, 2 ** 32 + 2 ** 31) if e < run_len]
    for big in (1, 0):
        head, got = check_tiles(host_check, words, offset, 4, big, lambda i: np.uint64(offset + run_len) + i, run_len,
                                probes)
        assert head["wide"] == (1 if run_len >= 2 ** 30 else 0)
        assert head["units_per_run"] == (run_len % 4 + run_len + 3) // 4


def test_tile_map_of_column_shards_with_equal_and_unequal_phases(host_check):
    """Ragged column shards (many runs): row lengths whose runs all start at the same phase (4100) and
    at rotating phases (4101), 4- and 8-element units, narrow and wide index types."""
    for rows, cols, unit_elems, big in ((16384, 4100, 4, 1), (16384, 4101, 4, 1), (4096, 4101, 8, 0), (300, 333, 4, 0),
                                        (300, 333, 8, 0), (2 ** 20 + 3, 4101, 4, 1)):
        words = sharding_words([rows, cols], [3], [("S", 1)], [1])
        w = -(-cols // 3)                      # rank 1's columns [w, 2w)
        offset = 4096

        def position_of(i, w=w, cols=cols):
            return np.uint64(offset) + (i // np.uint64(w)) * np.uint64(cols) + np.uint64(w) + i % np.uint64(w)

        n = rows * w
        head, _ = check_tiles(host_check, words, offset, unit_elems, big, position_of, n,
                              [n // 2, n // 3, 2 ** 31] if n > 2 ** 31 else [n // 2, n // 3])
        assert head["wide"] == (1 if n >= 2 ** 30 else 0)
        # The short form of the map serves the narrow shards whose row length is a multiple of four; check_tiles
        # has then walked it next to the general form (the program reports any field that differs).
        assert head["short"] == (cols % 4 == 0 and n < 2 ** 30)


def test_short_tile_map_at_its_limits(host_check):
    """The short form of the tile map (one division and two multiply-adds per block) needs a stride between runs
    of at least as many generator blocks as a run can touch.  Rows of a padded tensor, reached through the
    global stride, give runs that nearly fill their stride: stride / 4 equal to the blocks per run (taken),
    one below (refused: the general form serves), and every phase; each slot is still written exactly once
    with its own position."""
    rows, offset = 3000, 1 << 20
    for length, lead, row_stride, want_short in ((17, 3, 20, True), (18, 3, 20, False), (17, 0, 20, True),
                                                 (19, 1, 20, True), (18, 2, 20, True), (33, 7, 40, True),
                                                 (38, 1, 40, True), (38, 3, 40, False), (21, 2, 24, True)):
        # Shape [rows, 2, length] with strides [row_stride, lead, 1]; the rank holds index 1 of the middle dimension,
        # so its runs start at lead + r * row_stride (phase lead % 4).
        words = sharding_words([rows, 2, length], [2], [("S", 1)], [1], stride=[row_stride, lead, 1])
        if lead == 0:   # phase 0 from a plain replicated tensor with padded rows
            words = sharding_words([rows, length], [1], [("R",)], [0], stride=[row_stride, 1])

        def position_of(i, length=length, lead=lead, row_stride=row_stride):
            return np.uint64(offset + lead) + (i // np.uint64(length)) * np.uint64(row_stride) + i % np.uint64(length)

        n = rows * length
        for unit_elems in (4, 8):
            head, _ = check_tiles(host_check, words, offset, unit_elems, 0, position_of, n, [n // 2, n // 3, n - 5])
            assert head["short"] == want_short, (length, lead, row_stride)
            assert head["units_per_run"] == (lead % 4 + length + 3) // 4


def test_tile_map_on_random_column_shards(host_check):
    """Seeded random column shards - row counts, widths, paddings (row strides that are and are not multiples of
    four), mesh sizes, ranks, unit sizes, both tile sizes: every slot of the probed tiles is written exactly once
    with its own stream position, whichever form of the map the library takes (both are walked where the short
    form applies), and the short form is taken exactly when the row stride is a multiple of four."""
    rng = np.random.default_rng(20240607)
    done = short = 0
    while done < 60:
        rows = int(rng.integers(40, 4000))
        cols = int(rng.integers(40, 3000))
        m = int(rng.integers(2, 6))
        coord = int(rng.integers(0, m))
        pad = int(rng.choice([0, 0, 1, 2, 3, 4, 8, 13]))
        chunk = -(-cols // m)
        start = coord * chunk
        w = min(chunk, cols - start)
        if w < 16:
            continue
        row_stride = cols + pad
        offset = 4 * int(rng.integers(0, 1 << 30))
        unit_elems = int(rng.choice([4, 8]))
        big = int(rng.integers(0, 2)) if unit_elems == 4 else 0
        aligned = (start % 4 == 0 and row_stride % 4 == 0 and w % unit_elems == 0)
        if aligned:
            continue                      # takes the aligned kernel: no tile map
        words = sharding_words([rows, cols], [m], [("S", 1)], [coord], stride=[row_stride, 1] if pad else None)

        def position_of(i, w=w, start=start, row_stride=row_stride, offset=offset):
            return np.uint64(offset + start) + (i // np.uint64(w)) * np.uint64(row_stride) + i % np.uint64(w)

        n = rows * w
        head, _ = check_tiles(host_check, words, offset, unit_elems, big, position_of, n,
                              [int(x) for x in rng.integers(0, n, size=3)])
        assert head["short"] == (row_stride % 4 == 0), (rows, cols, m, coord, pad)
        short += head["short"]
        done += 1
    assert 10 <= short <= 50


def test_staging_limits_of_an_operator(host_check):
    """An operator may leave shards outside an element-count window, or with short runs, to the kernel without
    staging (the fp32 normal fill above 2^24 elements; the 16-bit fills outside 2^21 .. 2^25 or with runs under 256)."""
    RAGGED = 3
    for rows, cols, limits, want in ((4096, 4096, (0, 1 << 24, 16), TILED_BIG),          # 5.6 M elements: inside
                                     (16384, 4096, (0, 1 << 24, 16), RAGGED),            # 22 M: beyond the window
                                     (1024, 4096, (0, 1 << 24, 16), TILED),              # 1.4 M: small tile
                                     (1024, 4096, (1 << 21, 1 << 25, 256), RAGGED),      # below the window
                                     (2048, 4096, (1 << 21, 1 << 25, 256), TILED),       # 2.8 M, runs of 1366
                                     (30000, 303, (1 << 21, 1 << 25, 256), RAGGED),      # 3 M, runs of 101: too short
                                     (30000, 303, (0, 0, 16), TILED)):
        words = sharding_words([rows, cols], [3], [("S", 1)], [1])
        head = parse_t(host_check([tile_request(words, 0, 4, 1, 1, 1 << 22, 0, [], limits)])[0])
        assert head["flavour"] == want, (rows, cols, limits)


def test_divisions_by_launch_constants_against_exact_integers(host_check):
    """The kernels divide by launch constants: with a high multiply and a shift where dividends stay below 2^31
    (plan.h: Div32), by the compiler's division on the 64-bit index path (Div64).  Divisors of every size class - 1, powers of two and their neighbours,
    the largest values, random ones - against Python's integers on dividends that sit on and next to multiples of
    the divisor, at the ends of the range, and at random."""
    rng = np.random.default_rng(64)
    divisors = [1, 2, 3, 5, 7, 10, 255, 256, 257, 1366, 4096, 65535, 65536, 65537, 2 ** 31 - 1, 2 ** 31, 2 ** 31 + 1,
                2 ** 32 - 1, 2 ** 32, 2 ** 32 + 1, 2 ** 33 + 5, 2 ** 40 - 87, 2 ** 62, 2 ** 63 - 1, 2 ** 63, 2 ** 63 + 1,
                2 ** 64 - 2, 2 ** 64 - 1]
    divisors += [int(x) for x in rng.integers(1, 2 ** 20, size=40)] + [int(x) for x in rng.integers(1, 2 ** 62, size=40)]
    divisors += [int(rng.integers(1, 2 ** 32)) * int(rng.integers(1, 2 ** 31)) for _ in range(20)]
    lines, cases = [], []
    for d in divisors:
        ns = {0, 1, d - 1, d, d + 1, 2 * d - 1, 2 * d, 2 ** 31 - 1, 2 ** 31, 2 ** 32 - 1, 2 ** 32, 2 ** 63 - 1, 2 ** 63,
              2 ** 64 - 1, 2 ** 64 - 2, (2 ** 64 - 1) // d * d, (2 ** 64 - 1) // d * d - 1}
        ns |= {int(k) * d + int(r) for k, r in zip(rng.integers(0, max(1, (2 ** 64 - 1) // d), size=24, dtype=np.uint64),
                                                   rng.integers(0, min(d, 2 ** 62), size=24))}
        ns |= {int(x) for x in rng.integers(0, 2 ** 63, size=16)} | {int(x) for x in rng.integers(0, 2 ** 31, size=16)}
        ns = sorted(x for x in ns if 0 <= x < 2 ** 64)
        lines.append("D %d %s" % (d, " ".join(str(x) for x in ns)))
        cases.append((d, ns))
    for line, (d, ns) in zip(host_check(lines), cases):
        wide, narrow = line[1:].split("|")
        assert [int(x) for x in wide.split()] == [x // d for x in ns], d
        if d <= 2 ** 31:
            assert [int(x) for x in narrow.split()] == [x // d for x in ns if x < 2 ** 31], d


def test_shards_that_need_64_bit_indices_are_cut_into_pieces(host_check):
    """A shard of 2^30 elements and more is served by the 32-bit kernels piece by piece when its outermost axis of
    runs can be cut into groups of 32 or more indices that fit: the pieces cover the axis, fit, and start on
    128-byte lines; a shard that cannot be cut (one run; rows too long) keeps the 64-bit kernels."""
    cases = [([2 ** 17, 2 ** 15], [2], [("S", 1)], [1], 4, True, 2 ** 14, 2 ** 17, 2 ** 15),      # rows of 16384 elements
             ([2 ** 25, 100], [2], [("S", 1)], [1], 4, True, 50, 2 ** 25, 100),                   # rows of 50
             ([2 ** 20, 4099], [2], [("S", 1)], [1], 4, True, 2049, 2 ** 20, 4099),               # ragged rows
             ([16, 2 ** 12, 2 ** 15], [2], [("S", 2)], [0], 8, True, 2 ** 14, 2 ** 16, 2 ** 15),  # two axes that merge into one
             ([16, 2 ** 13, 2 ** 14], [2], [("S", 1)], [1], 8, True, 2 ** 26, 16, 2 ** 27),       # runs of 2^26: 15 rows per piece
             ([64, 2 ** 26], [2], [("S", 1)], [1], 4, True, 2 ** 25, 64, 2 ** 26),                # rows of 2^25: 31 per piece
             ([2 ** 32], [2], [("S", 0)], [1], 4, True, None, None, None),                        # a single run
             ([2 ** 14, 2 ** 15], [2], [("S", 1)], [1], 4, False, None, None, None)]              # fits 32 bits as a whole
    for shape, mesh, pls, coord, unit_elems, wide, per_index, extent, stride in cases:
        out = host_check(["P %s 0 %d" % (sharding_words(shape, mesh, pls, coord), unit_elems)])[0].split()
        assert out[0] == "P" and int(out[1]) == int(wide), shape
        cut, rows, got_per, got_extent, got_stride, fit = (int(x) for x in out[2:8])
        if per_index is None:
            assert (not wide) or cut == 0, shape
            continue
        assert (got_per, got_extent, got_stride) == (per_index, extent, stride), shape
        want_cut = (2 ** 30 - 1) // per_index >= 32 and extent >= 1
        assert cut == int(want_cut), shape
        if cut:
            assert rows % 32 == 0 and rows >= 32 and rows * per_index < 2 ** 30 and fit == 1, shape
            assert rows + 32 > (2 ** 30 - 1) // per_index      # the largest such group
