"""Pins of the CPU oracle against things other than itself (no GPU needed):
published known-answer vectors, an independent big-integer evaluation, the paper's
merge invariant by brute force, closed forms, library routines and statistics."""
import itertools
import math
import os
import struct
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from helpers import NotGatherable, all_placements, merge_shards, mesh_coords

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _lines(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [l.strip() for l in f if l.strip() and not l.startswith("#")]


# ---------------------------------------------------------------- generator ----
def test_philox_known_answer_vectors():
    rows = _lines("philox4x32_10_kat.txt")
    assert len(rows) == 3
    for row in rows:
        lhs, rhs = row.split("->")
        w = [int(t, 16) for t in lhs.split()]
        want = [int(t, 16) for t in rhs.split()]
        assert oracle.philox4x32_10(w[:4], w[4:6]) == want


def _philox_bigint(ctr, key):
    """Philox-4x32-10 re-derived with unbounded Python integers from the SC'11
    description: an S-P network whose S-box is (L, R) -> (mullo(R, M), mulhi(R, M) ^ k ^ L)."""
    M = (0xD2511F53, 0xCD9E8D57)
    W = (0x9E3779B9, 0xBB67AE85)
    x = list(ctr)
    for r in range(10):
        k = [(key[0] + r * W[0]) % 2**32, (key[1] + r * W[1]) % 2**32]
        full0 = M[0] * x[0]
        full1 = M[1] * x[2]
        x = [(full1 // 2**32) ^ x[1] ^ k[0], full1 % 2**32, (full0 // 2**32) ^ x[3] ^ k[1], full0 % 2**32]
    return x


def test_philox_matches_bigint_rederivation():
    assert _philox_bigint([0] * 4, [0] * 2) == [0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8]
    rng = np.random.default_rng(2024)
    for _ in range(2000):
        w = [int(v) for v in rng.integers(0, 2**32, size=6)]
        assert oracle.philox4x32_10(w[:4], w[4:]) == _philox_bigint(w[:4], w[4:])


def test_philox_is_a_bijection_on_sampled_counters():
    # Distinct counters under one key never collide (the generator is a permutation).
    outs = {tuple(oracle.philox4x32_10([c, 0, 0, 0], [5, 9])) for c in range(4096)}
    assert len(outs) == 4096


def test_stream_layout_worked_blocks():
    # draw(seed, p): key = seed words, counter = block number, word = p mod 4.
    for row in _lines("worked_blocks.txt"):
        lhs, rhs = row.split("->")
        seed, block = [int(t) for t in lhs.split()]
        want = [int(t, 16) for t in rhs.split()]
        assert [oracle.draw(seed, 4 * block + l) for l in range(4)] == want
        assert _philox_bigint([block % 2**32, block >> 32, 0, 0], [seed % 2**32, seed >> 32]) == want


def test_seed_high_word_is_key_word_one():
    seed = (0x299f31d0 << 32) | 0xa4093822
    b = (0x05a308d3 << 32) | 0x243f6a88   # 4 * b still fits 64 bits
    # Counter words 2,3 are zero in the stream layout, so compare with the big-int form.
    want = _philox_bigint([0x243f6a88, 0x05a308d3, 0, 0], [0xa4093822, 0x299f31d0])
    assert [oracle.draw(seed, 4 * b + l) for l in range(4)] == want


def test_worked_values():
    for row in _lines("worked_values.txt"):
        lhs, rhs = row.split("->")
        op, seed, offset, j = lhs.split()
        seed, offset, j = int(seed), int(offset), int(j)
        n = j + 1
        sh = ([n], [1], [("R",)], [0])
        if op == "uniform":
            got = float(oracle.uniform(sh, oracle.F32, 0.0, 1.0, seed, offset, i_begin=j)[j])
            assert got == float(rhs)
        else:
            got = float(oracle.normal_f64_values(sh, 0.0, 1.0, seed, offset, i_begin=j)[j])
            assert abs(got - float(rhs)) < 1e-13 + 1e-13 * abs(float(rhs))


# ------------------------------------------------------------- geometry -------
def test_chunk_rule_matches_torch_chunk():
    for n in range(0, 40):
        for parts in range(1, 9):
            ref = torch.chunk(torch.arange(n), parts) if n else ()
            for r in range(parts):
                got = oracle.index_list([n], [parts], [("S", 0)], [r], 0)
                want = ref[r].numpy() if r < len(ref) else np.zeros(0, dtype=np.int64)
                assert np.array_equal(got, want), (n, parts, r)


def test_config_shapes_from_the_workload_list():
    # Ragged split named in the workload list: 4096 columns over 3 ranks -> 1366, 1366, 1364.
    sizes = [oracle.local_shape([4096, 4096], [3], [("S", 1)], [r])[0] for r in range(3)]
    assert sizes == [[4096, 1366], [4096, 1366], [4096, 1364]]
    assert oracle.local_shape([4096, 14336], [2, 4], [("S", 0), ("S", 1)], [1, 3])[0] == [2048, 3584]
    assert oracle.local_shape([8, 4096, 4096], [8], [("S", 1)], [5])[0] == [8, 512, 4096]
    shp, n = oracle.local_shape([8, 32, 4096, 4096], [4, 2], [("S", 1), ("S", 1)], [2, 1])
    assert shp == [8, 4, 4096, 4096] and n == 536870912
    # Nested split of one dimension: rank (a, b) holds heads 8a+4b .. 8a+4b+3.
    assert list(oracle.index_list([8, 32, 4, 4], [4, 2], [("S", 1), ("S", 1)], [2, 1], 1)) == [20, 21, 22, 23]
    # Interleaved: 32 heads in 4 groups of 8, rank r of 8 holds head r of every group.
    assert list(oracle.index_list([8, 32, 4, 4], [8], [("IS", 1, 4)], [3], 1)) == [3, 11, 19, 27]


def test_identity_special_cases():
    # One rank, or Replicate everywhere: j = i.
    for sh in (([5, 7], [1], [("R",)], [0]), ([5, 7], [2, 3], [("R",), ("R",)], [1, 2])):
        assert np.array_equal(oracle.global_indices(*sh).reshape(-1), np.arange(35, dtype=np.uint64))
    # Shard(0) of a contiguous tensor is a contiguous slice of the flat global tensor.
    for r in range(4):
        j = oracle.global_indices([8, 6], [4], [("S", 0)], [r]).reshape(-1)
        assert np.array_equal(j, np.arange(12 * r, 12 * r + 12, dtype=np.uint64))
    # Unsharded values are the stream itself.
    got = oracle.raw_u32(([3, 5], [1], [("R",)], [0]), 99, 8).reshape(-1)
    assert list(got) == [oracle.draw(99, 8 + i) for i in range(15)]


def test_global_index_matches_numpy_fancy_indexing():
    # j(i) against an independent route: index an arange "global tensor" with the
    # per-dimension lists via numpy's own gather.
    rng = np.random.default_rng(5)
    for _ in range(60):
        nd = int(rng.integers(1, 5))
        shape = [int(v) for v in rng.integers(1, 8, size=nd)]
        md = int(rng.integers(1, 4))
        mesh = [int(v) for v in rng.integers(1, 5, size=md)]
        pl = [("S", int(rng.integers(0, nd))) if rng.random() < 0.7 else ("R",) for _ in range(md)]
        coord = [int(rng.integers(0, p)) for p in mesh]
        lists = [oracle.index_list(shape, mesh, pl, coord, d) for d in range(nd)]
        glob = np.arange(int(np.prod(shape)), dtype=np.uint64).reshape(shape)
        want = glob[np.ix_(*lists)]
        got = oracle.global_indices(shape, mesh, pl, coord)
        assert np.array_equal(got, want)


SHAPES = [[1], [7], [12], [2, 6], [6, 4], [5, 3], [3, 4, 2], [4, 6, 3], [2, 3, 2, 4], [1, 6, 1, 3], [6, 2, 2, 2, 3]]
MESHES = [[1], [2], [3], [4], [2, 2], [2, 3], [3, 2], [4, 2], [2, 2, 2]]


def _valid(shape, mesh, pls):
    # InterleavedShard needs its group count to divide the (already cut) dimension.
    try:
        for c in mesh_coords(mesh):
            oracle.local_shape(shape, mesh, list(pls), list(c))
        return True
    except oracle.OracleError:
        return False


def test_merge_invariant_brute_force():
    """Section 2.3 / Section 5: merging every rank's local tensor gives exactly the
    tensor a single device generates.  Raw draws, every mesh and placement."""
    seed, offset = 0xC0FFEE12345, 64
    checked = 0
    for shape in SHAPES:
        numel = int(np.prod(shape))
        single = np.array([oracle.draw(seed, offset + j) for j in range(numel)], dtype=np.uint32).reshape(shape)
        for mesh in MESHES:
            if len(mesh) == 3 and len(shape) > 3:
                continue
            for pls in all_placements(len(shape), len(mesh)):
                if not _valid(shape, mesh, pls):
                    continue
                shards = {c: oracle.raw_u32((shape, mesh, list(pls), list(c)), seed, offset)
                          for c in mesh_coords(mesh)}
                # Nothing is caught here: replicas that differ, or pieces that do not fit together,
                # fail the test (every valid case of this grid can be gathered by concatenation).
                merged = merge_shards(shards, mesh, pls)
                assert merged.shape == tuple(shape), (shape, mesh, pls)
                assert np.array_equal(merged, single), (shape, mesh, pls)
                checked += 1
    assert checked > 3000


def test_merge_invariant_has_teeth_against_per_rank_seed_and_offset():
    """Designs (d) and (e) of Section 5 (a different seed, or a different offset, per
    rank) must fail the same merge test: the toy example of Section 2.3."""
    shape, mesh, pls = [8], [2], [("S", 0)]
    single = np.array([oracle.draw(1, j) for j in range(8)], dtype=np.uint32)
    per_rank_seed = {(r,): np.array([oracle.draw(1 + r, i) for i in range(4)], dtype=np.uint32) for r in range(2)}
    assert not np.array_equal(merge_shards(per_rank_seed, mesh, pls), single)
    # (e): each rank starts at a rank-dependent offset but walks its local indices;
    # for a row-sharded tensor that happens to agree, for a column-sharded one it does not.
    shape2, pls2 = [4, 4], [("S", 1)]
    single2 = np.array([oracle.draw(1, j) for j in range(16)], dtype=np.uint32).reshape(4, 4)
    per_rank_off = {(r,): np.array([oracle.draw(1, 8 * r + i) for i in range(8)], dtype=np.uint32).reshape(4, 2)
                    for r in range(2)}
    assert not np.array_equal(merge_shards(per_rank_off, [2], pls2), single2)
    good = {(r,): oracle.raw_u32((shape2, [2], pls2, [r]), 1, 0) for r in range(2)}
    assert np.array_equal(merge_shards(good, [2], pls2), single2)


def test_merge_refuses_replicas_that_differ_and_pieces_that_do_not_fit():
    """The merge used by the invariant tests must itself fail on what the invariant forbids."""
    good = {(r,): oracle.raw_u32(([6], [2], [("R",)], [r]), 1, 0) for r in range(2)}
    assert np.array_equal(merge_shards(good, [2], [("R",)]), good[(0,)])
    bad = dict(good)
    bad[(1,)] = bad[(1,)].copy()
    bad[(1,)][3] ^= 1
    with pytest.raises(AssertionError, match="replicas differ"):
        merge_shards(bad, [2], [("R",)])
    with pytest.raises(NotGatherable):
        merge_shards({(0,): np.arange(3), (1,): np.arange(3)}, [2], [("IS", 0, 2)])


def test_values_do_not_depend_on_the_sharding():
    # Each element is fixed by seed, offset and global index alone (Section 5).
    shape = [6, 8]
    base = oracle.raw_u32((shape, [1], [("R",)], [0]), 3, 4)
    for mesh, pls in (([2], [("S", 0)]), ([4], [("S", 1)]), ([2, 2], [("S", 1), ("S", 1)]), ([3], [("IS", 0, 2)])):
        for c in mesh_coords(mesh):
            j = oracle.global_indices(shape, mesh, pls, list(c))
            local = oracle.raw_u32((shape, mesh, pls, list(c)), 3, 4)
            assert np.array_equal(local, base.reshape(-1)[j.astype(np.int64)])
    assert not np.array_equal(oracle.raw_u32((shape, [1], [("R",)], [0]), 4, 4), base)
    assert not np.array_equal(oracle.raw_u32((shape, [1], [("R",)], [0]), 3, 8), base)


def test_offset_additivity_and_progression():
    # G(seed, offset + 4k, j) == G(seed, offset, j + 4k): a later call continues the stream.
    sh = lambda n: ([n], [1], [("R",)], [0])
    a = oracle.raw_u32(sh(64), 7, 0)
    b = oracle.raw_u32(sh(32), 7, 32)
    assert np.array_equal(a[32:], b)
    n1 = oracle.normal_f64_values(sh(64), 0.0, 1.0, 7, 0)
    n2 = oracle.normal_f64_values(sh(32), 0.0, 1.0, 7, 32)
    assert np.array_equal(n1[32:], n2)
    assert oracle.advance_offset([4096, 4096], 0) == 16777216
    assert oracle.advance_offset([5], 8) == 16
    assert oracle.advance_offset([8], 8) == 16
    assert oracle.advance_offset([3, 3], 0) == 12
    assert oracle.advance_offset([], 4) == 8
    assert oracle.advance_offset([0, 9], 4) == 4


def test_global_stride_changes_only_the_index_map():
    j = oracle.global_indices([3, 4], [1], [("R",)], [0], global_stride=[1, 3])
    assert np.array_equal(j, (np.arange(3)[:, None] + 3 * np.arange(4)[None, :]).astype(np.uint64))


def test_offset_advance_under_a_global_stride_hand_worked():
    """Section 5, design (f): every rank steps to the next global offset.  Under a non-contiguous
    global view the operator reaches stream positions up to the LAST global flat index, so the
    step is that index + 1 rounded up to a whole block.  Hand-worked:
      [30,36] rows padded to 40: last index 29*40 + 35 = 1195 -> 1196 positions (1080 elements);
      [3,5] with strides [7,1]:  last index 2*7 + 4 = 18 -> 19 -> 20;
      [3,4] transposed [1,3]:    last index 2 + 9 = 11 -> 12;
      [6,10,12] strides [1,6,60]: last 5 + 54 + 660 = 719 -> 720;
      [2,3] strides [100,7]:     last 100 + 14 = 114 -> 115 -> 116 (6 elements);
      the last one with 5 virtual threads: ceil(115 / 5) = 23 steps -> 24."""
    assert oracle.advance_offset([30, 36], 0, [40, 1]) == 1196
    assert oracle.advance_offset([30, 36], 64, [40, 1]) == 64 + 1196
    assert oracle.advance_offset([3, 5], 8, [7, 1]) == 8 + 20
    assert oracle.advance_offset([3, 4], 0, [1, 3]) == 12
    assert oracle.advance_offset([6, 10, 12], 4, [1, 6, 60]) == 4 + 720
    assert oracle.advance_offset([2, 3], 0, [100, 7]) == 116
    assert oracle.advance_offset([2, 3], 0, [100, 7], 5) == 24
    assert oracle.advance_offset([0, 3], 8, [100, 7]) == 8          # empty tensor: nothing consumed
    # The invariant the rule exists for: the next operator's positions start beyond every position
    # this one used, on every rank, and the step does not depend on the sharding.
    rng = np.random.default_rng(12)
    for _ in range(200):
        nd = int(rng.integers(1, 4))
        shape = [int(v) for v in rng.integers(1, 7, size=nd)]
        order = list(rng.permutation(nd))
        stride, acc = [0] * nd, 1
        for d in order:
            stride[d] = acc
            acc *= shape[d] + int(rng.integers(0, 3))
        off = 4 * int(rng.integers(0, 100))
        nxt = oracle.advance_offset(shape, off, stride)
        j = oracle.global_indices(shape, [1], [("R",)], [0], global_stride=stride)
        assert nxt % 4 == 0 and off + int(j.max()) < nxt <= off + int(j.max()) + 4


def test_randint_hand_worked_values():
    """Integers worked by hand from the golden generator words (tests/golden/worked_randint.txt)."""
    rows = _lines("worked_randint.txt")
    assert len(rows) >= 40
    for row in rows:
        lhs, rhs = row.split("->")
        seed, offset, j, low, high = [int(t) for t in lhs.split()]
        got = oracle.randint(([j + 1], [1], [("R",)], [0]), low, high, seed, offset, i_begin=j)
        assert int(got[j]) == int(rhs), row


def test_invalid_descriptions_are_rejected():
    with pytest.raises(oracle.OracleError):
        oracle.local_shape([4], [2], [("P",)], [0])
    with pytest.raises(oracle.OracleError):
        oracle.local_shape([4], [2], [("S", 1)], [0])
    with pytest.raises(oracle.OracleError):
        oracle.local_shape([4], [2], [("S", 0)], [2])
    with pytest.raises(oracle.OracleError):
        oracle.local_shape([6], [2], [("IS", 0, 4)], [0])
    with pytest.raises(oracle.OracleError):
        oracle.local_shape([6], [0], [("S", 0)], [0])


# ---------------------------------------------------------- conversions -------
def _f32_bits(v):
    return struct.unpack("<I", struct.pack("<f", v))[0]


def test_uniform_closed_forms():
    assert oracle.uniform_f32(0) == 0.0
    assert _f32_bits(oracle.uniform_f32(0xFFFFFFFF)) == 0x3F7FFFFF
    assert oracle.uniform_f32(0x80000000) == 0.5
    assert oracle.uniform_f32(0x000000FF) == 0.0          # low 8 bits are not used
    assert oracle.uniform_f32(0x00000100) == 2.0 ** -24
    for x in (0, 1 << 8, 12345 << 8, 0xFFFFFFFF):
        assert Fraction(oracle.uniform_f32(x)) == Fraction(x >> 8, 2 ** 24)
    # [low, high): stays inside, monotone in the draw, hits low exactly.
    assert oracle.uniform_f32(0, -3.0, 5.0) == -3.0
    prev = -math.inf
    for x in range(0, 2 ** 32, 2 ** 32 // 257):
        v = oracle.uniform_f32(x, -3.0, 5.0)
        assert -3.0 <= v < 5.0 and v >= prev
        prev = v
    # The top draw would round to high: it is pulled just below.
    top = oracle.uniform_f32(0xFFFFFFFF, 0.0, 3.0)
    assert top < 3.0 and top == float(np.nextafter(np.float32(3.0), np.float32(0.0)))
    # bfloat16: never reaches high either.
    assert oracle.uniform_bf16(0xFFFFFFFF) == 0x3F7F
    assert oracle.uniform_bf16(0) == 0
    assert oracle.float_from_bf16(oracle.uniform_bf16(0xFFFFFFFF, -1.0, 1.0)) < 1.0


def test_bf16_rounding_matches_torch_and_exact_arithmetic():
    rng = np.random.default_rng(11)
    bits = rng.integers(0, 2 ** 32, size=20000, dtype=np.uint64).astype(np.uint32)
    special = np.array([0, 0x80000000, 0x3F800000, 0x3F808000, 0x3F818000, 0x3F808001, 0x3F807FFF,
                        0x7F7FFFFF, 0x7F800000, 0xFF800000, 0x00000001, 0x00008000, 0x00018000,
                        0x007FFFFF, 0x3F7FFFFF, 0x3EFFFFFF], dtype=np.uint32)
    bits = np.concatenate([bits, special])
    f = bits.view(np.float32)
    t = torch.from_numpy(f.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    for v, want in zip(f, t):
        if np.isnan(v):
            assert oracle.float_from_bf16(oracle.bf16_from_float(float(v))) != oracle.float_from_bf16(oracle.bf16_from_float(float(v)))
            continue
        assert oracle.bf16_from_float(float(v)) == int(want), hex(_f32_bits(float(v)))
    # From double: a single rounding, checked with exact rationals (ties to even).
    for d in (1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -40, 1.0 + 2.0 ** -8 - 2.0 ** -40,
              0.02 * 1.2345, -3.75e-3, 1e-40, 3.0e38, -1.0 - 2.0 ** -9):
        h = oracle.bf16_from_double(d)
        got = Fraction(oracle.float_from_bf16(h))
        lo = Fraction(oracle.float_from_bf16((h - 1) & 0xFFFF)) if h & 0x7FFF else None
        hi = Fraction(oracle.float_from_bf16((h + 1) & 0xFFFF))
        err = abs(Fraction(d) - got)
        for other in (lo, hi):
            if other is None or math.isinf(float(other)):
                continue
            e2 = abs(Fraction(d) - other)
            assert err < e2 or (err == e2 and h % 2 == 0)
    assert oracle.bf16_from_double(6.0e38) == 0x7F80 and oracle.bf16_from_double(-3.39e38) == 0xFF7F
    assert oracle.bf16_from_double(1.0 + 2.0 ** -8) == 0x3F80       # tie -> even
    assert oracle.bf16_from_double(1.0 + 3 * 2.0 ** -8) == 0x3F82   # tie -> even
    assert oracle.bf16_from_double(1.0 + 2.0 ** -8 + 2.0 ** -40) == 0x3F81


def test_normal_closed_forms():
    r0 = math.sqrt(48 * math.log(2))                                  # u1 = 2^-24
    assert abs(oracle.normal_f64(0, 0, False) - r0) < 1e-14
    assert abs(r0 - 5.768107546) < 1e-8
    assert oracle.normal_f64(0, 0, True) == 0.0
    assert oracle.normal_f64(0xFFFFFFFF, 0x12345678, False) == 0.0    # u1 = 1 -> radius 0
    assert oracle.normal_f64(0xFFFFFFFF, 0x12345678, True) == 0.0
    assert abs(oracle.normal_f64(0, 0x40000000, False)) < 1e-15       # cos(pi/2)
    assert abs(oracle.normal_f64(0, 0x40000000, True) - r0) < 1e-14   # sin(pi/2)
    assert abs(oracle.normal_f64(0, 0x80000000, False) + r0) < 1e-14  # cos(pi)
    assert abs(oracle.normal_f64(5 << 8, 0, False, 2.0, 0.5) - (2.0 + 0.5 * math.sqrt(-2 * math.log(6 / 2 ** 24)))) < 1e-14
    # Pair identities: n_even^2 + n_odd^2 = -2 ln u1 and the angle is 2 pi u2.
    rng = np.random.default_rng(3)
    for xa, xb in rng.integers(0, 2 ** 32, size=(500, 2)):
        xa, xb = int(xa), int(xb)
        c, s = oracle.normal_f64(xa, xb, False), oracle.normal_f64(xa, xb, True)
        u1, u2 = ((xa >> 8) + 1) / 2 ** 24, (xb >> 8) / 2 ** 24
        assert abs(c * c + s * s + 2 * math.log(u1)) < 1e-12
        if c * c + s * s > 1e-6:
            assert abs((math.atan2(s, c) / (2 * math.pi)) % 1.0 - u2) < 1e-9


def test_normal_pairs_follow_the_block_layout():
    # Positions p and p^1 share the draw pair (words 0,1 or 2,3 of block p // 4).
    seed, off = 21, 12
    vals = oracle.normal_f64_values(([16], [1], [("R",)], [0]), 0.0, 1.0, seed, off)
    for j in range(16):
        p = off + j
        xa, xb = oracle.draw(seed, p - p % 2), oracle.draw(seed, p - p % 2 + 1)
        assert vals[j] == oracle.normal_f64(xa, xb, p % 2 == 1)
    f32 = oracle.normal(([16], [1], [("R",)], [0]), oracle.F32, 0.0, 1.0, seed, off)
    assert np.array_equal(f32, vals.astype(np.float32))
    b16 = oracle.normal(([16], [1], [("R",)], [0]), oracle.BF16, 1.0, 0.02, seed, off)
    v2 = oracle.normal_f64_values(([16], [1], [("R",)], [0]), 1.0, 0.02, seed, off)
    assert list(b16) == [oracle.bf16_from_double(float(v)) for v in v2]


def test_dropout_closed_forms():
    assert oracle.dropout_threshold(0.1) == 0xE66666
    assert _f32_bits(oracle.dropout_scale(0.1)) == 0x3F8E38E4
    assert oracle.dropout_threshold(0.0) == 2 ** 24 and oracle.dropout_scale(0.0) == 1.0
    assert oracle.dropout_threshold(1.0) == 0
    assert oracle.dropout_threshold(0.5) == 2 ** 23 and oracle.dropout_scale(0.5) == 2.0
    sh = ([4, 8], [2], [("S", 1)], [1])
    x = np.array([1.5, -2.0, 0.0, -0.0, np.inf, -np.inf, np.nan, 1e-39, 3.0, 4.0, 5.0, 6.0, 7.0, 8.0, 9.0, 10.0],
                 dtype=np.float32)
    y, m = oracle.dropout(sh, oracle.F32, 0.0, 5, 0, x)
    assert np.array_equal(y.view(np.uint32).reshape(-1), x.view(np.uint32)) and m.all()     # p = 0: identity
    y, m = oracle.dropout(sh, oracle.F32, 1.0, 5, 0, x)
    assert not y.view(np.uint32).any() and not m.any()                                        # p = 1: +0 everywhere
    # General p: mask is the integer test on the draw; kept = x * scale in fp32; dropped = +0.
    y, m = oracle.dropout(sh, oracle.F32, 0.4, 5, 0, x)
    j = oracle.global_indices(*sh).reshape(-1)
    keep = np.array([(oracle.draw(5, int(v)) >> 8) < oracle.dropout_threshold(0.4) for v in j])
    assert np.array_equal(m.reshape(-1).astype(bool), keep) and keep.any() and not keep.all()
    want = np.where(keep, x * np.float32(oracle.dropout_scale(0.4)), np.float32(0.0))
    yy = y.reshape(-1)
    for a, b, k in zip(yy, want, keep):
        assert (np.isnan(a) and np.isnan(b)) or _f32_bits(float(a)) == _f32_bits(float(b))
        if not k:
            assert _f32_bits(float(a)) == 0
    # bfloat16: the product is rounded to fp32, then to bfloat16 - the same as torch's own ops.
    rng = np.random.default_rng(8)
    xb = torch.from_numpy(rng.standard_normal(32).astype(np.float32)).to(torch.bfloat16)
    y, m = oracle.dropout(sh if False else ([32], [1], [("R",)], [0]), oracle.BF16, 0.1, 9, 4,
                          xb.view(torch.int16).numpy().view(np.uint16))
    ref = (xb.float() * oracle.dropout_scale(0.1)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(y, np.where(m.astype(bool), ref, 0))


# ---------------------------------------------------------- statistics --------
def test_statistics_of_the_three_distributions():
    from scipy import stats
    n = 1 << 18
    sh = ([n], [1], [("R",)], [0])
    u = oracle.uniform(sh, oracle.F32, 0.0, 1.0, 1234, 0, threads=4).astype(np.float64)
    assert abs(u.mean() - 0.5) < 4 / math.sqrt(12 * n)
    assert stats.kstest(u, "uniform").pvalue > 1e-4
    z = oracle.normal_f64_values(sh, 0.0, 1.0, 7, 0, threads=4)
    assert abs(z.mean()) < 4 / math.sqrt(n)
    assert abs(z.var() - 1.0) < 4 * math.sqrt(2 / n)
    assert abs(stats.kurtosis(z)) < 0.05
    assert stats.kstest(z, "norm").pvalue > 1e-4
    # Neighbouring elements (cos / sin of one pair) are uncorrelated.
    assert abs(np.corrcoef(z[0::2], z[1::2])[0, 1]) < 4 / math.sqrt(n / 2)
    x = np.ones(n, dtype=np.float32)
    _, m = oracle.dropout(sh, oracle.F32, 0.1, 1234, 0, x, threads=4)
    keep = oracle.dropout_threshold(0.1) / 2 ** 24
    assert abs(m.mean() - keep) < 4 * math.sqrt(0.09 / n)
    r = oracle.randint(sh, -3, 7, 5, 0, threads=4)
    assert r.min() == -3 and r.max() == 6
    assert stats.chisquare(np.bincount(r + 3, minlength=10)).pvalue > 1e-4
    assert list(oracle.randint(([8], [1], [("R",)], [0]), 10, 17, 5, 0)) == [10 + oracle.draw(5, i) % 7 for i in range(8)]


# ------------------------------------------------ virtual-thread layout -------
def test_virtual_thread_layout_follows_algorithm_1_to_the_letter():
    """theta > 0: virtual thread tau = j mod theta, virtual offset beta = offset + j / theta,
    generator called with (seed, tau, beta).  Checked against the big-integer generator."""
    seed = (0x1234 << 32) | 0xABCDEF01
    key = [seed % 2 ** 32, seed >> 32]
    for theta, offset, n in ((1, 0, 40), (7, 8, 100), (64, 4, 300), (1 << 40, 12, 50)):
        got = oracle.raw_u32(([n], [1], [("R",)], [0], None, theta), seed, offset)
        for j in (0, 1, 2, n // 2, n - 1):
            tau, beta = j % theta, offset + j // theta
            q = beta // 4
            want = _philox_bigint([q % 2 ** 32, q >> 32, tau % 2 ** 32, tau >> 32], key)[beta % 4]
            assert int(got[j]) == want, (theta, j)
    # theta >= numel: every element is its own virtual thread at the call's offset.
    got = oracle.raw_u32(([10], [1], [("R",)], [0], None, 1000), 5, 8)
    assert list(got) == [_philox_bigint([2, 0, j, 0], [5, 0])[0] for j in range(10)]
    # theta = 1: one thread walks the whole tensor - the flat stream again.
    a = oracle.raw_u32(([37], [1], [("R",)], [0], None, 1), 5, 8)
    b = oracle.raw_u32(([37], [1], [("R",)], [0]), 5, 8)
    assert np.array_equal(a, b)


def test_virtual_thread_layout_keeps_the_merge_invariant_and_the_offset_rule():
    seed, offset, theta = 99, 16, 5
    for shape, mesh, pls in (([6, 10], [2, 2], [("S", 0), ("S", 1)]), ([24], [3], [("IS", 0, 4)]), ([4, 9], [3], [("S", 1)])):
        single = oracle.raw_u32((shape, [1], [("R",)], [0], None, theta), seed, offset)
        shards = {c: oracle.raw_u32((shape, mesh, pls, list(c), None, theta), seed, offset) for c in mesh_coords(mesh)}
        assert np.array_equal(merge_shards(shards, mesh, pls), single)
        z = oracle.normal_f64_values((shape, [1], [("R",)], [0], None, theta), 0.0, 1.0, seed, offset).reshape(-1)
        # Elements j and j + theta sit in neighbouring words of one thread's stream: they form a
        # Box-Muller pair when the lower one's word is even.
        for j in range(z.size - theta):
            beta = offset + j // theta
            if beta % 2 == 0:
                xa = int(single.reshape(-1)[j]); xb = int(single.reshape(-1)[j + theta])
                assert z[j] == oracle.normal_f64(xa, xb, False) and z[j + theta] == oracle.normal_f64(xa, xb, True)
    # Each of theta threads steps ceil(N / theta) times; the offset moves by that, rounded up to 4.
    assert oracle.advance_offset([6, 10], 16, None, 5) == 16 + 12
    assert oracle.advance_offset([6, 10], 16, None, 60) == 16 + 4
    assert oracle.advance_offset([6, 10], 16, None, 1) == 16 + 60
    # The next call's values do not overlap this call's.
    nxt = oracle.advance_offset([6, 10], offset, None, theta)
    a = oracle.raw_u32(([6, 10], [1], [("R",)], [0], None, theta), seed, offset).reshape(-1)
    b = oracle.raw_u32(([6, 10], [1], [("R",)], [0], None, theta), seed, nxt).reshape(-1)
    assert not set(a.tolist()) & set(b.tolist())


def test_dropout_add_is_dropout_then_an_fp32_add():
    sh = ([6, 10], [2], [("S", 1)], [1])
    rng = np.random.default_rng(2)
    x = rng.standard_normal(30).astype(np.float32)
    r = rng.standard_normal(30).astype(np.float32)
    y, m = oracle.dropout_add(sh, oracle.F32, 0.3, 4, 0, x, r)
    yd, md = oracle.dropout(sh, oracle.F32, 0.3, 4, 0, x)
    assert np.array_equal(m, md)
    assert np.array_equal(y.reshape(-1), r + yd.reshape(-1))          # numpy fp32 add = one rounding
    # bfloat16: product and sum are fp32, one rounding to bfloat16 at the end - torch's own ops agree.
    xb = torch.from_numpy(x).to(torch.bfloat16)
    rb = torch.from_numpy(r).to(torch.bfloat16)
    y, m = oracle.dropout_add(sh, oracle.BF16, 0.3, 4, 0, xb.view(torch.int16).numpy().view(np.uint16),
                              rb.view(torch.int16).numpy().view(np.uint16))
    keep = torch.from_numpy(m.reshape(-1).astype(bool))
    ref = (rb.float() + torch.where(keep, xb.float() * oracle.dropout_scale(0.3), torch.zeros(30))).to(torch.bfloat16)
    assert np.array_equal(y.reshape(-1), ref.view(torch.int16).numpy().view(np.uint16))


def test_dropout_threshold_rounds_to_nearest():
    # (1 - p) 2^24 = 9227468.8 for p = 0.45: nearest is ...469 (a floor would give ...468).
    assert oracle.dropout_threshold(0.45) == 9227469
    assert oracle.dropout_threshold(0.55) == 7549747      # 7549747.2 rounds down
    assert oracle.dropout_threshold(2.0 ** -25) == 2 ** 24  # 2^24 - 0.5 rounds half up to 2^24: nothing is dropped


# ---------------------------------------------------------- binary16 ----------
def test_f16_conversions_match_numpy_on_every_pattern_and_midpoint():
    """numpy's float16 is an independent implementation of IEEE binary16: every bit pattern decodes to
    the same value, and rounding agrees on random doubles over 15 decades, on every midpoint between
    neighbouring values (ties to even), just beside the midpoints, and at the overflow boundary."""
    pats = np.arange(65536, dtype=np.uint16)
    vals = pats.view(np.float16).astype(np.float64)
    for h in range(65536):
        v = oracle.double_from_f16(h)
        assert v == vals[h] or (math.isnan(v) and math.isnan(vals[h])), hex(h)
    rng = np.random.default_rng(1)
    mids = (vals[:0x7BFF] + vals[1:0x7C00]) / 2
    xs = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-9, 6, 20000), mids, -mids,
                         mids * (1 + 2.0 ** -40), mids * (1 - 2.0 ** -40),
                         [0.0, -0.0, 65504, 65519.99, 65520, 65535, 65536, 1e9, -1e9, 2.0 ** -24, 2.0 ** -25,
                          2.0 ** -25 * 1.0000001, 2.0 ** -26, np.inf, -np.inf]])
    with np.errstate(over="ignore"):
        ref = xs.astype(np.float16).view(np.uint16)
    for x, r in zip(xs, ref):
        assert oracle.f16_from_double(float(x)) == int(r), repr(float(x))
    assert oracle.f16_from_double(float("nan")) & 0x7C00 == 0x7C00 and oracle.f16_from_double(float("nan")) & 0x3FF
    assert oracle.f16_from_double(1.0 + 2.0 ** -11) == 0x3C00        # tie -> even
    assert oracle.f16_from_double(1.0 + 3 * 2.0 ** -11) == 0x3C02    # tie -> even
    assert oracle.f16_from_double(65520.0) == 0x7C00 and oracle.f16_from_double(65519.999) == 0x7BFF


def test_f16_operators_are_the_fp32_value_rounded_once():
    """uniform: the fp32 value rounded to binary16 (numpy), pulled below `high` when the rounding reaches
    it; normal: the double value rounded once; dropout and dropout + residual: fp32 product / sum rounded
    once - all rebuilt here with numpy's float16."""
    assert oracle.uniform_f16(0) == 0 and oracle.uniform_f16(0xFFFFFFFF) == 0x3BFF   # 1 - 2^-24 rounds to 1 -> pulled
    assert oracle.uniform_f16(0x80000000) == 0x3800
    rng = np.random.default_rng(3)
    for low, high in ((0.0, 1.0), (-1.0, 1.0), (-0.03, 0.03), (2.0, 2.001), (-65504.0, 65504.0), (-3.0, 0.0)):
        lo32, hi32 = np.float32(low), np.float32(high)
        for x in list(rng.integers(0, 2 ** 32, 300)) + [0, 0xFFFFFFFF, 0xFFFFFF00, 0xFFFFFEFF]:
            got = oracle.uniform_f16(int(x), low, high)
            r32 = np.float32(oracle.uniform_f32(int(x), low, high))
            h = np.float16(r32)
            assert float(np.uint16(got).view(np.float16)) < float(hi32)
            if float(h) < float(hi32):
                assert got == int(h.view(np.uint16)), (low, high, hex(int(x)))
            else:   # pulled back: the largest binary16 below high
                below = np.nextafter(np.float16(hi32), np.float16(-np.inf)) if float(np.float16(hi32)) >= float(hi32) \
                    else np.float16(hi32)
                assert got == int(below.view(np.uint16)), (low, high, hex(int(x)))
    sh = ([6, 10], [2], [("S", 1)], [1])
    v = oracle.normal_f64_values(sh, 0.5, 3.0, 4, 8).reshape(-1)
    assert np.array_equal(oracle.normal(sh, oracle.F16, 0.5, 3.0, 4, 8).reshape(-1), v.astype(np.float16).view(np.uint16))
    with np.errstate(over="ignore"):
        big = oracle.normal(sh, oracle.F16, 0.0, 40000.0, 4, 8).reshape(-1)
        vb = oracle.normal_f64_values(sh, 0.0, 40000.0, 4, 8).reshape(-1)
        assert np.array_equal(big, vb.astype(np.float16).view(np.uint16)) and (big & 0x7FFF == 0x7C00).any()
    x = np.concatenate([rng.standard_normal(24) * 100, [0.0, -0.0, 6.0e-8, -6.0e-8, 65504.0, -65504.0]]
                       ).astype(np.float16)
    r = (rng.standard_normal(30) * 100).astype(np.float16)
    scale = np.float32(oracle.dropout_scale(0.3))
    y, m = oracle.dropout(sh, oracle.F16, 0.3, 4, 0, x.view(np.uint16))
    keep = m.reshape(-1).astype(bool)
    md = oracle.dropout(sh, oracle.F32, 0.3, 4, 0, x.astype(np.float32))[1]
    assert np.array_equal(m, md) and keep.any() and not keep.all()
    with np.errstate(over="ignore"):
        prod = x.astype(np.float32) * scale
        want = np.where(keep, prod.astype(np.float16).view(np.uint16), np.uint16(0))
        assert np.array_equal(y.reshape(-1), want)
        y2, m2 = oracle.dropout_add(sh, oracle.F16, 0.3, 4, 0, x.view(np.uint16), r.view(np.uint16))
        total = r.astype(np.float32) + np.where(keep, prod, np.float32(0))
        assert np.array_equal(m2, m) and np.array_equal(y2.reshape(-1), total.astype(np.float16).view(np.uint16))
