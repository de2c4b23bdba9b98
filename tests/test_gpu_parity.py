"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs, element by element.  Bars: raw draws, uniforms, dropout outputs and masks and
integers are bit-exact; fp32 normals within 1e-6 * max(|ref|, std) of the double-precision
definition; bf16 / fp16 normals within one ulp of the 16-bit type (neighbouring value)."""
import itertools
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2509_07003_amd as v
from helpers import merge_shards, mesh_coords
from paper_2509_07003_amd import workloads as W

pytestmark = pytest.mark.gpu
THREADS = min(16, os.cpu_count() or 1)
DEV = "cuda"


def say(msg):
    print(msg, flush=True)


# dtype name -> (torch dtype, library code, oracle code)
DT = {"f32": (torch.float32, v.F32, oracle.F32), "bf16": (torch.bfloat16, v.BF16, oracle.BF16),
      "f16": (torch.float16, v.F16, oracle.F16)}


def to_device(a, dtype):
    """numpy float32 array, or uint16 bit patterns of a 16-bit dtype -> device tensor of that dtype."""
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32).reshape(-1)).to(DEV)
    return torch.from_numpy(np.ascontiguousarray(a).reshape(-1).view(np.int16)).to(DEV).view(DT[dtype][0])


def to_host(t, dtype):
    return t.cpu().numpy() if dtype == "f32" else t.view(torch.int16).cpu().numpy().view(np.uint16)


# ------------------------------------------------------------------ helpers ----
def gpu_fill(op, dtype, sharding_args, seed, offset, **params):
    """Runs one fill through the C ABI; returns a numpy array of the local shard
    (uint32 raw, float32, uint16 bf16 bits or int64)."""
    sh = v.Sharding(*sharding_args)
    shape, n = v.vesrng_local_shape(sh)
    if op == "raw":
        out = torch.empty(max(n, 1), dtype=torch.int32, device=DEV)
        v.vesrng_raw_u32(sh, seed, offset, out)
        res = out.cpu().numpy().view(np.uint32)
    elif op == "randint":
        out = torch.empty(max(n, 1), dtype=torch.int64, device=DEV)
        v.vesrng_randint(sh, params["low"], params["high"], seed, offset, out)
        res = out.cpu().numpy()
    else:
        out = torch.empty(max(n, 1), dtype=DT[dtype][0], device=DEV)
        code = DT[dtype][1]
        if op == "uniform":
            v.vesrng_uniform(sh, code, params.get("low", 0.0), params.get("high", 1.0), seed, offset, out)
        else:
            v.vesrng_normal(sh, code, params.get("mean", 0.0), params.get("std", 1.0), seed, offset, out)
        res = to_host(out, dtype)
    torch.cuda.synchronize()
    return res[:n].reshape(shape)


def gpu_dropout(dtype, sharding_args, p, seed, offset, x_np, with_mask=True, in_place=False):
    sh = v.Sharding(*sharding_args)
    shape, n = v.vesrng_local_shape(sh)
    x = to_device(x_np, dtype)
    y = x if in_place else torch.empty_like(x)
    mask = torch.full((max(n, 1),), 7, dtype=torch.uint8, device=DEV) if with_mask else None
    v.vesrng_dropout(sh, DT[dtype][1], p, seed, offset, x, y, mask)
    torch.cuda.synchronize()
    yn = to_host(y, dtype)
    return yn[:n].reshape(shape), (mask.cpu().numpy()[:n].reshape(shape) if with_mask else None)


def bf16_ordinal(bits):
    """Monotone integer code of the bit patterns of a 16-bit float, bfloat16 or binary16: both are
    sign-magnitude (+0 and -0 coincide)."""
    b = bits.astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)


def assert_float_bits_equal(got, want, what, dtype="bf16"):
    """Bit-exact, except that any NaN matches any NaN (payloads are unspecified).  `dtype` names the
    16-bit format when the arrays hold uint16 patterns."""
    if got.dtype == np.float32:
        g, w = got.view(np.uint32), want.view(np.uint32)
        nan_g, nan_w = np.isnan(got), np.isnan(want)
    else:
        g, w = got, want
        expo, frac = (0x7C00, 0x03FF) if dtype == "f16" else (0x7F80, 0x007F)
        nan_g = ((got & expo) == expo) & ((got & frac) != 0)
        nan_w = ((want & expo) == expo) & ((want & frac) != 0)
    assert np.array_equal(nan_g, nan_w), what + ": NaN positions differ"
    bad = (g != w) & ~nan_g
    assert not bad.any(), "%s: %d mismatches, first at %s" % (what, bad.sum(), np.argwhere(bad)[:3].tolist())


def check_normal(got, sharding_args, dtype, mean, std, seed, offset, what, i_begin=0, i_end=-1):
    ref = oracle.normal_f64_values(tuple(sharding_args), mean, std, seed, offset, i_begin=i_begin,
                                   i_end=i_end, threads=THREADS).reshape(-1)
    g = got.reshape(-1)
    sl = slice(i_begin, None if i_end < 0 else i_end)
    ref, g = ref[sl], g[sl]
    if dtype == "f32":
        err = np.abs(g.astype(np.float64) - ref)
        tol = 1e-6 * np.maximum(np.abs(ref), std)
        worst = float((err / tol).max()) if err.size else 0.0
        assert worst <= 1.0, "%s: error is %.3f of the tolerance" % (what, worst)
        return worst
    # 16-bit outputs: the kernel rounds an fp32 value that lies within the fp32 tolerance of the
    # reference, so - rounding being monotone - its result must lie between the roundings of
    # ref - tol and ref + tol.  Where the format's spacing exceeds 2 tol (|ref| > 2^(bits + 2) tol
    # for `bits` fraction bits) that is the reference value or its neighbour: one ulp; closer to
    # zero the interval spans a few of the ever finer steps, and the other sign of a vanishing value.
    tol = 1e-6 * np.maximum(np.abs(ref), std)
    lo = bf16_ordinal(_bits16(ref - tol, dtype))
    hi = bf16_ordinal(_bits16(ref + tol, dtype))
    go = bf16_ordinal(g)
    bad = (go < lo) | (go > hi)
    assert not bad.any(), "%s: %d values outside the rounding interval, first %s" % (what, bad.sum(), np.argwhere(bad)[:3].tolist())
    assert (hi - lo)[np.abs(ref) > (2.0 ** 12 if dtype == "f16" else 2.0 ** 9) * tol].max(initial=0) <= 1
    want = oracle.normal(tuple(sharding_args), DT[dtype][2], mean, std, seed, offset, i_begin=i_begin,
                         i_end=i_end, threads=THREADS).reshape(-1)[sl]
    return float((g != want).mean()) if g.size else 0.0


def _bits16(a64, dtype):
    """float64 -> the 16-bit dtype, one rounding, by a library (torch for bfloat16, numpy for binary16)."""
    if dtype == "f16":
        with np.errstate(over="ignore"):
            return np.ascontiguousarray(a64).astype(np.float16).view(np.uint16)
    t = torch.from_numpy(np.ascontiguousarray(a64)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


# ------------------------------------------------------------- the configs ----
def test_c1_uniform_f32_row_shards_bit_exact():
    w = W.C1
    shards = {}
    for c in mesh_coords(w.mesh_shape):
        say("C1 rank %s" % (c,))
        args = w.sharding_args(c)
        got = gpu_fill("uniform", "f32", args, w.seed, 0)
        want = oracle.uniform(tuple(args), oracle.F32, 0.0, 1.0, w.seed, 0, threads=THREADS)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
        raw = gpu_fill("raw", None, args, w.seed, 0)
        assert np.array_equal(raw, oracle.raw_u32(tuple(args), w.seed, 0, threads=THREADS))
        shards[c] = got
    single = gpu_fill("uniform", "f32", (w.global_shape, [1], [("R",)], [0]), w.seed, 0)
    assert np.array_equal(merge_shards(shards, w.mesh_shape, w.placements), single)
    # The first worked values of this configuration (see tests/golden/worked_values.txt).
    assert single.reshape(-1)[0] == np.float32(0.1272079348564148)
    assert shards[(1,)].reshape(-1)[0] == np.float32(0.630875825881958)


def test_c2_normal_f32_ragged_column_shards_and_offset_progression():
    w = W.C2
    sh_any = v.Sharding(*w.sharding_args([0]))
    off2 = v.vesrng_advance_offset(sh_any, 0)
    assert off2 == 4096 * 4096
    for call, off in enumerate((0, off2)):
        shards = {}
        for c in mesh_coords(w.mesh_shape):
            say("C2 call %d rank %s" % (call, c))
            args = w.sharding_args(c)
            got = gpu_fill("normal", "f32", args, w.seed, off)
            worst = check_normal(got, args, "f32", 0.0, 1.0, w.seed, off, "C2 call %d rank %s" % (call, c))
            say("  worst error / tolerance = %.3f" % worst)
            raw = gpu_fill("raw", None, args, w.seed, off)
            assert np.array_equal(raw, oracle.raw_u32(tuple(args), w.seed, off, threads=THREADS))
            shards[c] = got
        assert [s.shape[1] for s in shards.values()] == [1366, 1366, 1364]
        single = gpu_fill("normal", "f32", (w.global_shape, [1], [("R",)], [0]), w.seed, off)
        merged = merge_shards(shards, w.mesh_shape, w.placements)
        assert np.array_equal(merged.view(np.uint32), single.view(np.uint32))   # bit-wise on the GPU itself
        if call == 1:
            # Second call == elements [2^24, 2^25) of a 1-D stream of 2^25 elements at offset 0.
            both = gpu_fill("normal", "f32", ([2 * off2], [1], [("R",)], [0]), w.seed, 0)
            assert np.array_equal(both[off2:].view(np.uint32), single.reshape(-1).view(np.uint32))
            assert not np.array_equal(both[:off2].view(np.uint32), single.reshape(-1).view(np.uint32))


def test_c3_normal_bf16_weight_init_2d_mesh():
    w = W.C3
    shards = {}
    for c in mesh_coords(w.mesh_shape):
        say("C3 rank %s" % (c,))
        args = w.sharding_args(c)
        got = gpu_fill("normal", "bf16", args, w.seed, 0, mean=0.0, std=0.02)
        assert got.shape == (2048, 3584)
        frac = check_normal(got, args, "bf16", 0.0, 0.02, w.seed, 0, "C3 rank %s" % (c,))
        say("  fraction not equal to the rounded reference = %.2e" % frac)
        shards[c] = got
    single = gpu_fill("normal", "bf16", (w.global_shape, [1], [("R",)], [0]), w.seed, 0, mean=0.0, std=0.02)
    assert np.array_equal(merge_shards(shards, w.mesh_shape, w.placements), single)
    vals = torch.from_numpy(single.view(np.int16)).view(torch.bfloat16).float()
    assert abs(float(vals.mean())) < 1e-4 and abs(float(vals.std()) - 0.02) < 2e-4


def test_c4_dropout_bf16_sequence_sharded():
    w = W.C4
    for c in mesh_coords(w.mesh_shape):
        say("C4 rank %s" % (c,))
        args = w.sharding_args(c)
        x = W.host_activations([8, 512, 4096], w.input_seed + c[0], "normal", "bf16")
        y, m = gpu_dropout("bf16", args, 0.1, w.seed, 0, x)
        yo, mo = oracle.dropout(tuple(args), oracle.BF16, 0.1, w.seed, 0, x, threads=THREADS)
        assert np.array_equal(m, mo)
        assert_float_bits_equal(y, yo, "C4 rank %s" % (c,))
        assert abs(m.mean() - 0.9) < 1e-3


def _c5_check(w, coord):
    args = w.sharding_args(coord)
    shape, n = v.vesrng_local_shape(v.Sharding(*args))
    assert shape == [8, 4, 4096, 4096]
    say("%s: making input on the device" % w.name)
    x = W.device_activations(shape, w.input_seed, "softmax", "bf16").reshape(-1)
    y = torch.empty_like(x)
    mask = torch.empty(n, dtype=torch.uint8, device=DEV)
    say("  launching")
    v.vesrng_dropout(v.Sharding(*args), v.BF16, 0.1, w.seed, 0, x, y, mask)
    torch.cuda.synchronize()
    xh = x.view(torch.int16).cpu().numpy().view(np.uint16)
    yh = y.view(torch.int16).cpu().numpy().view(np.uint16)
    mh = mask.cpu().numpy()
    # Whole-shard properties, then element-by-element parity over the WHOLE shard (the threaded
    # oracle does 2^29 elements in about a second).
    assert abs(mh.mean() - 0.899999976) < 5.2e-5
    assert not yh[mh == 0].any()
    say("  oracle on all %d elements" % n)
    yo, mo = oracle.dropout(tuple(args), oracle.BF16, 0.1, w.seed, 0, xh, threads=THREADS)
    assert np.array_equal(mh, mo.reshape(-1))
    del mo
    assert_float_bits_equal(yh, yo.reshape(-1), w.name)


def test_c5_dropout_bf16_attention_probabilities_nested_shard_full_size():
    _c5_check(W.C5, W.C5.bench_coord)


def test_c5_dropout_bf16_interleaved_reading_full_size():
    _c5_check(W.C5_INTERLEAVED, W.C5_INTERLEAVED.bench_coord)


# ------------------------------------------------- scaled operator matrix -----
GRID_SHAPES = {1: [100003], 2: [301, 333], 3: [37, 53, 51], 4: [11, 13, 14, 50], 5: [7, 6, 9, 10, 22]}


def _grid_cases():
    for nd, shape in GRID_SHAPES.items():
        for d in range(nd):
            yield shape, [3], [("S", d)]
        for a, b in itertools.product(range(nd), repeat=2):
            yield shape, [2, 3], [("S", a), ("S", b)]


@pytest.mark.parametrize("op,dtype", [("raw", None), ("uniform", "f32"), ("uniform", "bf16"), ("normal", "f32"),
                                       ("normal", "bf16"), ("dropout", "f32"), ("dropout", "bf16"),
                                       ("randint", None), ("uniform", "f16"), ("normal", "f16"), ("dropout", "f16")])
def test_operator_matrix_1d_to_5d_single_and_double_sharding(op, dtype):
    """Scaled version of the paper's per-operator table: every operator, 1-D to 5-D tensors,
    sharding on every dimension and every ordered pair of dimensions, odd extents."""
    seed, offset = 0x5EED0001CAFE, 1 << 34    # exercises both key words and the high counter word
    count = 0
    for shape, mesh, pls in _grid_cases():
        for c in mesh_coords(mesh):
            args = (shape, mesh, pls, list(c))
            what = "%s %s %s %s %s" % (op, dtype, shape, pls, c)
            say(what)
            targs = tuple(args)
            if op == "raw":
                assert np.array_equal(gpu_fill("raw", None, args, seed, offset), oracle.raw_u32(targs, seed, offset)), what
            elif op == "randint":
                got = gpu_fill("randint", None, args, seed, offset, low=-5, high=1000003)
                assert np.array_equal(got, oracle.randint(targs, -5, 1000003, seed, offset)), what
            elif op == "uniform":
                got = gpu_fill("uniform", dtype, args, seed, offset, low=-2.5, high=7.25)
                want = oracle.uniform(targs, DT[dtype][2], -2.5, 7.25, seed, offset)
                assert_float_bits_equal(got, want, what, dtype=dtype)
            elif op == "normal":
                got = gpu_fill("normal", dtype, args, seed, offset, mean=1.5, std=0.25)
                check_normal(got, args, dtype, 1.5, 0.25, seed, offset, what)
            else:
                n = oracle.local_shape(*args)[1]
                xf = W.adversarial_f32(n, seed=count)
                x = xf if dtype == "f32" else W.bits16_from_f32(xf, dtype)
                y, m = gpu_dropout(dtype, args, 0.3, seed, offset, x)
                yo, mo = oracle.dropout(targs, DT[dtype][2], 0.3, seed, offset, x)
                assert np.array_equal(m, mo), what
                assert_float_bits_equal(y, yo, what, dtype=dtype)
            count += 1
    assert count > 300


def test_gpu_shards_merge_to_the_gpu_single_device_tensor_bitwise():
    """The paper's invariant on the product itself, including normals (bit-wise)."""
    seed, offset = 99, 8
    for shape, mesh, pls in [([129, 131], [2, 2], [("S", 0), ("S", 1)]), ([64, 66], [4], [("S", 1)]),
                             ([12, 40, 9], [2, 3], [("S", 1), ("S", 1)]), ([6, 32, 10], [8], [("IS", 1, 4)]),
                             ([48, 10], [2, 2], [("IS", 0, 4), ("R",)])]:
        for op, dtype in (("normal", "f32"), ("normal", "bf16"), ("uniform", "bf16"), ("raw", None)):
            shards = {c: gpu_fill(op, dtype, (shape, mesh, pls, list(c)), seed, offset) for c in mesh_coords(mesh)}
            single = gpu_fill(op, dtype, (shape, [1], [("R",)], [0]), seed, offset)
            merged = merge_shards(shards, mesh, pls)
            assert merged.tobytes() == single.tobytes(), (shape, mesh, pls, op, dtype)


# ------------------------------------------------------------ edge cases ------
def test_tiny_empty_and_zero_dim_tensors():
    for n in list(range(0, 10)) + [15, 16, 17, 31, 33]:
        args = ([n], [1], [("R",)], [0])
        assert np.array_equal(gpu_fill("raw", None, args, 5, 4), oracle.raw_u32(args, 5, 4))
        got = gpu_fill("uniform", "bf16", args, 5, 4)
        assert np.array_equal(got, oracle.uniform(args, oracle.BF16, 0.0, 1.0, 5, 4))
    # More ranks than rows: ranks 2 and 3 of 4 hold nothing of 2 rows.
    for r in range(4):
        args = ([2, 5], [4], [("S", 0)], [r])
        got = gpu_fill("uniform", "f32", args, 5, 0)
        assert np.array_equal(got, oracle.uniform(args, oracle.F32, 0.0, 1.0, 5, 0))
        assert got.size == (5 if r < 2 else 0)
    zero_d = ([], [2], [("R",)], [1])
    assert np.array_equal(gpu_fill("raw", None, zero_d, 5, 0), oracle.raw_u32(zero_d, 5, 0))
    # Unsharded dimension of extent 1 and a column shard one element wide.
    for args in (([5, 1, 7], [2], [("S", 2)], [1]), ([64, 3], [3], [("S", 1)], [2])):
        assert np.array_equal(gpu_fill("raw", None, args, 5, 0), oracle.raw_u32(args, 5, 0))


def test_uniform_bounds_and_upper_guard():
    n = 1 << 16
    args = ([n], [1], [("R",)], [0])
    for dtype, code in (("f32", oracle.F32), ("bf16", oracle.BF16), ("f16", oracle.F16)):
        for low, high in ((0.0, 1.0), (-1.0, 1.0), (0.0, 3.0), (5.0, 5.0), (-0.02, 0.02), (1e-3, 1.0 + 1e-3),
                          (-3.0, 0.0), (2.0005, 2.001), (-1e-6, 1e-6), (0.1, 0.1), (-7.0, -6.99), (1.0, 1.0 + 2.0 ** -20)):
            got = gpu_fill("uniform", dtype, args, 77, 0, low=low, high=high)
            want = oracle.uniform(args, code, low, high, 77, 0)
            assert_float_bits_equal(got, want, "uniform %s [%g,%g)" % (dtype, low, high), dtype=dtype)
            vals = got if dtype == "f32" else torch.from_numpy(got.view(np.int16)).view(DT[dtype][0]).float().numpy()
            # A 16-bit dtype cannot represent every low: the bound below is low rounded to the dtype.
            floor = np.float32(low) if dtype == "f32" else torch.tensor(low, dtype=torch.float32).to(DT[dtype][0]).float().numpy()
            # ... nor every value below high when the range is narrower than its spacing.
            narrow = dtype != "f32" and high - low < 0.01
            assert vals.min() >= floor and (vals.max() < np.float32(high) or low == high or narrow)


def test_dropout_degenerate_probabilities_special_values_in_place_and_no_mask():
    n = 4096 + 5
    args = ([n], [1], [("R",)], [0])
    xf = W.adversarial_f32(n, 4)
    for dtype, code in (("f32", oracle.F32), ("bf16", oracle.BF16)):
        x = xf if dtype == "f32" else W.bf16_bits_from_f32(xf)
        for p in (0.0, 1.0, 0.1, 0.5, 0.999999, 1e-9):
            yo, mo = oracle.dropout(args, code, p, 3, 0, x)
            y, m = gpu_dropout(dtype, args, p, 3, 0, x)
            assert np.array_equal(m, mo), (dtype, p)
            assert_float_bits_equal(y, yo, "dropout %s p=%g" % (dtype, p))
            y2, _ = gpu_dropout(dtype, args, p, 3, 0, x, with_mask=False, in_place=True)
            assert_float_bits_equal(y2, yo, "dropout in place %s p=%g" % (dtype, p))
        y, m = gpu_dropout(dtype, args, 0.0, 3, 0, x)
        assert y.tobytes() == np.ascontiguousarray(x).tobytes() and m.all()      # p = 0 is the identity, bit for bit
        y, m = gpu_dropout(dtype, args, 1.0, 3, 0, x)
        assert not y.view(np.uint8).any() and not m.any()                         # p = 1 writes +0 everywhere


def test_randint_ranges():
    args = ([1 << 15], [2], [("S", 0)], [1])
    for low, high in ((0, 1), (0, 2), (-3, 4), (10, 10 + (1 << 31)), (0, 1 << 32), (-(1 << 40), -(1 << 40) + 4294967295)):
        got = gpu_fill("randint", None, args, 8, 0, low=low, high=high)
        assert np.array_equal(got, oracle.randint(args, low, high, 8, 0)), (low, high)


def test_launch_on_a_side_stream():
    args = ([1 << 18], [1], [("R",)], [0])
    s = torch.cuda.Stream()
    out = torch.empty(1 << 18, dtype=torch.float32, device=DEV)
    with torch.cuda.stream(s):
        v.vesrng_uniform(v.Sharding(*args), v.F32, 0.0, 1.0, 6, 0, out)
    s.synchronize()
    assert np.array_equal(out.cpu().numpy(), oracle.uniform(args, oracle.F32, 0.0, 1.0, 6, 0, threads=THREADS))


def test_wide_index_path_beyond_2_to_31_local_elements():
    """Local shards with more than 2^31 elements take the 64-bit index kernels; the paper's
    table goes up to 16 GB tensors.  Parity on sampled ranges (the oracle is scalar)."""
    # Unsharded [65537, 65536] fp32 = 2^32 + 65536 elements (16 GiB): one run, aligned kernel.
    # (Two dimensions keep the oracle's explicit index lists short.)
    shape = [65537, 65536]
    n = shape[0] * shape[1]
    args = (shape, [1], [("R",)], [0])
    out = torch.empty(n, dtype=torch.float32, device=DEV)
    say("wide: 16 GiB uniform fill")
    v.vesrng_uniform(v.Sharding(*args), v.F32, 0.0, 1.0, 21, 0, out)
    torch.cuda.synchronize()
    for b, e in ((0, 4096), ((1 << 31) - 2048, (1 << 31) + 2048), ((1 << 32) - 2048, (1 << 32) + 2048), (n - 4096, n)):
        want = oracle.uniform(args, oracle.F32, 0.0, 1.0, 21, 0, i_begin=b, i_end=e).reshape(-1)[b:e]
        assert np.array_equal(out[b:e].cpu().numpy(), want), (b, e)
    del out
    # 2-D column shard, ragged (odd origin and width), 2^31 + ... local elements of raw draws.
    shape, mesh, pls, c = [(1 << 15) + 1, (1 << 17) + 6], [2], [("S", 1)], [1]
    args = (shape, mesh, pls, c)
    lshape, ln = v.vesrng_local_shape(v.Sharding(*args))
    assert ln > 1 << 31 and lshape[1] % 4 != 0
    out = torch.empty(ln, dtype=torch.int32, device=DEV)
    say("wide: ragged raw fill of %d elements" % ln)
    v.vesrng_raw_u32(v.Sharding(*args), 22, 1 << 36, out)
    torch.cuda.synchronize()
    for b, e in ((0, 8192), (ln // 2 - 4096, ln // 2 + 4096), (ln - 8192, ln)):
        want = oracle.raw_u32(args, 22, 1 << 36, i_begin=b, i_end=e).reshape(-1)[b:e]
        assert np.array_equal(out[b:e].cpu().numpy().view(np.uint32), want), (b, e)
    del out


def test_single_misaligned_run_of_more_than_2_to_32_elements():
    """One contiguous shard of 2^32 + 1 elements that starts off a generator-block boundary: the staging
    kernel's large-tile form with a single run longer than any 32-bit quantity (its tile map is checked
    slot by slot on the host by the sanitizer tests; here the kernel itself, on sampled windows, for the
    raw draws, and the normal fill through the same path).  A 1-D tensor of 2^33 + 2 elements is never
    listed by the oracle: the shard's values are those of the unsharded stream at offset + 2^32 + 1."""
    run = (1 << 32) + 1
    shape, mesh, pls, c = [2 * run], [2], [("S", 0)], [1]
    sh = v.Sharding(shape, mesh, pls, c)
    assert v.vesrng_local_shape(sh) == ([run], run)
    seed, offset = 77, 1 << 40
    windows = ((0, 6000), ((1 << 31) - 6000, (1 << 31) + 6000), ((1 << 32) - 6000, run))
    out = torch.empty(run, dtype=torch.int32, device=DEV)
    say("misaligned run: raw fill of %d elements" % run)
    v.vesrng_raw_u32(sh, seed, offset, out)
    torch.cuda.synchronize()
    for b, e in windows:
        # Offset additivity (a pinned property of the oracle): element i of the shard is element
        # i - b of a small unsharded tensor whose stream starts 4-aligned just below offset + run + b.
        p0 = offset + run + b
        base = p0 - p0 % 4
        flat = oracle.raw_u32(([e - b + 4], [1], [("R",)], [0]), seed, base)
        assert np.array_equal(out[b:e].cpu().numpy().view(np.uint32), flat[p0 - base:p0 - base + e - b]), (b, e)
    say("misaligned run: fp32 normal fill")
    outf = out.view(torch.float32)
    v.vesrng_normal(sh, v.F32, 0.0, 1.0, seed, offset, outf)
    torch.cuda.synchronize()
    for b, e in windows:
        p0 = offset + run + b
        base = p0 - p0 % 4
        ref = oracle.normal_f64_values(([e - b + 4], [1], [("R",)], [0]), 0.0, 1.0, seed, base)[p0 - base:p0 - base + e - b]
        err = np.abs(outf[b:e].cpu().numpy().astype(np.float64) - ref)
        assert (err <= 1e-6 * np.maximum(np.abs(ref), 1.0)).all(), (b, e)


# ------------------------------------------- general route and global stride ---
NOT_BOXES = [
    ([96], [2, 3], [("IS", 0, 2), ("S", 0)]),                       # interleaved, then cut across the groups
    ([5, 72], [3, 2, 2], [("IS", 1, 4), ("IS", 1, 3), ("S", 1)]),   # interleave on interleave, groups do not nest
    ([8, 30, 3], [2, 4], [("IS", 1, 5), ("S", 1)]),                 # ragged chunks that straddle groups
]


@pytest.mark.parametrize("op,dtype", [("raw", None), ("uniform", "bf16"), ("normal", "f32"), ("dropout", "bf16"),
                                       ("dropout", "f32"), ("randint", None)])
def test_shards_that_are_not_boxes(op, dtype):
    """Nested / repeated InterleavedShard whose result is not a box takes the element-wise kernel."""
    seed, offset = 31337, 4096
    for shape, mesh, pls in NOT_BOXES:
        shards = {}
        for c in mesh_coords(mesh):
            args = (shape, mesh, pls, list(c))
            what = "%s %s %s" % (op, dtype, args)
            say(what)
            if op == "raw":
                got = gpu_fill("raw", None, args, seed, offset)
                assert np.array_equal(got, oracle.raw_u32(args, seed, offset)), what
                shards[c] = got
            elif op == "randint":
                assert np.array_equal(gpu_fill("randint", None, args, seed, offset, low=0, high=97),
                                      oracle.randint(args, 0, 97, seed, offset)), what
            elif op == "uniform":
                assert_float_bits_equal(gpu_fill("uniform", dtype, args, seed, offset, low=-1.0, high=1.0),
                                        oracle.uniform(args, oracle.BF16, -1.0, 1.0, seed, offset), what)
            elif op == "normal":
                check_normal(gpu_fill("normal", dtype, args, seed, offset), args, dtype, 0.0, 1.0, seed, offset, what)
            else:
                n = oracle.local_shape(*args)[1]
                xf = W.adversarial_f32(n, seed=n)
                x = xf if dtype == "f32" else W.bf16_bits_from_f32(xf)
                y, m = gpu_dropout(dtype, args, 0.25, seed, offset, x)
                yo, mo = oracle.dropout(args, oracle.F32 if dtype == "f32" else oracle.BF16, 0.25, seed, offset, x)
                assert np.array_equal(m, mo), what
                assert_float_bits_equal(y, yo, what)
        if op == "raw":
            # Every global element is held by exactly one rank and carries the single-device value.
            single = gpu_fill("raw", None, (shape, [1], [("R",)], [0]), seed, offset).reshape(-1)
            seen = np.zeros(single.size, dtype=np.int32)
            for c, vals in shards.items():
                j = oracle.global_indices(shape, mesh, pls, list(c)).reshape(-1).astype(np.int64)
                assert np.array_equal(vals.reshape(-1), single[j])
                seen[j] += 1
            assert (seen == 1).all()


def test_non_contiguous_global_view():
    """Algorithm 1 takes the global stride as an input: a transposed (column-major) global tensor
    and a padded one.  Values follow the global flat index, whatever the local layout."""
    seed = 77
    for shape, stride, mesh, pls in [([48, 40], [1, 48], [2, 2], [("S", 0), ("S", 1)]),       # transposed
                                     ([30, 36], [40, 1], [3], [("S", 1)]),                    # rows padded to 40
                                     ([6, 10, 12], [1, 6, 60], [2], [("S", 2)])]:             # fully reversed order
        off = 8
        for c in mesh_coords(mesh):
            args = (shape, mesh, pls, list(c), stride)
            sh = v.Sharding(*args)
            lshape, n = v.vesrng_local_shape(sh)
            out = torch.empty(n, dtype=torch.int32, device=DEV)
            v.vesrng_raw_u32(sh, seed, off, out)
            got = out.cpu().numpy().view(np.uint32).reshape(lshape)
            assert np.array_equal(got, oracle.raw_u32(args, seed, off)), args
            o2 = torch.empty(n, dtype=torch.float32, device=DEV)
            v.vesrng_normal(sh, v.F32, 0.0, 1.0, seed, off, o2)
            ref = oracle.normal_f64_values(args, 0.0, 1.0, seed, off).reshape(-1)
            err = np.abs(o2.cpu().numpy().astype(np.float64) - ref)
            assert (err <= 1e-6 * np.maximum(np.abs(ref), 1.0)).all(), args
        nxt = v.vesrng_advance_offset(v.Sharding(shape, mesh, pls, [0] * len(mesh), stride), off)
        assert nxt == oracle.advance_offset(shape, off, stride)


def test_dropout_backward_regenerates_the_mask():
    """Mask-free dropout: with mask = NULL the pass moves 4 B/element instead of 5, and the
    backward pass is the same call on the incoming gradient with the forward's (seed, offset):
    it regenerates the keep decisions instead of reading a stored mask."""
    args = ([64, 96, 50], [4], [("S", 1)], [2])
    n = oracle.local_shape(*args)[1]
    rng = np.random.default_rng(5)
    x = W.bf16_bits_from_f32(rng.standard_normal(n).astype(np.float32))
    gy = W.bf16_bits_from_f32(rng.standard_normal(n).astype(np.float32))
    y, m = gpu_dropout("bf16", args, 0.2, 999, 64, x)
    gx, _ = gpu_dropout("bf16", args, 0.2, 999, 64, gy, with_mask=False)
    gxo, mo = oracle.dropout(args, oracle.BF16, 0.2, 999, 64, gy)
    assert np.array_equal(gx, gxo) and np.array_equal(m, mo)
    assert not gx[m == 0].any() and (gx[m == 1] != 0).mean() > 0.99


@pytest.mark.parametrize("theta", [1, 7, 1024, 1 << 40])
def test_virtual_thread_layout(theta):
    """Algorithm 1 to the letter (global thread count theta): every operator, sharded, against the oracle."""
    seed, offset = (0xBEEF << 32) | 17, 1 << 33
    for shape, mesh, pls in (([129, 67], [2, 3], [("S", 0), ("S", 1)]), ([4, 36, 5], [4], [("IS", 1, 3)])):
        single = None
        shards = {}
        for c in mesh_coords(mesh):
            args = (shape, mesh, pls, list(c), None, theta)
            sh = v.Sharding(*args)
            lshape, n = v.vesrng_local_shape(sh)
            what = "theta=%d %s" % (theta, args[:4])
            say(what)
            out = torch.empty(max(n, 1), dtype=torch.int32, device=DEV)
            v.vesrng_raw_u32(sh, seed, offset, out)
            raw = out.cpu().numpy().view(np.uint32)[:n].reshape(lshape)
            assert np.array_equal(raw, oracle.raw_u32(args, seed, offset)), what
            shards[c] = raw
            o2 = torch.empty(max(n, 1), dtype=torch.float32, device=DEV)
            v.vesrng_normal(sh, v.F32, 0.0, 1.0, seed, offset, o2)
            ref = oracle.normal_f64_values(args, 0.0, 1.0, seed, offset).reshape(-1)
            err = np.abs(o2.cpu().numpy()[:n].astype(np.float64) - ref)
            assert (err <= 1e-6 * np.maximum(np.abs(ref), 1.0)).all(), what
            o3 = torch.empty(max(n, 1), dtype=torch.bfloat16, device=DEV)
            v.vesrng_uniform(sh, v.BF16, 0.0, 1.0, seed, offset, o3)
            assert np.array_equal(o3.view(torch.int16).cpu().numpy().view(np.uint16)[:n].reshape(lshape),
                                  oracle.uniform(args, oracle.BF16, 0.0, 1.0, seed, offset)), what
            x = W.bf16_bits_from_f32(W.adversarial_f32(n, seed=n))
            xd = torch.from_numpy(x.view(np.int16)).to(DEV).view(torch.bfloat16)
            y = torch.empty_like(xd)
            m = torch.empty(max(n, 1), dtype=torch.uint8, device=DEV)
            v.vesrng_dropout(sh, v.BF16, 0.5, seed, offset, xd, y, m)
            yo, mo = oracle.dropout(args, oracle.BF16, 0.5, seed, offset, x)
            assert np.array_equal(m.cpu().numpy()[:n].reshape(lshape), mo), what
            assert_float_bits_equal(y.view(torch.int16).cpu().numpy().view(np.uint16)[:n].reshape(lshape), yo, what)
        sh1 = v.Sharding(shape, [1], [("R",)], [0], None, theta)
        out = torch.empty(int(np.prod(shape)), dtype=torch.int32, device=DEV)
        v.vesrng_raw_u32(sh1, seed, offset, out)
        single = out.cpu().numpy().view(np.uint32).reshape(shape)
        assert np.array_equal(merge_shards(shards, mesh, pls), single)
        assert v.vesrng_advance_offset(sh1, offset) == oracle.advance_offset(shape, offset, None, theta)


@pytest.mark.parametrize("theta", [4, 8, 64, 256, 4096])
def test_virtual_thread_layout_one_generator_call_per_four_outputs(theta):
    """Contiguous shards (unsharded tensors, row shards) that are many step groups long take the
    kernel in which a thread owns a column of virtual threads and four steps: all four words of every
    generator block are used.  Every operator and dtype against the oracle, ragged ends included."""
    seed, offset = (0xFACE << 32) | 99, 1 << 35
    cases = [([1000, 80], [1], [("R",)], [0]),                     # unsharded
             ([1000, 80], [4], [("S", 0)], [2]),                   # row shard: origin 40000
             ([999, 88], [3], [("S", 0)], [1]),                    # 333 rows: origin 29304, ragged length
             ([262144 + 8 * 3 + 5], [1], [("R",)], [0]),           # 1-D, last unit partial
             ([64, 4096 + 8], [2], [("S", 0)], [1])]
    ran = 0
    for shape, mesh, pls, c in cases:
        args = (shape, mesh, pls, c, None, theta)
        sh = v.Sharding(*args)
        lshape, n = v.vesrng_local_shape(sh)
        if n < 64 * theta:
            continue
        ran += 1
        what = "theta=%d %s" % (theta, args[:4])
        say(what)
        assert np.array_equal(gpu_fill("raw", None, args, seed, offset), oracle.raw_u32(args, seed, offset, threads=THREADS)), what
        assert np.array_equal(gpu_fill("randint", None, args, seed, offset, low=-7, high=1000),
                              oracle.randint(args, -7, 1000, seed, offset, threads=THREADS)), what
        for dtype in ("f32", "bf16", "f16"):
            got = gpu_fill("uniform", dtype, args, seed, offset, low=-1.0, high=2.0)
            want = oracle.uniform(args, DT[dtype][2], -1.0, 2.0, seed, offset, threads=THREADS)
            assert_float_bits_equal(got, want, what + " uniform " + dtype, dtype=dtype)
            got = gpu_fill("normal", dtype, args, seed, offset, mean=0.5, std=2.0)
            check_normal(got, args, dtype, 0.5, 2.0, seed, offset, what + " normal " + dtype)
            xf = W.adversarial_f32(n, seed=theta)
            x = xf if dtype == "f32" else W.bits16_from_f32(xf, dtype)
            y, m = gpu_dropout(dtype, args, 0.2, seed, offset, x)
            yo, mo = oracle.dropout(args, DT[dtype][2], 0.2, seed, offset, x, threads=THREADS)
            assert np.array_equal(m, mo), what
            assert_float_bits_equal(y, yo, what + " dropout " + dtype, dtype=dtype)
            y, _ = gpu_dropout(dtype, args, 0.2, seed, offset, x, with_mask=False, in_place=True)
            assert_float_bits_equal(y, yo, what + " dropout in place " + dtype, dtype=dtype)
        r = W.bf16_bits_from_f32(W.adversarial_f32(n, seed=theta + 1))
        xb = W.bf16_bits_from_f32(xf)
        yo, mo = oracle.dropout_add(args, oracle.BF16, 0.2, seed, offset, xb, r, threads=THREADS)
        xd, rd = to_device(xb, "bf16"), to_device(r, "bf16")
        yd = torch.empty_like(xd)
        md = torch.empty(n, dtype=torch.uint8, device=DEV)
        v.vesrng_dropout_add(sh, v.BF16, 0.2, seed, offset, xd, rd, yd, md)
        torch.cuda.synchronize()
        assert np.array_equal(md.cpu().numpy().reshape(lshape), mo), what
        assert_float_bits_equal(to_host(yd, "bf16").reshape(lshape), yo, what + " dropout_add")
    assert ran >= 1
    # The shards of a row-sharded tensor merge to the unsharded tensor in this layout too.
    shape, mesh, pls = [1024, 96], [4], [("S", 0)]
    if 64 * theta <= 256 * 96:
        shards = {c: gpu_fill("raw", None, (shape, mesh, pls, list(c), None, theta), seed, offset) for c in mesh_coords(mesh)}
        single = gpu_fill("raw", None, (shape, [1], [("R",)], [0], None, theta), seed, offset)
        assert np.array_equal(merge_shards(shards, mesh, pls), single)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_dropout_add_residual(dtype):
    """Fused dropout + residual add, aligned / tiled / element-wise kernels, in place on either input."""
    seed, offset = 2024, 128
    code, ocode = (v.F32, oracle.F32) if dtype == "f32" else (v.BF16, oracle.BF16)
    for args in (([64, 4096], [4], [("S", 0)], [3]),                               # aligned
                 ([8, 64, 1024], [2], [("S", 1)], [1]),                            # aligned, 8 runs of whole wavefronts
                 ([300, 333], [3], [("S", 1)], [1]),                               # ragged column shard (tiled)
                 ([40, 7], [2], [("S", 1)], [1]),                                  # runs of 3: element-wise
                 ([96], [2, 3], [("IS", 0, 2), ("S", 0)], [1, 1])):                # not a box
        sh = v.Sharding(*args)
        lshape, n = v.vesrng_local_shape(sh)
        xf, rf = W.adversarial_f32(n, seed=1), W.adversarial_f32(n, seed=2)
        x, r = (xf, rf) if dtype == "f32" else (W.bf16_bits_from_f32(xf), W.bf16_bits_from_f32(rf))
        yo, mo = oracle.dropout_add(args, ocode, 0.1, seed, offset, x, r)

        def dev(a):
            return (torch.from_numpy(a).to(DEV) if dtype == "f32"
                    else torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16))

        def host(t):
            return t.cpu().numpy() if dtype == "f32" else t.view(torch.int16).cpu().numpy().view(np.uint16)

        for alias in ("none", "x", "residual"):
            xd, rd = dev(x), dev(r)
            yd = {"none": torch.empty_like(xd), "x": xd, "residual": rd}[alias]
            m = torch.empty(max(n, 1), dtype=torch.uint8, device=DEV)
            v.vesrng_dropout_add(sh, code, 0.1, seed, offset, xd, rd, yd, m)
            torch.cuda.synchronize()
            what = "dropout_add %s %s alias=%s" % (dtype, args, alias)
            assert np.array_equal(m.cpu().numpy()[:n].reshape(lshape), mo), what
            assert_float_bits_equal(host(yd)[:n].reshape(lshape), yo, what)


def test_random_descriptions_all_kernel_flavours():
    """Seeded random meshes / placements / strides / layouts / offsets: raw draws, fp32 normals and
    bf16 dropout against the oracle.  Exercises the choice between the aligned, tiled, ragged and
    element-wise kernels and the 0 / 1 / many run-axis specialisations."""
    from test_host_abi import _random_description
    rng = np.random.default_rng(977)
    done = 0
    while done < 160:
        shape, mesh, pls, coord, stride = _random_description(rng, max_extent=40)
        theta = int(rng.choice([0, 0, 0, 3, 64]))
        try:
            n = oracle.local_shape(shape, mesh, pls, coord)[1]
        except oracle.OracleError:
            continue
        if n == 0 or n > 400000:
            continue
        seed = int(rng.integers(0, 2 ** 63))
        offset = 4 * int(rng.integers(0, 2 ** 40))
        args = (shape, mesh, pls, coord, stride, theta)
        what = str(args)
        say(what)
        sh = v.Sharding(*args)
        lshape = v.vesrng_local_shape(sh)[0]
        out = torch.empty(n, dtype=torch.int32, device=DEV)
        v.vesrng_raw_u32(sh, seed, offset, out)
        assert np.array_equal(out.cpu().numpy().view(np.uint32).reshape(lshape), oracle.raw_u32(args, seed, offset)), what
        o2 = torch.empty(n, dtype=torch.float32, device=DEV)
        v.vesrng_normal(sh, v.F32, -1.0, 2.0, seed, offset, o2)
        ref = oracle.normal_f64_values(args, -1.0, 2.0, seed, offset).reshape(-1)
        err = np.abs(o2.cpu().numpy().astype(np.float64) - ref)
        assert (err <= 1e-6 * np.maximum(np.abs(ref), 2.0)).all(), what
        x = W.bf16_bits_from_f32(W.adversarial_f32(n, seed=done))
        xd = torch.from_numpy(x.view(np.int16)).to(DEV).view(torch.bfloat16)
        y = torch.empty_like(xd)
        m = torch.empty(n, dtype=torch.uint8, device=DEV)
        v.vesrng_dropout(sh, v.BF16, 0.15, seed, offset, xd, y, m)
        yo, mo = oracle.dropout(args, oracle.BF16, 0.15, seed, offset, x)
        assert np.array_equal(m.cpu().numpy().reshape(lshape), mo), what
        assert_float_bits_equal(y.view(torch.int16).cpu().numpy().view(np.uint16).reshape(lshape), yo, what)
        done += 1


def test_random_mid_sized_descriptions():
    """Seeded random tensors of two to five dimensions with 1 M to 12 M local elements on random meshes (Shard and
    InterleavedShard, some with padded global strides): sizes at which the staging windows of the operators, the
    large tile, and the kernels written out for one, two and three axes of runs are all in play.  Raw draws, the bf16
    uniform fill, the fp32 normal fill and fused bf16 dropout against the threaded oracle."""
    rng = np.random.default_rng(31415)
    done = 0
    while done < 14:
        nd = int(rng.integers(2, 6))
        target = float(rng.uniform(2e6, 4e7))
        cuts = np.sort(rng.uniform(0, 1, size=nd - 1))
        parts = np.diff(np.concatenate([[0.0], cuts, [1.0]]))
        shape = [max(2, int(round(target ** p))) for p in parts]
        if rng.random() < 0.6:
            shape[-1] = max(shape[-1], int(rng.integers(64, 3000)))      # an innermost dimension long enough to tile
        md = int(rng.integers(1, 4))
        mesh = [int(x) for x in rng.integers(2, 4, size=md)]
        pls = []
        for _ in range(md):
            d = int(rng.integers(0, nd))
            pls.append(("S", d) if rng.random() < 0.8 else ("IS", d, int(rng.integers(2, 4))))
        coord = [int(rng.integers(0, p)) for p in mesh]
        stride = None
        if rng.random() < 0.25:
            stride, acc = [0] * nd, 1
            for d in range(nd - 1, -1, -1):
                stride[d] = acc
                acc *= shape[d] + int(rng.integers(0, 4))
        try:
            n = oracle.local_shape(shape, mesh, pls, coord)[1]
        except oracle.OracleError:
            continue
        if n < 1_000_000 or n > 12_000_000 or int(np.prod(shape)) > 150_000_000:
            continue
        seed, offset = int(rng.integers(0, 2 ** 63)), 4 * int(rng.integers(0, 2 ** 40))
        args = (shape, mesh, pls, coord, stride)
        what = "%s (%d local elements)" % (args, n)
        say("random mid-sized " + what)
        got = gpu_fill("raw", None, args, seed, offset)
        assert np.array_equal(got, oracle.raw_u32(args, seed, offset, threads=THREADS)), what
        got = gpu_fill("uniform", "bf16", args, seed, offset, low=-2.0, high=2.0)
        assert np.array_equal(got, oracle.uniform(args, oracle.BF16, -2.0, 2.0, seed, offset, threads=THREADS)), what
        got = gpu_fill("normal", "f32", args, seed, offset, mean=0.25, std=1.5)
        check_normal(got, args, "f32", 0.25, 1.5, seed, offset, "normal f32 " + what)
        x = W.bf16_bits_from_f32(W.adversarial_f32(n, seed=done))
        yo, mo = oracle.dropout(args, oracle.BF16, 0.2, seed, offset, x, threads=THREADS)
        y, mk = gpu_dropout("bf16", args, 0.2, seed, offset, x)
        assert np.array_equal(mk, mo), what
        assert_float_bits_equal(y, yo, "dropout bf16 " + what)
        done += 1


def test_ceiling_probes_do_what_they_say():
    """The measurement aids (their own library): store patterns in every form, copy, dropout traffic
    pattern, generator-only and issue-rate loops, the clock probe and the device properties the
    roofline's denominators come from."""
    from paper_2509_07003_amd import bench_binding as b
    cus, shader_khz, memory_khz, bus_bits, wall_khz = b.vesrng_bench_device_info()
    assert cus == torch.cuda.get_device_properties(0).multi_processor_count
    assert shader_khz > 0 and memory_khz > 0 and bus_bits >= 1024 and wall_khz > 0
    units = 4096 + 3
    want = np.arange(units, dtype=np.int32)[:, None] + np.arange(4, dtype=np.int32)[None, :]
    for kind in (b.PROBE_STORE, b.PROBE_STORE_NT, b.PROBE_STORE_PLAIN, b.PROBE_STORE_GRID_STRIDE,
                 b.PROBE_STORE_4_PER_THREAD):
        say("store probe %d" % kind)
        a = torch.zeros(units * 4 + 4, dtype=torch.int32, device=DEV)
        b.vesrng_bench_probe(kind, units, None, a)
        torch.cuda.synchronize()
        got = a.cpu().numpy()
        assert np.array_equal(got[:units * 4].reshape(units, 4), want), kind
        assert not got[units * 4:].any(), kind                      # nothing past the last unit
    # Unaligned form: unit t at words 4t + 1 .. 4t + 4, the last unit left out.
    u = torch.zeros(units * 4, dtype=torch.int32, device=DEV)
    b.vesrng_bench_probe(b.PROBE_STORE_UNALIGNED, units, None, u)
    torch.cuda.synchronize()
    got = u.cpu().numpy()
    assert got[0] == 0 and np.array_equal(got[1:4 * (units - 1) + 1].reshape(units - 1, 4), want[:units - 1])
    assert not got[4 * (units - 1) + 1:].any()
    a = a[:units * 4].clone()
    bb = torch.zeros_like(a)
    b.vesrng_bench_probe(b.PROBE_COPY, units, a, bb)
    for kind in (b.PROBE_DROPOUT_TRAFFIC, b.PROBE_DROPOUT_TRAFFIC_NT, b.PROBE_DROPOUT_TRAFFIC_LOAD_PLAIN,
                 b.PROBE_DROPOUT_TRAFFIC_LOAD_SC1, b.PROBE_DROPOUT_TRAFFIC_LOAD_SC0SC1,
                 b.PROBE_DROPOUT_TRAFFIC_7_WAVES, b.PROBE_DROPOUT_TRAFFIC_6_WAVES):
        m = torch.zeros(units * 2, dtype=torch.int32, device=DEV)
        c = torch.zeros_like(a)
        b.vesrng_bench_probe(kind, units, a, c, m)
        torch.cuda.synchronize()
        assert torch.equal(a, c)
        assert np.array_equal(m.cpu().numpy().reshape(units, 2), want[:, :2] & 0x01010101)
    # Wide-mask form: x and y as in the others (whole waves of unit pairs only), 16 mask bytes per thread.
    wu = 1024
    aw = a[:wu * 4].clone()
    c = torch.zeros_like(aw)
    m = torch.zeros(wu * 2, dtype=torch.int32, device=DEV)
    b.vesrng_bench_probe(b.PROBE_DROPOUT_TRAFFIC_WIDE_MASK, wu, aw, c, m)
    torch.cuda.synchronize()
    assert torch.equal(aw, c) and m.cpu().numpy().any()
    # Generator-only and issue-rate loops generate and discard: bb must stay a copy of a.
    b.vesrng_bench_probe(b.PROBE_PHILOX, 1 << 20, None, bb)
    b.vesrng_bench_probe(b.PROBE_PHILOX_TWO_XOR, 1 << 20, None, bb)
    for cls in range(len(b.ALU_CLASSES)):
        say("issue-rate loop %s" % b.ALU_CLASSES[cls])
        b.vesrng_bench_alu(cls, 64, 4, bb)
    torch.cuda.synchronize()
    assert torch.equal(a, bb)
    ticks = torch.zeros(4, dtype=torch.int64, device=DEV)
    b.vesrng_bench_clock(2000, ticks)
    torch.cuda.synchronize()
    t = ticks.cpu().numpy()
    assert t[0] > 0 and t[1] > 0 and t[3] == 2000


def test_in_place_dropout_on_ragged_and_non_box_shards():
    for args in (([300, 333], [3], [("S", 1)], [1]), ([40, 7], [2], [("S", 1)], [1]),
                 ([96], [2, 3], [("IS", 0, 2), ("S", 0)], [1, 1]), ([5, 9, 11], [2, 2], [("S", 2), ("S", 0)], [1, 0])):
        n = oracle.local_shape(*args)[1]
        for dtype, code in (("f32", oracle.F32), ("bf16", oracle.BF16)):
            xf = W.adversarial_f32(n, seed=7)
            x = xf if dtype == "f32" else W.bf16_bits_from_f32(xf)
            yo, mo = oracle.dropout(args, code, 0.35, 12, 64, x)
            y, m = gpu_dropout(dtype, args, 0.35, 12, 64, x, with_mask=True, in_place=True)
            assert np.array_equal(m, mo), (args, dtype)
            assert_float_bits_equal(y, yo, "in-place dropout %s %s" % (dtype, args))


def test_calls_can_be_captured_in_a_hip_graph_and_replayed():
    """The entry points only enqueue kernels (no allocation, no synchronisation, no memset), so a
    caller can capture them; every replay must reproduce the eager result."""
    args = ([64, 1030], [3], [("S", 1)], [1])            # ragged: tiled dropout + ragged normal
    sh = v.Sharding(*args)
    lshape, n = v.vesrng_local_shape(sh)
    x_bits = W.bf16_bits_from_f32(np.random.default_rng(3).standard_normal(n).astype(np.float32))
    x = torch.from_numpy(x_bits.view(np.int16)).to(DEV).view(torch.bfloat16)
    y = torch.empty_like(x)
    mask = torch.empty(n, dtype=torch.uint8, device=DEV)
    z = torch.empty(n, dtype=torch.float32, device=DEV)
    yo, mo = oracle.dropout(args, oracle.BF16, 0.1, 5, 0, x_bits)
    zo = oracle.normal_f64_values(args, 0.0, 1.0, 5, 4096).reshape(-1)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        v.vesrng_dropout(sh, v.BF16, 0.1, 5, 0, x, y, mask)      # warm-up outside the capture
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            v.vesrng_dropout(sh, v.BF16, 0.1, 5, 0, x, y, mask)
            v.vesrng_normal(sh, v.F32, 0.0, 1.0, 5, 4096, z)
    for replay in range(3):
        y.fill_(1.0)
        mask.fill_(9)
        z.fill_(-7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(mask.cpu().numpy().reshape(lshape), mo), replay
        assert np.array_equal(y.view(torch.int16).cpu().numpy().view(np.uint16).reshape(lshape), yo), replay
        err = np.abs(z.cpu().numpy().astype(np.float64) - zo)
        assert (err <= 1e-6 * np.maximum(np.abs(zo), 1.0)).all(), replay


def test_large_masked_dropout_launch_form_in_a_graph_and_against_the_oracle():
    """Aligned fused dropout that writes a mask is launched with at most seven resident waves per SIMD once it has
    2^23 units and more (untouched dynamic LDS per workgroup).  The values must not depend on that: a 2^26-element
    bf16 shard and a 2^25-element fp32 shard against the oracle on sampled windows, against the same call without a
    mask (launched at the hardware's eight waves), and captured in a HIP graph and replayed."""
    seed, offset = 97531, 1 << 35
    rng = np.random.default_rng(5)
    for dtype, code, n in (("bf16", oracle.BF16, 1 << 26), ("f32", oracle.F32, 1 << 25)):
        args = ([n], [1], [("R",)], [0])
        sh = v.Sharding(*args)
        x = torch.randn(n, dtype=torch.float32, device=DEV)
        x = x.to(torch.bfloat16) if dtype == "bf16" else x
        y = torch.empty_like(x)
        y2 = torch.empty_like(x)
        mask = torch.empty(n, dtype=torch.uint8, device=DEV)
        say("large masked dropout %s" % dtype)
        v.vesrng_dropout(sh, DT[dtype][1], 0.2, seed, offset, x, y, mask)
        v.vesrng_dropout(sh, DT[dtype][1], 0.2, seed, offset, x, y2, None)       # the launch form without the cap
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16 if dtype == "bf16" else torch.int32),
                           y2.view(torch.int16 if dtype == "bf16" else torch.int32))
        x_host = to_host(x, dtype)
        for begin in [0, n - 4096] + [int(b) for b in rng.integers(0, n - 4096, size=6)]:
            yo, mo = oracle.dropout(args, code, 0.2, seed, offset, x_host, i_begin=begin, i_end=begin + 4096)
            assert np.array_equal(mask[begin:begin + 4096].cpu().numpy(), mo.reshape(-1)[begin:begin + 4096]), (dtype, begin)
            assert_float_bits_equal(to_host(y[begin:begin + 4096], dtype), yo.reshape(-1)[begin:begin + 4096],
                                    "large masked dropout %s at %d" % (dtype, begin), dtype=dtype)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        y3 = torch.empty_like(x)
        m3 = torch.empty_like(mask)
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                v.vesrng_dropout(sh, DT[dtype][1], 0.2, seed, offset, x, y3, m3)
        for replay in range(2):
            y3.fill_(3.0)
            m3.fill_(9)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(m3, mask), (dtype, replay)
            assert torch.equal(y3.view(torch.int16 if dtype == "bf16" else torch.int32),
                               y.view(torch.int16 if dtype == "bf16" else torch.int32)), (dtype, replay)
        del x, y, y2, y3, mask, m3


@pytest.mark.parametrize("label,shape", [("262 KB", [8, 16, 8, 8, 8]), ("64 MB", [16, 32, 32, 32, 32]),
                                          ("1 GB", [32, 64, 32, 64, 64])])
def test_table5_sizes_5d_double_sharding(label, shape):
    """The paper's per-operator table at its own tensor sizes (fp32 element counts of 262 KB, 64 MB
    and 1 GB; the 16 GB point is test_wide_index_path...): 5-D tensors, sharded on two different
    dimensions and twice on the same dimension, one rank of each checked against the threaded oracle."""
    numel = int(np.prod(shape))
    assert numel * 4 in (262144, 64 << 20, 1 << 30)
    seed, offset = 20240611, 1 << 20
    for mesh, pls, coord in (([2, 2], [("S", 1), ("S", 3)], [1, 0]), ([2, 4], [("S", 4), ("S", 4)], [1, 2]),
                             ([4], [("S", 0)], [3])):
        args = (shape, mesh, pls, coord)
        what = "%s %s" % (label, args)
        say(what)
        got = gpu_fill("uniform", "f32", args, seed, offset)
        want = oracle.uniform(args, oracle.F32, 0.0, 1.0, seed, offset, threads=THREADS)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), what
        del got, want
        got = gpu_fill("normal", "bf16", args, seed, offset, mean=0.0, std=0.02)
        check_normal(got, args, "bf16", 0.0, 0.02, seed, offset, what)
        del got
        n = oracle.local_shape(*args)[1]
        x = W.bf16_bits_from_f32(np.random.default_rng(n % 1000).standard_normal(n, dtype=np.float32))
        y, m = gpu_dropout("bf16", args, 0.1, seed, offset, x)
        yo, mo = oracle.dropout(args, oracle.BF16, 0.1, seed, offset, x, threads=THREADS)
        assert np.array_equal(m, mo), what
        assert_float_bits_equal(y, yo, what)


def _table5_shardings(ndim=5):
    """Every single shard dimension "#a" (1-D mesh of 4) and every ordered pair "#a and #b", a = b
    included (2-D mesh 2 x 2): the sharding column of the paper's per-operator table."""
    for a in range(ndim):
        yield [4], [("S", a)], [a % 4]
    for k, (a, b) in enumerate(itertools.product(range(ndim), repeat=2)):
        yield [2, 2], [("S", a), ("S", b)], [k % 2, (k // 2) % 2]


@pytest.mark.parametrize("ops", ["raw+randint", "uniform", "normal", "dropout"])
def test_table5_full_double_sharding_grid_at_64mb(ops):
    """The paper's micro-benchmark grid (App. C, Table 5) at its 64 MB point (2^24 fp32 elements, 5-D):
    all 5 single and all 25 double shardings, every operator and dtype, one rank of each against the
    threaded oracle element by element; a second shape with odd extents makes every shard ragged."""
    seed, offset = 20250101, 1 << 30
    even, odd = [16, 32, 32, 32, 32], [15, 33, 31, 34, 31]
    assert int(np.prod(even)) * 4 == 64 << 20
    count = 0
    for shape in (even, odd):
        for k, (mesh, pls, coord) in enumerate(_table5_shardings()):
            args = (shape, mesh, pls, coord)
            what = "%s %s" % (ops, args)
            say(what)
            light = shape is odd and k % 3 != 0      # the odd shape: every third sharding in full
            if ops == "raw+randint":
                assert np.array_equal(gpu_fill("raw", None, args, seed, offset),
                                      oracle.raw_u32(args, seed, offset, threads=THREADS)), what
                if not light:
                    assert np.array_equal(gpu_fill("randint", None, args, seed, offset, low=-3, high=100000),
                                          oracle.randint(args, -3, 100000, seed, offset, threads=THREADS)), what
            elif ops == "uniform":
                for dtype in ("f32", "bf16") + (("f16",) if k % 5 == 0 else ()):
                    if light and dtype != "bf16":
                        continue
                    got = gpu_fill("uniform", dtype, args, seed, offset, low=-1.0, high=1.0)
                    want = oracle.uniform(args, DT[dtype][2], -1.0, 1.0, seed, offset, threads=THREADS)
                    assert_float_bits_equal(got, want, what + dtype, dtype=dtype)
            elif ops == "normal":
                for dtype in ("f32", "bf16") + (("f16",) if k % 5 == 1 else ()):
                    if light and dtype != "f32":
                        continue
                    got = gpu_fill("normal", dtype, args, seed, offset, mean=0.0, std=0.02)
                    check_normal(got, args, dtype, 0.0, 0.02, seed, offset, what + dtype)
            else:
                n = oracle.local_shape(*args)[1]
                xf = np.random.default_rng(k).standard_normal(n, dtype=np.float32)
                for dtype in ("bf16", "f32") + (("f16",) if k % 5 == 2 else ()):
                    if light and dtype != "bf16":
                        continue
                    x = xf if dtype == "f32" else W.bits16_from_f32(xf, dtype)
                    y, m = gpu_dropout(dtype, args, 0.1, seed, offset, x)
                    yo, mo = oracle.dropout(args, DT[dtype][2], 0.1, seed, offset, x, threads=THREADS)
                    assert np.array_equal(m, mo), what + dtype
                    assert_float_bits_equal(y, yo, what + dtype, dtype=dtype)
            count += 1
    assert count == 60


def _windows(n, width=20000):
    """Sampled index windows of a local shard: both ends, the middle, and the 2^31 / 2^32 crossings."""
    marks = [0, n // 3, n // 2, (1 << 31), (1 << 32), n - width]
    out = []
    for mk in marks:
        b = max(0, min(n - width, mk - width // 2))
        if all(abs(b - ob) >= width for ob, _ in out):
            out.append((b, b + width))
    return out


@pytest.mark.parametrize("label,shape", [("1 GB", [32, 64, 32, 64, 64]), ("16 GB", [64, 64, 64, 128, 128])])
def test_table5_large_tensors_on_sampled_windows(label, shape):
    """The 1 GB and 16 GB points of the paper's table (2^28 and 2^32 fp32 elements): a nested shard of
    one dimension, an interleaved shard, a ragged shard of the innermost dimension and a ragged nested
    shard of two inner dimensions; fp32 uniform fill, fp32 normal fill and fused bf16 dropout, compared
    with the oracle on sampled windows of the local shard (the oracle is scalar)."""
    numel = int(np.prod(shape))
    assert numel * 4 in (1 << 30, 16 << 30)
    seed, offset = 424242, 1 << 37
    cases = [([2, 4], [("S", 1), ("S", 1)], [1, 2]),               # "#1 and #1": nested, same dimension
             ([8], [("IS", 1, 4)], [5]),                           # interleaved: heads dealt out in 4 groups
             ([3], [("S", 4)], [1]),                               # ragged innermost dimension (64 or 128 over 3)
             ([3, 3], [("S", 3), ("S", 4)], [2, 2]),               # "#3 and #4", both ragged
             ([2], [("S", 1)], [1])]                               # "#1": aligned runs; 2^31 local elements at 16 GB (64-bit index kernels)
    for mesh, pls, coord in cases:
        args = (shape, mesh, pls, coord)
        sh = v.Sharding(*args)
        lshape, n = v.vesrng_local_shape(sh)
        what = "%s %s (%d local elements)" % (label, args, n)
        say(what)
        wins = _windows(n)
        out = torch.empty(n, dtype=torch.float32, device=DEV)
        v.vesrng_uniform(sh, v.F32, 0.0, 1.0, seed, offset, out)
        torch.cuda.synchronize()
        for b, e in wins:
            want = oracle.uniform(args, oracle.F32, 0.0, 1.0, seed, offset, i_begin=b, i_end=e).reshape(-1)[b:e]
            assert np.array_equal(out[b:e].cpu().numpy(), want), (what, b, e)
        v.vesrng_normal(sh, v.F32, 0.0, 1.0, seed, offset, out)
        torch.cuda.synchronize()
        for b, e in wins:
            ref = oracle.normal_f64_values(args, 0.0, 1.0, seed, offset, i_begin=b, i_end=e).reshape(-1)[b:e]
            err = np.abs(out[b:e].cpu().numpy().astype(np.float64) - ref)
            assert (err <= 1e-6 * np.maximum(np.abs(ref), 1.0)).all(), (what, b, e)
        del out
        # Fused bf16 dropout: input made on the device, the windows copied to the host for the oracle.
        gen = torch.Generator(device=DEV)
        gen.manual_seed(n % 1000)
        x = torch.empty(n, dtype=torch.bfloat16, device=DEV)
        x.normal_(generator=gen)
        y = torch.empty_like(x)
        mask = torch.empty(n, dtype=torch.uint8, device=DEV)
        v.vesrng_dropout(sh, v.BF16, 0.1, seed, offset, x, y, mask)
        torch.cuda.synchronize()
        xh = np.zeros(n, dtype=np.uint16)               # untouched pages cost nothing
        for b, e in wins:
            xh[b:e] = x[b:e].view(torch.int16).cpu().numpy().view(np.uint16)
        for b, e in wins:
            yo, mo = oracle.dropout(args, oracle.BF16, 0.1, seed, offset, xh, i_begin=b, i_end=e)
            assert np.array_equal(mask[b:e].cpu().numpy(), mo.reshape(-1)[b:e]), (what, b, e)
            assert_float_bits_equal(y[b:e].view(torch.int16).cpu().numpy().view(np.uint16), yo.reshape(-1)[b:e], what)
        keep = float(mask[:1 << 24].float().mean())
        assert abs(keep - 0.9) < 1e-3
        del x, y, mask, xh


def test_shards_beyond_2_to_30_elements_served_piece_by_piece():
    """A shard of 2^30 elements and more with an axis of runs is cut along that axis into pieces that the 32-bit
    kernels serve, one launch each (rows per piece: the largest multiple of 32 whose elements stay below 2^30).
    Windows around every piece boundary, at both ends and in the middle against the oracle: rows of 50 and of 37
    elements off the block grid (staged fp32 uniform, randint), rows of 100 aligned elements (bf16 normal, fused
    bf16 dropout; with residual against a shard that fits 32 bits as a whole), and a shard with rows too long to
    cut, which keeps the 64-bit kernels."""
    seed, offset = 77177, 1 << 36
    width = 6000

    def windows(n, per_index):
        rows = ((1 << 30) - 1) // per_index
        rows -= rows % 32
        marks = [0, n - width, n // 2] + [k * rows * per_index for k in range(1, -(-n // (rows * per_index)))]
        out = []
        for mk in marks:
            b = max(0, min(n - width, mk - width // 2))
            out.append((b, b + width))
        return out

    # Rows of 50 elements starting at column 50 (phase 2): ragged, staged; 1.68e9 elements.
    args = ([1 << 25, 100], [2], [("S", 1)], [1])
    sh = v.Sharding(*args)
    n = v.vesrng_local_shape(sh)[1]
    assert n == 50 << 25
    say("pieces: ragged rows of 50, %d elements" % n)
    out = torch.empty(n, dtype=torch.float32, device=DEV)
    v.vesrng_uniform(sh, v.F32, -1.0, 1.0, seed, offset, out)
    torch.cuda.synchronize()
    wins = windows(n, 50)
    assert len(wins) >= 4
    for b, e in wins:
        want = oracle.uniform(args, oracle.F32, -1.0, 1.0, seed, offset, i_begin=b, i_end=e).reshape(-1)[b:e]
        assert np.array_equal(out[b:e].cpu().numpy(), want), (b, e)
    del out
    args_w = ([1 << 25, 74], [2], [("S", 1)], [1])          # rows of 37 from column 37: 1.24e9 elements, cut in two
    sh_w = v.Sharding(*args_w)
    nw = v.vesrng_local_shape(sh_w)[1]
    outi = torch.empty(nw, dtype=torch.int64, device=DEV)
    v.vesrng_randint(sh_w, -7, 1 << 31, seed, offset, outi)
    torch.cuda.synchronize()
    for b, e in windows(nw, 37):
        want = oracle.randint(args_w, -7, 1 << 31, seed, offset, i_begin=b, i_end=e).reshape(-1)[b:e]
        assert np.array_equal(outi[b:e].cpu().numpy(), want), (b, e)
    args_a = ([1 << 25, 72], [2], [("S", 1)], [1])          # rows of 36 from column 36: whole blocks, the aligned kernel
    sh_a = v.Sharding(*args_a)
    na = v.vesrng_local_shape(sh_a)[1]
    assert (1 << 30) < na <= nw
    v.vesrng_randint(sh_a, 0, 1000, seed, offset, outi[:na])
    torch.cuda.synchronize()
    for b, e in windows(na, 36):
        want = oracle.randint(args_a, 0, 1000, seed, offset, i_begin=b, i_end=e).reshape(-1)[b:e]
        assert np.array_equal(outi[b:e].cpu().numpy(), want), (b, e)
    del outi

    # Rows of 100 aligned elements: bf16 normal fill and fused dropout + residual.
    args = ([1 << 24, 200], [2], [("S", 1)], [1])
    sh = v.Sharding(*args)
    n = v.vesrng_local_shape(sh)[1]
    say("pieces: aligned rows of 100, %d elements" % n)
    wins = windows(n, 100)
    y = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    v.vesrng_normal(sh, v.BF16, 0.0, 1.0, seed, offset, y)
    torch.cuda.synchronize()
    got = np.zeros(n, dtype=np.uint16)              # untouched pages cost nothing
    for b, e in wins:
        got[b:e] = y[b:e].view(torch.int16).cpu().numpy().view(np.uint16)
    for b, e in wins:
        check_normal(got, args, "bf16", 0.0, 1.0, seed, offset, "pieces normal bf16 [%d, %d)" % (b, e), i_begin=b, i_end=e)
    del got
    gen = torch.Generator(device=DEV)
    gen.manual_seed(5)
    x = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    x.normal_(generator=gen)
    r = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    r.normal_(generator=gen)
    mask = torch.empty(n, dtype=torch.uint8, device=DEV)
    v.vesrng_dropout(sh, v.BF16, 0.25, seed, offset, x, y, mask)
    torch.cuda.synchronize()
    xh = np.zeros(n, dtype=np.uint16)
    for b, e in wins:
        xh[b:e] = x[b:e].view(torch.int16).cpu().numpy().view(np.uint16)
    for b, e in wins:
        yo, mo = oracle.dropout(args, oracle.BF16, 0.25, seed, offset, xh, i_begin=b, i_end=e)
        assert np.array_equal(mask[b:e].cpu().numpy(), mo.reshape(-1)[b:e]), (b, e)
        assert_float_bits_equal(y[b:e].view(torch.int16).cpu().numpy().view(np.uint16), yo.reshape(-1)[b:e],
                                "pieces dropout bf16 [%d, %d)" % (b, e))
    del xh
    # Dropout + residual (the residual pointer moves with the pieces too): the lower half of the rows is also a shard
    # of its own (rows cut in two as well) that fits 32-bit indices and holds the piece boundary; same values expected.
    v.vesrng_dropout_add(sh, v.BF16, 0.25, seed, offset, x, r, y, mask)
    half = (1 << 23) * 100
    sub = v.Sharding([1 << 24, 200], [2, 2], [("S", 1), ("S", 0)], [1, 1])
    assert v.vesrng_local_shape(sub)[1] == half and half < ((1 << 30) // 100 // 32 * 32) * 100 < n
    y2 = torch.empty(half, dtype=torch.bfloat16, device=DEV)
    m2 = torch.empty(half, dtype=torch.uint8, device=DEV)
    v.vesrng_dropout_add(sub, v.BF16, 0.25, seed, offset, x[half:], r[half:], y2, m2)
    torch.cuda.synchronize()
    assert torch.equal(m2, mask[half:]) and torch.equal(y2.view(torch.int16), y[half:].view(torch.int16))
    del x, r, y, mask, y2, m2

    # Rows of 2^26 elements: fewer than 32 fit a piece, so the 64-bit kernels serve the shard as a whole.
    args = ([16, 1 << 13, 1 << 14], [2], [("S", 1)], [1])
    sh = v.Sharding(*args)
    n = v.vesrng_local_shape(sh)[1]
    assert n == 1 << 30
    out = torch.empty(n, dtype=torch.float32, device=DEV)
    v.vesrng_uniform(sh, v.F32, 0.0, 1.0, seed, offset, out)
    torch.cuda.synchronize()
    for b, e in ((0, width), (n // 2 - width, n // 2 + width), (n - width, n)):
        want = oracle.uniform(args, oracle.F32, 0.0, 1.0, seed, offset, i_begin=b, i_end=e).reshape(-1)[b:e]
        assert np.array_equal(out[b:e].cpu().numpy(), want), (b, e)
    del out


# ------------------------------------------------------------- binary16 -------
F16_CASES = [([64, 4096], [4], [("S", 0)], [3]),                                 # aligned
             ([6, 64, 512], [2, 2], [("S", 1), ("S", 0)], [1, 1]),               # aligned, several runs of whole wavefronts
             ([300, 333], [3], [("S", 1)], [1]),                                 # ragged column shard (tiled for dropout)
             ([40, 7], [2], [("S", 1)], [1]),                                    # runs of 3: element-wise edges only
             ([5, 6, 7, 8, 9], [2, 2], [("S", 1), ("S", 3)], [1, 0]),            # 5-D, two sharded dims
             ([96], [2, 3], [("IS", 0, 2), ("S", 0)], [1, 1]),                   # not a box
             ([33, 50], [2], [("S", 1)], [0], None, 64)]                         # virtual-thread layout


def test_f16_fills_all_kernel_flavours():
    """IEEE binary16 outputs: uniforms bit-exact (several ranges, the upper guard included), normals
    within the rounding interval of the double-precision value."""
    seed, offset = 99, 4096
    for args in F16_CASES:
        say("f16 fills %s" % (args,))
        for low, high in ((0.0, 1.0), (-0.05, 0.05), (2.0, 2.001), (-65504.0, 65504.0)):
            got = gpu_fill("uniform", "f16", args, seed, offset, low=low, high=high)
            want = oracle.uniform(args, oracle.F16, low, high, seed, offset)
            assert np.array_equal(got, want), (args, low, high)
        for mean, std in ((0.0, 1.0), (0.0, 0.02), (3.0, 1e-4)):
            got = gpu_fill("normal", "f16", args, seed, offset, mean=mean, std=std)
            check_normal(got, args, "f16", mean, std, seed, offset, "normal f16 %s" % (args,))
    # The guard at work on a long stream: every value stays below high although rounding reaches it.
    n = 1 << 18
    flat = ([n], [1], [("R",)], [0])
    got = gpu_fill("uniform", "f16", flat, 77, 0)
    assert np.array_equal(got, oracle.uniform(flat, oracle.F16, 0.0, 1.0, 77, 0, threads=THREADS))
    assert got.max() == 0x3BFF and (got == 0x3BFF).sum() > n // 4096
    sh = v.Sharding(*flat)
    out = torch.empty(n, dtype=torch.float16, device=DEV)
    for low, high in ((-70000.0, 1.0), (0.0, 65536.0)):
        with pytest.raises(v.VesrngError) as e:
            v.vesrng_uniform(sh, v.F16, low, high, 1, 0, out)
        assert e.value.status == 7
    with pytest.raises(v.VesrngError) as e:
        v.vesrng_uniform(sh, 3, 0.0, 1.0, 1, 0, out)
    assert e.value.status == 8


def test_staged_normal_and_sixteen_bit_fills_on_mid_sized_ragged_shards():
    """The fp32 normal fill below 2^24 elements and the 16-bit uniform and normal fills of 2^21 .. 2^25 elements (runs
    of 256 and more) take the staging kernel on ragged shards; just outside those windows they take the kernel without
    staging.  Both sides of every limit against the oracle, with the short and the general form of the tile map."""
    seed, offset = 13579, 1 << 33
    inside = [([2048, 4096], [3], [("S", 1)], [1]),          # 2.8 M elements, runs of 1366, one phase
              ([2100, 4101], [3], [("S", 1)], [2]),          # 2.9 M, runs of 1367, rotating phases
              ([9000, 1028], [2], [("S", 1)], [1], [1030, 1])]  # 4.6 M, padded rows (stride not a multiple of four)
    outside = [([1500, 4096], [3], [("S", 1)], [1]),         # 2.0 M: below the 16-bit window
               ([12000, 600], [3], [("S", 1)], [1]),         # 2.4 M but runs of 200: too short for the 16-bit fills
               ([2 ** 14, 4100], [3], [("S", 1)], [1])]      # 22 M: above the fp32 normal window, inside the 16-bit one
    for args in inside + outside:
        say("staged fills %s" % (args,))
        for dtype, code in (("bf16", oracle.BF16), ("f16", oracle.F16)):
            got = gpu_fill("uniform", dtype, args, seed, offset, low=-1.0, high=1.0)
            want = oracle.uniform(args, code, -1.0, 1.0, seed, offset, threads=THREADS)
            assert np.array_equal(got, want), (args, dtype)
            got = gpu_fill("normal", dtype, args, seed, offset, mean=0.5, std=2.0)
            check_normal(got, args, dtype, 0.5, 2.0, seed, offset, "normal %s %s" % (dtype, args))
        got = gpu_fill("normal", "f32", args, seed, offset, mean=-1.0, std=0.5)
        check_normal(got, args, "f32", -1.0, 0.5, seed, offset, "normal f32 %s" % (args,))
        del got, want


def test_f16_dropout_and_residual_add_all_kernel_flavours():
    seed, offset = 2025, 64
    for k, args in enumerate(F16_CASES):
        say("f16 dropout %s" % (args,))
        sh = v.Sharding(*args)
        lshape, n = v.vesrng_local_shape(sh)
        with np.errstate(over="ignore"):
            x = W.f16_bits_from_f32(W.adversarial_f32(n, seed=10 + k) * np.float32(3.0))
        r = W.f16_bits_from_f32(W.adversarial_f32(n, seed=20 + k))
        for p in (0.1, 0.0, 1.0, 0.5):
            yo, mo = oracle.dropout(args, oracle.F16, p, seed, offset, x)
            y, m = gpu_dropout("f16", args, p, seed, offset, x)
            assert np.array_equal(m, mo), (args, p)
            assert_float_bits_equal(y, yo, "dropout f16 %s p=%g" % (args, p), dtype="f16")
            y2, _ = gpu_dropout("f16", args, p, seed, offset, x, with_mask=False, in_place=True)
            assert_float_bits_equal(y2, yo, "dropout f16 in place %s p=%g" % (args, p), dtype="f16")
        yo, mo = oracle.dropout_add(args, oracle.F16, 0.1, seed, offset, x, r)
        xd, rd = to_device(x, "f16"), to_device(r, "f16")
        yd = torch.empty_like(xd)
        m = torch.empty(max(n, 1), dtype=torch.uint8, device=DEV)
        v.vesrng_dropout_add(sh, v.F16, 0.1, seed, offset, xd, rd, yd, m)
        torch.cuda.synchronize()
        assert np.array_equal(m.cpu().numpy()[:n].reshape(lshape), mo), args
        assert_float_bits_equal(to_host(yd, "f16")[:n].reshape(lshape), yo, "dropout_add f16 %s" % (args,), dtype="f16")
    # Overflow on the way out is IEEE's: 60000 * 1.25 rounds to infinity on both sides.
    flat = ([64], [1], [("R",)], [0])
    x = W.f16_bits_from_f32(np.full(64, 60000.0, dtype=np.float32))
    y, m = gpu_dropout("f16", flat, 0.2, 1, 0, x)
    assert set(np.unique(y).tolist()) == {0, 0x7C00} and np.array_equal(y, oracle.dropout(flat, oracle.F16, 0.2, 1, 0, x)[0])


def test_concurrent_host_threads_on_their_own_streams():
    """The library keeps no state between calls: four host threads issue different operators on
    their own streams at the same time (ctypes drops the GIL for the call) and every result is
    the one a lone call gives."""
    import threading
    jobs = [("raw", None, ([333, 517], [3], [("S", 1)], [1]), {}),
            ("uniform", "bf16", ([64, 4096], [4], [("S", 0)], [2]), {}),
            ("normal", "f32", ([5, 6, 7, 8, 9], [2, 2], [("S", 1), ("S", 3)], [1, 1]), {"mean": 1.0, "std": 2.0}),
            ("uniform", "f16", ([96, 40], [2, 3], [("IS", 0, 2), ("S", 0)], [1, 1]), {"low": -1.0, "high": 1.0})]
    alone = [gpu_fill(op, dt, args, 31, 64, **kw) for op, dt, args, kw in jobs]
    results, errors = [None] * len(jobs), []

    def work(k):
        try:
            op, dt, args, kw = jobs[k]
            sh = v.Sharding(*args)
            n = v.vesrng_local_shape(sh)[1]
            stream = torch.cuda.Stream()
            tdt = torch.int32 if op == "raw" else DT[dt][0]
            outs = [torch.empty(n, dtype=tdt, device=DEV) for _ in range(50)]
            for out in outs:
                if op == "raw":
                    v.vesrng_raw_u32(sh, 31, 64, out, stream=stream)
                elif op == "uniform":
                    v.vesrng_uniform(sh, DT[dt][1], kw.get("low", 0.0), kw.get("high", 1.0), 31, 64, out, stream=stream)
                else:
                    v.vesrng_normal(sh, DT[dt][1], kw["mean"], kw["std"], 31, 64, out, stream=stream)
            stream.synchronize()
            results[k] = [o.view(torch.int16 if o.element_size() == 2 else torch.int32).cpu().numpy() for o in outs]
        except Exception as e:  # noqa: BLE001 - reported below, in the main thread
            errors.append((k, repr(e)))

    threads = [threading.Thread(target=work, args=(k,)) for k in range(len(jobs))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for k, want in enumerate(alone):
        for got in results[k]:
            assert got.tobytes() == want.tobytes(), jobs[k]


def test_generator_sequence_of_operators_matches_one_device_doing_the_same_sequence():
    """RNG-state progression over several operators: every rank of a 2 x 2 mesh runs the same
    sequence of calls on differently sharded tensors with its own Generator; each shard equals the
    oracle at the offset the sequence has reached, all ranks end on the same offset, and the merged
    shards equal what ONE device produces with the same sequence on the unsharded tensors."""
    mesh = [2, 2]
    seq = [("uniform", "f32", [64, 48], [("S", 0), ("S", 1)]),
           ("normal", "bf16", [33, 50], [("S", 1), ("R",)]),
           ("randint", None, [7, 5, 6], [("R",), ("S", 2)]),
           ("dropout", "f16", [40, 24], [("S", 0), ("S", 0)]),
           ("raw", None, [96], [("IS", 0, 2), ("S", 0)])]
    x_global = {k: W.f16_bits_from_f32(np.random.default_rng(k).standard_normal(int(np.prod(s[2])), dtype=np.float32)
                                       ).reshape(s[2]) for k, s in enumerate(seq) if s[0] == "dropout"}

    def run(mesh_shape, placements_of, coord):
        g = v.Generator(seed=2468, offset=16)
        outs, offsets = [], []
        for k, (op, dt, shape, pls) in enumerate(seq):
            args = (shape, mesh_shape, placements_of(pls), list(coord))
            sh = v.Sharding(*args)
            lshape, n = v.vesrng_local_shape(sh)
            offsets.append(g.offset)
            if op == "raw":
                out = torch.empty(max(n, 1), dtype=torch.int32, device=DEV)
                g.raw_u32_(sh, out)
                res = out.cpu().numpy().view(np.uint32)
            elif op == "randint":
                out = torch.empty(max(n, 1), dtype=torch.int64, device=DEV)
                g.randint_(sh, out, -5, 1000)
                res = out.cpu().numpy()
            elif op == "dropout":
                idx = oracle.global_indices(*args).reshape(-1)
                xs = x_global[k].reshape(-1)[idx.astype(np.int64)] if n else np.zeros(1, np.uint16)
                xd = to_device(xs, dt)
                y = torch.empty_like(xd)
                g.dropout(sh, DT[dt][1], 0.25, xd, y, None)
                res = to_host(y, dt)
            else:
                out = torch.empty(max(n, 1), dtype=DT[dt][0], device=DEV)
                if op == "uniform":
                    g.uniform_(sh, DT[dt][1], out, -1.0, 1.0)
                else:
                    g.normal_(sh, DT[dt][1], out, 0.5, 2.0)
                res = to_host(out, dt)
            torch.cuda.synchronize()
            outs.append((res[:n].reshape(lshape), args))
        return outs, offsets, g.offset

    single, offs1, end1 = run([1], lambda pls: [("R",)], (0,))
    per_rank = {c: run(mesh, lambda pls: pls, c) for c in mesh_coords(mesh)}
    assert all(r[1] == offs1 and r[2] == end1 for r in per_rank.values())        # lockstep, no exchange
    assert end1 == 16 + sum(4 * ((int(np.prod(s[2])) + 3) // 4) for s in seq)
    for k, (op, dt, shape, pls) in enumerate(seq):
        shards = {c: per_rank[c][0][k][0] for c in per_rank}
        if op == "normal":   # the GPU's own normals are the same function of the global index on every shard
            assert merge_shards(shards, mesh, pls).tobytes() == single[k][0].tobytes(), seq[k]
            check_normal(single[k][0], single[k][1], dt, 0.5, 2.0, 2468, offs1[k], str(seq[k]))
            continue
        assert merge_shards(shards, mesh, pls).tobytes() == single[k][0].tobytes(), seq[k]
        args = single[k][1]
        if op == "uniform":
            want = oracle.uniform(args, oracle.F32, -1.0, 1.0, 2468, offs1[k])
            assert np.array_equal(single[k][0].view(np.uint32), want.view(np.uint32))
        elif op == "randint":
            assert np.array_equal(single[k][0], oracle.randint(args, -5, 1000, 2468, offs1[k]))
        elif op == "raw":
            assert np.array_equal(single[k][0], oracle.raw_u32(args, 2468, offs1[k]))
        else:
            want = oracle.dropout(args, oracle.F16, 0.25, 2468, offs1[k], x_global[k].reshape(-1))[0]
            assert_float_bits_equal(single[k][0], want, str(seq[k]), dtype="f16")


def test_large_ragged_fp32_fills():
    """Ragged column shards big enough (2^22 elements and more) to take the large-tile form of the staging
    kernel - raw and uniform fp32 - and the fp32 normal fill on a shard of 2^26 elements, where it takes the kernel
    without staging, against the threaded oracle, with the rows' phases equal (row length 4100) and unequal (4101)."""
    seed, offset = 31337, 1 << 33
    for cols in (4100, 4101):
        args = ([16384, cols], [3], [("S", 1)], [1])
        n = oracle.local_shape(*args)[1]
        assert n >= 1 << 24
        say("large ragged %s" % (args,))
        got = gpu_fill("raw", None, args, seed, offset)
        assert np.array_equal(got, oracle.raw_u32(args, seed, offset, threads=THREADS)), args
        for low, high in ((0.0, 1.0), (-2.0, 3.0)):
            got = gpu_fill("uniform", "f32", args, seed, offset, low=low, high=high)
            want = oracle.uniform(args, oracle.F32, low, high, seed, offset, threads=THREADS)
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (args, low, high)
        del got, want
        args = ([49152, cols], [3], [("S", 1)], [2])
        assert oracle.local_shape(*args)[1] >= 1 << 26
        say("large ragged %s" % (args,))
        got = gpu_fill("normal", "f32", args, seed, offset, mean=-1.0, std=3.0)
        check_normal(got, args, "f32", -1.0, 3.0, seed, offset, "normal f32 %s" % (args,))
        del got


def test_column_shards_whose_runs_share_one_phase():
    """Ragged shards with ONE axis of runs and a stride between runs that is a multiple of four (a column shard of
    a matrix whose row length is a multiple of four; rows of a padded tensor): the staging kernel takes the short
    form of its tile map.  Small tile and large tile, every operator that is staged, every phase, and strides
    that a run's generator blocks fill exactly (and overfill by one: the general form then serves)."""
    seed, offset = 8642, 1 << 34
    cases = [([1000, 1000], [3], [("S", 1)], [1]),                    # runs of 334 at phase 2
             ([513, 2048], [5], [("S", 1)], [3]),                     # runs of 410 at phase 2
             ([777, 404], [4], [("S", 1)], [3]),                      # runs of 101 at phase 3
             ([3000, 2, 17], [2], [("S", 1)], [1], [20, 3, 1]),       # stride 20 = 4 x (blocks per run): exact fit
             ([3000, 2, 18], [2], [("S", 1)], [1], [20, 3, 1]),       # one block more than the stride holds
             ([3000, 2, 19], [2], [("S", 1)], [1], [20, 1, 1]),       # phase 1
             ([5000, 1030], [1], [("R",)], [0], [1032, 1]),           # phase 0, ragged only at the run's end (large tile)
             ([5000, 1032], [2], [("S", 1)], [1])]                    # runs of 516 from column 516 (aligned: not staged)
    for args in cases:
        n = oracle.local_shape(*args[:4])[1]
        say("one-phase runs %s" % (args,))
        got = gpu_fill("raw", None, args, seed, offset)
        assert np.array_equal(got, oracle.raw_u32(args, seed, offset, threads=THREADS)), args
        got = gpu_fill("uniform", "f32", args, seed, offset, low=-1.0, high=2.0)
        want = oracle.uniform(args, oracle.F32, -1.0, 2.0, seed, offset, threads=THREADS)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), args
        got = gpu_fill("randint", None, args, seed, offset, low=-5, high=(1 << 32) - 5)
        assert np.array_equal(got, oracle.randint(args, -5, (1 << 32) - 5, seed, offset, threads=THREADS)), args
        xf = W.adversarial_f32(n, seed=11)
        for dtype, code in (("f32", oracle.F32), ("bf16", oracle.BF16), ("f16", oracle.F16)):
            x = xf if dtype == "f32" else (W.bf16_bits_from_f32(xf) if dtype == "bf16" else W.f16_bits_from_f32(xf))
            yo, mo = oracle.dropout(args, code, 0.3, seed, offset, x)
            y, m = gpu_dropout(dtype, args, 0.3, seed, offset, x)
            assert np.array_equal(m, mo), (args, dtype)
            assert_float_bits_equal(y, yo, "dropout %s %s" % (dtype, args), dtype=dtype)


def test_random_column_shards_through_the_staging_kernel():
    """Seeded random column shards (row counts, widths, row paddings that are and are not multiples of four, mesh
    sizes, ranks, offsets), sized to take the small tile, the large tile, the short and the general tile map:
    raw draws, the fp32 uniform fill, randint and bf16 dropout against the oracle."""
    rng = np.random.default_rng(424242)
    done = 0
    while done < 16:
        rows = int(rng.integers(200, 9000))
        cols = int(rng.integers(64, 3000))
        m = int(rng.integers(2, 5))
        coord = int(rng.integers(0, m))
        pad = int(rng.choice([0, 0, 1, 3, 4, 8]))
        if rng.random() < 0.5:
            pad = (-cols) % 4 + 4 * int(rng.integers(0, 2))     # a row stride that is a multiple of four
        chunk = -(-cols // m)
        w = min(chunk, cols - coord * chunk)
        if w < 16 or ((coord * chunk) % 4 == 0 and (cols + pad) % 4 == 0 and w % 8 == 0):
            continue
        args = ([rows, cols], [m], [("S", 1)], [coord]) + (([cols + pad, 1],) if pad else ())
        seed, offset = int(rng.integers(0, 1 << 62)), 4 * int(rng.integers(0, 1 << 40))
        n = rows * w
        say("random column shard %s, %d elements" % (args, n))
        got = gpu_fill("raw", None, args, seed, offset)
        assert np.array_equal(got, oracle.raw_u32(args, seed, offset, threads=THREADS)), args
        got = gpu_fill("uniform", "f32", args, seed, offset, low=-3.0, high=0.5)
        want = oracle.uniform(args, oracle.F32, -3.0, 0.5, seed, offset, threads=THREADS)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), args
        got = gpu_fill("randint", None, args, seed, offset, low=10, high=1 << 20)
        assert np.array_equal(got, oracle.randint(args, 10, 1 << 20, seed, offset, threads=THREADS)), args
        x = W.bf16_bits_from_f32(W.adversarial_f32(n, seed=done))
        yo, mo = oracle.dropout(args, oracle.BF16, 0.45, seed, offset, x, threads=THREADS)
        y, mk = gpu_dropout("bf16", args, 0.45, seed, offset, x)
        assert np.array_equal(mk, mo), args
        assert_float_bits_equal(y, yo, "dropout bf16 %s" % (args,))
        done += 1


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_contiguous_shards_of_any_length(dtype):
    """A shard that is one contiguous run takes the vector kernel whatever its length; the last,
    partial unit is finished element by element.  Unsharded tensors and row shards of odd sizes,
    every floating-point operator."""
    seed, offset = 555, 40
    cases = [([n], [1], [("R",)], [0]) for n in (1, 2, 3, 5, 7, 9, 15, 17, 1001, 65543)]
    cases += [([7, 11, 13], [1], [("R",)], [0]), ([9, 1001], [2], [("S", 0)], [1]), ([5, 3, 7], [3], [("S", 0)], [2])]
    for args in cases:
        n = oracle.local_shape(*args)[1]
        got = gpu_fill("uniform", dtype, args, seed, offset, low=-1.0, high=2.0)
        want = oracle.uniform(args, DT[dtype][2], -1.0, 2.0, seed, offset)
        assert_float_bits_equal(got, want, "uniform %s %s" % (dtype, args), dtype=dtype)
        got = gpu_fill("normal", dtype, args, seed, offset, mean=1.0, std=0.5)
        check_normal(got, args, dtype, 1.0, 0.5, seed, offset, "normal %s %s" % (dtype, args))
        xf = W.adversarial_f32(n, seed=n)
        x = xf if dtype == "f32" else W.bits16_from_f32(xf, dtype)
        yo, mo = oracle.dropout(args, DT[dtype][2], 0.3, seed, offset, x)
        y, m = gpu_dropout(dtype, args, 0.3, seed, offset, x)
        assert np.array_equal(m, mo), (dtype, args)
        assert_float_bits_equal(y, yo, "dropout %s %s" % (dtype, args), dtype=dtype)
        y, _ = gpu_dropout(dtype, args, 0.3, seed, offset, x, with_mask=False, in_place=True)
        assert_float_bits_equal(y, yo, "dropout in place %s %s" % (dtype, args), dtype=dtype)
        r = xf[::-1].copy() if dtype == "f32" else W.bits16_from_f32(xf[::-1].copy(), dtype)
        yo, mo = oracle.dropout_add(args, DT[dtype][2], 0.3, seed, offset, x, r)
        sh = v.Sharding(*args)
        xd, rd = to_device(x, dtype), to_device(r, dtype)
        yd = torch.empty_like(xd)
        md = torch.empty(n, dtype=torch.uint8, device=DEV)
        v.vesrng_dropout_add(sh, DT[dtype][1], 0.3, seed, offset, xd, rd, yd, md)
        torch.cuda.synchronize()
        assert np.array_equal(md.cpu().numpy().reshape(mo.shape), mo), (dtype, args)
        assert_float_bits_equal(to_host(yd, dtype).reshape(yo.shape), yo, "dropout_add %s %s" % (dtype, args), dtype=dtype)


def test_bench_line_keeps_its_contract():
    """bench.py on this GPU, shortened: ONE JSON line with the keys the benchmark contract names, the roofline and
    CPU-baseline objects included, and a throughput that is neither above the HBM peak nor implausibly low."""
    import json
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--steps", "5", "--warmup", "2", "--no-extra"],
                         stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=240)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2 and d["vs_baseline"] is None and d["unit"] == "GB/s"
    assert d["config"]["workload"].startswith("C5") and d["config"]["settle_seconds"] >= 0.25
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s" and abs(r["frac"] - r["achieved"] / 8000.0) < 1e-9
    assert r["algorithmic_bytes_per_launch"] == 5 * d["config"]["elements"] and r["traffic"] is not None
    assert 0.9 < r["traffic"] / r["algorithmic_bytes_per_launch"] < 1.1
    assert 3000.0 < d["value"] < 8000.0 and 3000.0 < r["achieved"] < 8000.0
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["unit"] == "GB/s" and c["cores"] >= 1 and c["value"] > 0 and c["sample"]
