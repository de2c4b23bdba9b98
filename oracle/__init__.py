"""ctypes front end of the CPU oracle.

TEST INFRASTRUCTURE ONLY.  The oracle is the plain definition of what the sharded
random-number path computes (Section 5 and Algorithm 1 of the paper, with
Philox4x32-10 as the value generator).  Only tests/, __graft_entry__.smoke() and
bench.py's cpu_baseline leg may import this package; the product never does.

A sharding is described with plain Python values:
  global_shape  list of ints
  mesh_shape    list of ints
  placements    one per mesh dimension: ("R",), ("S", dim) or ("IS", dim, groups)
  mesh_coord    list of ints, this rank's coordinate in the mesh
  global_stride optional list of ints (elements); None = row-major contiguous
  virtual_threads optional int: Algorithm 1's global thread count; 0 = one flat stream
A "sharding" argument of the bulk functions is the tuple
(global_shape, mesh_shape, placements, mesh_coord[, global_stride[, virtual_threads]]).
bfloat16 data travels as numpy uint16 bit patterns.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

F32, BF16, F16 = 0, 1, 2
_KIND = {"R": 0, "S": 1, "IS": 2}
_lib = None


class _Flat(C.Structure):
    _fields_ = [("ndim", C.c_int32), ("global_shape", C.POINTER(C.c_int64)),
                ("global_stride", C.POINTER(C.c_int64)), ("mesh_ndim", C.c_int32),
                ("mesh_shape", C.POINTER(C.c_int32)), ("kind", C.POINTER(C.c_int32)),
                ("dim", C.POINTER(C.c_int32)), ("interleave", C.POINTER(C.c_int32)),
                ("mesh_coord", C.POINTER(C.c_int32)), ("virtual_threads", C.c_uint64)]


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build.ensure())   # rebuilt first when missing or older than its sources
        L.oracle_draw.restype = C.c_uint32
        L.oracle_draw.argtypes = [C.c_uint64, C.c_uint64]
        L.oracle_uniform_f32.restype = C.c_float
        L.oracle_uniform_f32.argtypes = [C.c_uint32, C.c_float, C.c_float]
        L.oracle_uniform_bf16.restype = C.c_uint16
        L.oracle_uniform_bf16.argtypes = [C.c_uint32, C.c_float, C.c_float]
        L.oracle_normal_f64.restype = C.c_double
        L.oracle_normal_f64.argtypes = [C.c_uint32, C.c_uint32, C.c_int, C.c_double, C.c_double]
        L.oracle_dropout_threshold.restype = C.c_uint32
        L.oracle_dropout_threshold.argtypes = [C.c_double]
        L.oracle_dropout_scale.restype = C.c_float
        L.oracle_dropout_scale.argtypes = [C.c_double]
        L.oracle_bf16_from_double.restype = C.c_uint16
        L.oracle_bf16_from_double.argtypes = [C.c_double]
        L.oracle_bf16_from_float.restype = C.c_uint16
        L.oracle_bf16_from_float.argtypes = [C.c_float]
        L.oracle_float_from_bf16.restype = C.c_float
        L.oracle_float_from_bf16.argtypes = [C.c_uint16]
        L.oracle_uniform_f16.restype = C.c_uint16
        L.oracle_uniform_f16.argtypes = [C.c_uint32, C.c_float, C.c_float]
        L.oracle_f16_from_double.restype = C.c_uint16
        L.oracle_f16_from_double.argtypes = [C.c_double]
        L.oracle_double_from_f16.restype = C.c_double
        L.oracle_double_from_f16.argtypes = [C.c_uint16]
        L.oracle_advance_offset.restype = C.c_uint64
        L.oracle_advance_offset.argtypes = [C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.c_int32, C.c_uint64,
                                            C.c_uint64]
        _lib = L
    return _lib


class OracleError(ValueError):
    pass


def _flat(global_shape, mesh_shape, placements, mesh_coord, global_stride=None, virtual_threads=0):
    nd, md = len(global_shape), len(mesh_shape)
    keep = []

    def arr(ctype, values):
        a = (ctype * max(1, len(values)))(*values)
        keep.append(a)
        return a

    kinds, dims, inter = [], [], []
    for p in placements:
        if p[0] not in _KIND:
            kinds.append(99)  # e.g. "P" (Partial): the oracle rejects it
        else:
            kinds.append(_KIND[p[0]])
        dims.append(p[1] if len(p) > 1 else 0)
        inter.append(p[2] if len(p) > 2 else 1)
    f = _Flat(nd, arr(C.c_int64, list(global_shape)),
              arr(C.c_int64, list(global_stride)) if global_stride is not None else None,
              md, arr(C.c_int32, list(mesh_shape)), arr(C.c_int32, kinds), arr(C.c_int32, dims),
              arr(C.c_int32, inter), arr(C.c_int32, list(mesh_coord)), virtual_threads)
    return f, keep


def _call(fn, *args):
    err = C.create_string_buffer(256)
    rc = fn(*args, err, 256)
    if rc != 0:
        raise OracleError(err.value.decode())


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*ctr)
    k = (C.c_uint32 * 2)(*key)
    o = (C.c_uint32 * 4)()
    lib().oracle_philox4x32_10(c, k, o)
    return list(o)


def draw(seed, position):
    return lib().oracle_draw(seed, position)


def uniform_f32(x, low=0.0, high=1.0):
    return lib().oracle_uniform_f32(x, low, high)


def uniform_bf16(x, low=0.0, high=1.0):
    return lib().oracle_uniform_bf16(x, low, high)


def normal_f64(xa, xb, odd, mean=0.0, std=1.0):
    return lib().oracle_normal_f64(xa, xb, int(odd), mean, std)


def dropout_threshold(p):
    return lib().oracle_dropout_threshold(p)


def dropout_scale(p):
    return lib().oracle_dropout_scale(p)


def bf16_from_double(v):
    return lib().oracle_bf16_from_double(v)


def bf16_from_float(v):
    return lib().oracle_bf16_from_float(v)


def float_from_bf16(h):
    return lib().oracle_float_from_bf16(h)


def uniform_f16(x, low=0.0, high=1.0):
    return lib().oracle_uniform_f16(x, low, high)


def f16_from_double(v):
    return lib().oracle_f16_from_double(v)


def double_from_f16(h):
    return lib().oracle_double_from_f16(h)


def local_shape(global_shape, mesh_shape, placements, mesh_coord):
    f, _k = _flat(global_shape, mesh_shape, placements, mesh_coord)
    shp = (C.c_int64 * max(1, len(global_shape)))()
    n = C.c_int64()
    _call(lib().oracle_local_shape, C.byref(f), shp, C.byref(n))
    return list(shp)[:len(global_shape)], n.value


def index_list(global_shape, mesh_shape, placements, mesh_coord, dim):
    shp, _ = local_shape(global_shape, mesh_shape, placements, mesh_coord)
    f, _k = _flat(global_shape, mesh_shape, placements, mesh_coord)
    out = np.zeros(max(1, shp[dim]), dtype=np.int64)
    _call(lib().oracle_index_list, C.byref(f), C.c_int32(dim), _ptr(out))
    return out[:shp[dim]]


def global_indices(global_shape, mesh_shape, placements, mesh_coord, global_stride=None):
    shp, n = local_shape(global_shape, mesh_shape, placements, mesh_coord)
    f, _k = _flat(global_shape, mesh_shape, placements, mesh_coord, global_stride)
    out = np.zeros(max(1, n), dtype=np.uint64)
    _call(lib().oracle_global_indices, C.byref(f), _ptr(out))
    return out[:n].reshape(shp)


def _bulk(name, sharding, np_dtype, head_args, i_begin, i_end, threads, out=None):
    global_shape, mesh_shape, placements, mesh_coord = sharding[:4]
    stride = sharding[4] if len(sharding) > 4 else None
    theta = sharding[5] if len(sharding) > 5 else 0
    shp, n = local_shape(global_shape, mesh_shape, placements, mesh_coord)
    f, _k = _flat(global_shape, mesh_shape, placements, mesh_coord, stride, theta)
    if out is None:
        out = np.zeros(max(1, n), dtype=np_dtype)
    _call(getattr(lib(), name), C.byref(f), *head_args, _ptr(out), C.c_int64(i_begin),
          C.c_int64(i_end), C.c_int(threads))
    return out[:n].reshape(shp)


def raw_u32(sharding, seed, offset, i_begin=0, i_end=-1, threads=1):
    return _bulk("oracle_raw_u32", sharding, np.uint32, [C.c_uint64(seed), C.c_uint64(offset)],
                 i_begin, i_end, threads)


def uniform(sharding, dtype, low, high, seed, offset, i_begin=0, i_end=-1, threads=1):
    return _bulk("oracle_uniform", sharding, np.float32 if dtype == F32 else np.uint16,
                 [C.c_int32(dtype), C.c_double(low), C.c_double(high), C.c_uint64(seed),
                  C.c_uint64(offset)], i_begin, i_end, threads)


def normal(sharding, dtype, mean, std, seed, offset, i_begin=0, i_end=-1, threads=1):
    return _bulk("oracle_normal", sharding, np.float32 if dtype == F32 else np.uint16,
                 [C.c_int32(dtype), C.c_double(mean), C.c_double(std), C.c_uint64(seed),
                  C.c_uint64(offset)], i_begin, i_end, threads)


def normal_f64_values(sharding, mean, std, seed, offset, i_begin=0, i_end=-1, threads=1):
    return _bulk("oracle_normal_f64_values", sharding, np.float64,
                 [C.c_double(mean), C.c_double(std), C.c_uint64(seed), C.c_uint64(offset)],
                 i_begin, i_end, threads)


def randint(sharding, low, high, seed, offset, i_begin=0, i_end=-1, threads=1):
    return _bulk("oracle_randint", sharding, np.int64,
                 [C.c_int64(low), C.c_int64(high), C.c_uint64(seed), C.c_uint64(offset)],
                 i_begin, i_end, threads)


def dropout(sharding, dtype, p, seed, offset, x, i_begin=0, i_end=-1, threads=1, want_mask=True):
    """x: flat or shaped numpy array of the local shard (float32, or uint16 bf16 bits).
    Returns (y, mask); elements outside [i_begin, i_end) are left zero."""
    global_shape, mesh_shape, placements, mesh_coord = sharding[:4]
    stride = sharding[4] if len(sharding) > 4 else None
    theta = sharding[5] if len(sharding) > 5 else 0
    shp, n = local_shape(global_shape, mesh_shape, placements, mesh_coord)
    npdt = np.float32 if dtype == F32 else np.uint16
    x = np.ascontiguousarray(x, dtype=npdt).reshape(-1)
    if x.size != n:
        raise OracleError("x must hold exactly the local shard")
    f, _k = _flat(global_shape, mesh_shape, placements, mesh_coord, stride, theta)
    y = np.zeros(max(1, n), dtype=npdt)
    mask = np.zeros(max(1, n), dtype=np.uint8) if want_mask else None
    xs = x if x.size else np.zeros(1, dtype=npdt)
    _call(lib().oracle_dropout, C.byref(f), C.c_int32(dtype), C.c_double(p), C.c_uint64(seed),
          C.c_uint64(offset), _ptr(xs), _ptr(y), _ptr(mask) if want_mask else None,
          C.c_int64(i_begin), C.c_int64(i_end), C.c_int(threads))
    return y[:n].reshape(shp), (mask[:n].reshape(shp) if want_mask else None)


def dropout_add(sharding, dtype, p, seed, offset, x, residual, threads=1):
    """y = residual + dropout(x) with one rounding to the dtype at the end.  Returns (y, mask)."""
    global_shape, mesh_shape, placements, mesh_coord = sharding[:4]
    stride = sharding[4] if len(sharding) > 4 else None
    theta = sharding[5] if len(sharding) > 5 else 0
    shp, n = local_shape(global_shape, mesh_shape, placements, mesh_coord)
    npdt = np.float32 if dtype == F32 else np.uint16
    x = np.ascontiguousarray(x, dtype=npdt).reshape(-1)
    residual = np.ascontiguousarray(residual, dtype=npdt).reshape(-1)
    if x.size != n or residual.size != n:
        raise OracleError("x and residual must hold exactly the local shard")
    f, _k = _flat(global_shape, mesh_shape, placements, mesh_coord, stride, theta)
    y = np.zeros(max(1, n), dtype=npdt)
    mask = np.zeros(max(1, n), dtype=np.uint8)
    pad = np.zeros(1, dtype=npdt)
    _call(lib().oracle_dropout_add, C.byref(f), C.c_int32(dtype), C.c_double(p), C.c_uint64(seed),
          C.c_uint64(offset), _ptr(x if n else pad), _ptr(residual if n else pad), _ptr(y), _ptr(mask),
          C.c_int64(0), C.c_int64(-1), C.c_int(threads))
    return y[:n].reshape(shp), mask[:n].reshape(shp)


def advance_offset(global_shape, offset, global_stride=None, virtual_threads=0):
    a = (C.c_int64 * max(1, len(global_shape)))(*global_shape)
    st = None if global_stride is None else (C.c_int64 * max(1, len(global_shape)))(*global_stride)
    return lib().oracle_advance_offset(a, st, len(global_shape), offset, virtual_threads)
