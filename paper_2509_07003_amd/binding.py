"""Argument marshalling for the C ABI in include/vesrng.h: nothing is computed here.

Device buffers may be passed as torch tensors (their data_ptr() is used) or as integer
device addresses; `stream` may be a torch.cuda.Stream, an integer hipStream_t or None
(None = torch's current stream when a tensor was passed, else the default stream).
There is no CPU fallback: if libvesrng.so cannot be built or loaded, importing fails.
"""
import ctypes as C
import os

from . import build as _build

F32, BF16, F16 = 0, 1, 2
_KIND = {"R": 0, "S": 1, "IS": 2, "P": 3}


class _Placement(C.Structure):
    _fields_ = [("kind", C.c_int32), ("dim", C.c_int32), ("interleave", C.c_int32)]


class _Sharding(C.Structure):
    _fields_ = [("ndim", C.c_int32), ("global_shape", C.POINTER(C.c_int64)),
                ("global_stride", C.POINTER(C.c_int64)), ("mesh_ndim", C.c_int32),
                ("mesh_shape", C.POINTER(C.c_int32)), ("placements", C.POINTER(_Placement)),
                ("mesh_coord", C.POINTER(C.c_int32)), ("virtual_threads", C.c_uint64)]


def library_path():
    return _build.lib_path("vesrng")


class VesrngError(RuntimeError):
    def __init__(self, status):
        self.status = status
        super().__init__("vesrng status %d: %s" % (status, vesrng_status_string(status)))


def _check(status):
    if status != 0:
        raise VesrngError(status)


def _signatures():
    st, vp, u64, i64, dbl, i32 = C.c_int, C.c_void_p, C.c_uint64, C.c_int64, C.c_double, C.c_int32
    sp = C.POINTER(_Sharding)
    return {
        "vesrng_local_shape": [sp, C.POINTER(i64), C.POINTER(i64)],
        "vesrng_advance_offset": [sp, u64, C.POINTER(u64)],
        "vesrng_global_index": [sp, i64, C.POINTER(i64), C.POINTER(u64)],
        "vesrng_global_index_general": [sp, i64, C.POINTER(i64), C.POINTER(u64)],
        "vesrng_raw_u32": [sp, u64, u64, vp, vp],
        "vesrng_uniform": [sp, i32, dbl, dbl, u64, u64, vp, vp],
        "vesrng_normal": [sp, i32, dbl, dbl, u64, u64, vp, vp],
        "vesrng_dropout": [sp, i32, dbl, u64, u64, vp, vp, vp, vp],
        "vesrng_dropout_add": [sp, i32, dbl, u64, u64, vp, vp, vp, vp, vp],
        "vesrng_randint": [sp, i64, i64, u64, u64, vp, vp],
    }


EXPORTS = sorted(list(_signatures()) + ["vesrng_status_string"])


def load_library(path):
    """ctypes handle of a library with the C ABI of include/vesrng.h, argument types declared."""
    lib = C.CDLL(path)
    for name, args in _signatures().items():
        fn = getattr(lib, name)
        fn.restype = C.c_int
        fn.argtypes = args
    lib.vesrng_status_string.restype = C.c_char_p
    lib.vesrng_status_string.argtypes = [C.c_int]
    return lib


# Missing, or built from other sources than the ones present: rebuilt here; if that fails the
# import fails.  There is nothing to fall back to.
_lib = load_library(_build.ensure("vesrng"))


def vesrng_status_string(status):
    return _lib.vesrng_status_string(status).decode()


class Sharding:
    """Host-side description: global shape, mesh shape, one placement per mesh dimension
    (("R",), ("S", dim), ("IS", dim, groups) or ("P",)), the rank's mesh coordinate and
    optionally the global stride in elements and Algorithm 1's global thread count (0 = flat stream)."""

    def __init__(self, global_shape, mesh_shape=(), placements=(), mesh_coord=(), global_stride=None,
                 virtual_threads=0):
        self.global_shape = [int(v) for v in global_shape]
        self.mesh_shape = [int(v) for v in mesh_shape]
        self.placements = [tuple(p) for p in placements]
        self.mesh_coord = [int(v) for v in mesh_coord]
        self.global_stride = None if global_stride is None else [int(v) for v in global_stride]
        nd, md = len(self.global_shape), len(self.mesh_shape)
        if len(self.placements) != md or len(self.mesh_coord) != md:
            raise ValueError("one placement and one coordinate per mesh dimension")
        self._shape = (C.c_int64 * max(1, nd))(*self.global_shape)
        self._stride = None if self.global_stride is None else (C.c_int64 * max(1, nd))(*self.global_stride)
        self._mesh = (C.c_int32 * max(1, md))(*self.mesh_shape)
        self._coord = (C.c_int32 * max(1, md))(*self.mesh_coord)
        self._pl = (_Placement * max(1, md))()
        for m, p in enumerate(self.placements):
            self._pl[m] = _Placement(_KIND[p[0]], p[1] if len(p) > 1 else 0, p[2] if len(p) > 2 else 1)
        self.virtual_threads = int(virtual_threads)
        self.c = _Sharding(nd, self._shape, self._stride, md, self._mesh, self._pl, self._coord, self.virtual_threads)

    def with_coord(self, mesh_coord):
        return Sharding(self.global_shape, self.mesh_shape, self.placements, mesh_coord, self.global_stride,
                        self.virtual_threads)


def _dev(buf):
    if buf is None:
        return None
    if isinstance(buf, int):
        return C.c_void_p(buf)
    return C.c_void_p(buf.data_ptr())


def _current_stream(device_index):
    """torch's current stream on the device as a raw hipStream_t (the private accessor is several
    times cheaper than torch.cuda.current_stream(), which matters for microsecond kernels)."""
    import torch
    raw = getattr(torch._C, "_cuda_getCurrentRawStream", None)
    if raw is not None:
        return raw(device_index if device_index is not None else torch.cuda.current_device())
    return torch.cuda.current_stream(device_index).cuda_stream


def _stream(stream, *bufs):
    if stream is None:
        for b in bufs:
            if b is not None and not isinstance(b, int):
                return C.c_void_p(_current_stream(b.device.index))
        return None
    if isinstance(stream, int):
        return C.c_void_p(stream)
    return C.c_void_p(stream.cuda_stream)


def vesrng_local_shape(sharding):
    shape = (C.c_int64 * max(1, len(sharding.global_shape)))()
    numel = C.c_int64()
    _check(_lib.vesrng_local_shape(C.byref(sharding.c), shape, C.byref(numel)))
    return list(shape)[:len(sharding.global_shape)], numel.value


def vesrng_advance_offset(sharding, offset):
    new = C.c_uint64()
    _check(_lib.vesrng_advance_offset(C.byref(sharding.c), offset, C.byref(new)))
    return new.value


def vesrng_global_index(sharding, local_index):
    n = len(local_index)
    src = (C.c_int64 * max(1, n))(*[int(v) for v in local_index])
    dst = (C.c_uint64 * max(1, n))()
    _check(_lib.vesrng_global_index(C.byref(sharding.c), n, src, dst))
    return list(dst)[:n]


def vesrng_global_index_general(sharding, local_index):
    n = len(local_index)
    src = (C.c_int64 * max(1, n))(*[int(v) for v in local_index])
    dst = (C.c_uint64 * max(1, n))()
    _check(_lib.vesrng_global_index_general(C.byref(sharding.c), n, src, dst))
    return list(dst)[:n]


def vesrng_raw_u32(sharding, seed, offset, out, stream=None):
    _check(_lib.vesrng_raw_u32(C.byref(sharding.c), seed, offset, _dev(out), _stream(stream, out)))


def vesrng_uniform(sharding, dtype, low, high, seed, offset, out, stream=None):
    _check(_lib.vesrng_uniform(C.byref(sharding.c), dtype, low, high, seed, offset, _dev(out),
                               _stream(stream, out)))


def vesrng_normal(sharding, dtype, mean, std, seed, offset, out, stream=None):
    _check(_lib.vesrng_normal(C.byref(sharding.c), dtype, mean, std, seed, offset, _dev(out),
                              _stream(stream, out)))


def vesrng_dropout(sharding, dtype, p, seed, offset, x, y, mask=None, stream=None):
    _check(_lib.vesrng_dropout(C.byref(sharding.c), dtype, p, seed, offset, _dev(x), _dev(y), _dev(mask),
                               _stream(stream, x, y, mask)))


def vesrng_dropout_add(sharding, dtype, p, seed, offset, x, residual, y, mask=None, stream=None):
    _check(_lib.vesrng_dropout_add(C.byref(sharding.c), dtype, p, seed, offset, _dev(x), _dev(residual), _dev(y),
                                   _dev(mask), _stream(stream, x, residual, y, mask)))


def vesrng_randint(sharding, low, high, seed, offset, out, stream=None):
    _check(_lib.vesrng_randint(C.byref(sharding.c), low, high, seed, offset, _dev(out),
                               _stream(stream, out)))
