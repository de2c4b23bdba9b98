"""Argument marshalling for the measurement aids of include/vesrng_bench.h (libvesrng_bench.so)
and for the design-choice variants of the library.  Only bench.py and its test import this
module; the product binding does not.  Nothing is computed here.
"""
import ctypes as C

from . import build as _build
from .binding import (BF16, F16, F32, Sharding, _check, _dev, _stream, load_library, vesrng_advance_offset,
                      vesrng_local_shape)

# vesrng_probe_kind
(PROBE_STORE, PROBE_COPY, PROBE_DROPOUT_TRAFFIC, PROBE_PHILOX, PROBE_STORE_NT, PROBE_STORE_PLAIN,
 PROBE_STORE_GRID_STRIDE, PROBE_STORE_UNALIGNED, PROBE_DROPOUT_TRAFFIC_NT, PROBE_PHILOX_TWO_XOR,
 PROBE_STORE_4_PER_THREAD, PROBE_DROPOUT_TRAFFIC_WIDE_MASK, PROBE_DROPOUT_TRAFFIC_LOAD_PLAIN,
 PROBE_DROPOUT_TRAFFIC_LOAD_SC1, PROBE_DROPOUT_TRAFFIC_LOAD_SC0SC1, PROBE_DROPOUT_TRAFFIC_7_WAVES,
 PROBE_DROPOUT_TRAFFIC_6_WAVES) = range(17)

# vesrng_alu_class, in the header's order
ALU_CLASSES = ["mad_u64_u32", "bitop3_b32", "add_u32", "fma_f32", "mul_f32", "cvt_f32_u32", "log_f32", "sqrt_f32",
               "sin_f32", "cos_f32", "cvt_pk_bf16_f32", "lshrrev_b32", "mul_lo_u32", "cmp_cndmask_b32"]

EXPORTS = ["vesrng_bench_alu", "vesrng_bench_clock", "vesrng_bench_device_info", "vesrng_bench_probe"]


def library_path():
    return _build.lib_path("bench")


def _load():
    lib = C.CDLL(_build.ensure("bench"))
    vp, u64, i32, u32 = C.c_void_p, C.c_uint64, C.c_int32, C.c_uint32
    lib.vesrng_bench_probe.argtypes = [i32, u64, vp, vp, vp, vp]
    lib.vesrng_bench_alu.argtypes = [i32, u32, u32, vp, vp]
    lib.vesrng_bench_clock.argtypes = [u32, vp, vp]
    lib.vesrng_bench_device_info.argtypes = [C.POINTER(i32)] * 5
    for name in EXPORTS:
        getattr(lib, name).restype = C.c_int
    return lib


_lib = _load()


def vesrng_bench_probe(kind, units, src, out, out2=None, stream=None):
    _check(_lib.vesrng_bench_probe(kind, units, _dev(src), _dev(out), _dev(out2), _stream(stream, src, out, out2)))


def vesrng_bench_alu(cls, workgroups, iters, out, stream=None):
    _check(_lib.vesrng_bench_alu(cls, workgroups, iters, _dev(out), _stream(stream, out)))


def vesrng_bench_clock(iters, out, stream=None):
    _check(_lib.vesrng_bench_clock(iters, _dev(out), _stream(stream, out)))


def vesrng_bench_device_info():
    """(compute units, shader clock kHz, memory clock kHz, memory bus bits, wall clock kHz) of the current device."""
    vals = [C.c_int32() for _ in range(5)]
    _check(_lib.vesrng_bench_device_info(*[C.byref(x) for x in vals]))
    return tuple(x.value for x in vals)


class Variant:
    """The library's fill and dropout entry points from one of the design-choice variant builds
    (same C ABI, one choice flipped; see build.TARGETS)."""

    def __init__(self, name):
        self.name = name
        self._lib = load_library(_build.ensure("variant_" + name))

    # What make_launcher-style callers need from the product binding, so that a variant can stand in for it.
    Sharding = Sharding
    F32, BF16, F16 = F32, BF16, F16

    def vesrng_local_shape(self, sharding):
        return vesrng_local_shape(sharding)

    def vesrng_advance_offset(self, sharding, offset):
        return vesrng_advance_offset(sharding, offset)

    def vesrng_raw_u32(self, sharding, seed, offset, out, stream=None):
        _check(self._lib.vesrng_raw_u32(C.byref(sharding.c), seed, offset, _dev(out), _stream(stream, out)))

    def vesrng_uniform(self, sharding, dtype, low, high, seed, offset, out, stream=None):
        _check(self._lib.vesrng_uniform(C.byref(sharding.c), dtype, low, high, seed, offset, _dev(out),
                                        _stream(stream, out)))

    def vesrng_normal(self, sharding, dtype, mean, std, seed, offset, out, stream=None):
        _check(self._lib.vesrng_normal(C.byref(sharding.c), dtype, mean, std, seed, offset, _dev(out),
                                       _stream(stream, out)))

    def vesrng_dropout(self, sharding, dtype, p, seed, offset, x, y, mask=None, stream=None):
        _check(self._lib.vesrng_dropout(C.byref(sharding.c), dtype, p, seed, offset, _dev(x), _dev(y), _dev(mask),
                                        _stream(stream, x, y, mask)))

    def vesrng_randint(self, sharding, low, high, seed, offset, out, stream=None):
        _check(self._lib.vesrng_randint(C.byref(sharding.c), low, high, seed, offset, _dev(out), _stream(stream, out)))

    def vesrng_dropout_add(self, sharding, dtype, p, seed, offset, x, residual, y, mask=None, stream=None):
        _check(self._lib.vesrng_dropout_add(C.byref(sharding.c), dtype, p, seed, offset, _dev(x), _dev(residual),
                                            _dev(y), _dev(mask), _stream(stream, x, residual, y, mask)))
