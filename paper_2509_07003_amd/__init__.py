"""vesrng: single-device-semantic sharded random fills and fused dropout on MI355X.

Thin ctypes binding over libvesrng.so (hand-written HIP kernels + a C ABI declared in
include/vesrng.h).  PyTorch is used by callers for device memory and streams only.
"""
from .binding import (  # noqa: F401
    BF16, F16, F32, Sharding, VesrngError, library_path, vesrng_advance_offset, vesrng_dropout, vesrng_dropout_add,
    vesrng_global_index, vesrng_global_index_general, vesrng_local_shape, vesrng_normal, vesrng_randint, vesrng_raw_u32,
    vesrng_status_string, vesrng_uniform)
from .generator import Generator  # noqa: F401,E402
