// Host-callable launchers of the gfx950 kernels.
#pragma once
#include <hip/hip_runtime_api.h>

#include <cstdint>

#include "geometry.hpp"

namespace vesrng {

enum OpKind : int32_t { kOpRaw = 0, kOpUniform = 1, kOpNormal = 2, kOpDropout = 3, kOpRandint = 4, kOpDropoutAdd = 5 };

// Everything an operator needs besides the index plan; passed by value.
struct OpParams {
  uint32_t key0 = 0, key1 = 0;  // seed, low and high word
  int32_t dtype = 0;            // vesrng_dtype of out / x / y
  // uniform: value = min(u * width + low, cap)
  float width = 1.f, low = 0.f;
  float cap = 1.f;              // largest value of the output dtype below high (high itself if high == low)
  uint32_t unit_range = 0;      // low == 0 and high == 1: the value is u itself
  // normal
  float mean = 0.f, stddev = 1.f;
  // dropout: keep = any && draw <= limit
  float scale = 1.f;
  uint32_t limit = 0;
  uint32_t keep_any = 1;
  // dropout + residual: y = residual + dropout(x); device pointer, same shape and dtype as x
  const void* residual = nullptr;
  // randint: out = base + draw mod range (range == 0 stands for 2^32)
  int64_t base = 0;
  uint32_t range = 0;
  uint32_t range_m = 0, range_s = 0;  // multiply-shift constants of the division by range
};

// Enqueues the kernel(s) that fill the rank's shard.  `x` and `mask` are used by
// dropout only (mask may be null).  Returns the HIP launch status.
hipError_t launch_op(OpKind op, const Geometry& g, uint64_t offset, const OpParams& prm,
                     const void* x, void* out, uint8_t* mask, hipStream_t stream);

}  // namespace vesrng
