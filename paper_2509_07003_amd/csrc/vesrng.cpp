// C ABI of the library, the entry points that enqueue kernels: argument checking and
// marshalling only; every step of the path (index decode, generator, conversion, stores)
// runs in the kernels.  The host-only entry points are in host_api.cpp.
#include "../../include/vesrng.h"

#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstring>
#include <limits>

#include "build_id.h"
#include "geometry.hpp"
#include "launch.hpp"

using namespace vesrng;

namespace {

bool misaligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

uint32_t f32_bits(float f) {
  uint32_t b;
  std::memcpy(&b, &f, sizeof b);
  return b;
}
float f32_from_bits(uint32_t b) {
  float f;
  std::memcpy(&f, &b, sizeof f);
  return f;
}

// fp32 -> bfloat16, round to nearest even (finite inputs).
uint32_t bf16_rne(float f) {
  const uint32_t b = f32_bits(f);
  return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}
float bf16_value(uint32_t h) { return f32_from_bits(h << 16); }

// fp32 -> IEEE binary16, round to nearest even (finite inputs; 65520 and above become infinity).
uint32_t f16_rne(float f) {
  const uint32_t b = f32_bits(f), sign = (b >> 16) & 0x8000u, mag = b & 0x7FFFFFFFu;
  if (mag >= 0x47800000u) return sign | 0x7C00u;  // 2^16 and above
  if (mag < 0x38800000u)                          // below 2^-14: a multiple of 2^-24
    return sign | static_cast<uint32_t>(std::nearbyint(std::ldexp(static_cast<double>(std::fabs(f)), 24)));
  const uint32_t r = mag - (112u << 23);          // rebias the exponent from 127 to 15
  return sign | ((r + 0xFFFu + ((r >> 13) & 1u)) >> 13);
}
float f16_value(uint32_t h) {
  const int e = static_cast<int>((h >> 10) & 31u);
  const float m = static_cast<float>(h & 1023u);
  float mag;
  if (e == 31) mag = std::numeric_limits<float>::infinity();
  else if (e == 0) mag = std::ldexp(m, -24);
  else mag = std::ldexp(1024.0f + m, e - 25);
  return (h & 0x8000u) ? -mag : mag;
}

uint32_t round_16(vesrng_dtype dt, float f) { return (dt == VESRNG_F16 ? f16_rne(f) : bf16_rne(f)) & 0xFFFFu; }
float value_16(vesrng_dtype dt, uint32_t h) { return dt == VESRNG_F16 ? f16_value(h) : bf16_value(h); }

// Largest value of the 16-bit dtype strictly below `high` (bit pattern), high finite.  The
// patterns are sign-magnitude: one step down is -1 above zero and +1 below it.
uint32_t below_16(vesrng_dtype dt, float high) {
  uint32_t h = round_16(dt, high);
  if (value_16(dt, h) >= high) {
    const float t = value_16(dt, h);
    if (t > 0.0f) h -= 1;
    else if (t == 0.0f) h = 0x8001u;
    else h += 1;
  }
  return h & 0xFFFFu;
}

bool known_float_dtype(vesrng_dtype dt) { return dt == VESRNG_F32 || dt == VESRNG_BF16 || dt == VESRNG_F16; }

// Checks shared by every generating entry point; fills geometry and the seed.
vesrng_status prepare(const vesrng_sharding* s, uint64_t seed, uint64_t offset, Geometry* g, OpParams* prm) {
  const vesrng_status st = build_geometry(s, g);
  if (st != VESRNG_OK) return st;
  if (offset % 4 != 0) return VESRNG_ERR_OFFSET_ALIGN;
  // The last stream position the whole tensor uses must not wrap (with virtual threads the
  // positions are smaller still: offset + j / theta).
  if (g->global_numel != 0 && offset > std::numeric_limits<uint64_t>::max() - g->max_global_index - 4)
    return VESRNG_ERR_OVERFLOW;
  prm->key0 = static_cast<uint32_t>(seed);
  prm->key1 = static_cast<uint32_t>(seed >> 32);
  return VESRNG_OK;
}

vesrng_status finish(hipError_t e) { return e == hipSuccess ? VESRNG_OK : VESRNG_ERR_HIP; }

vesrng_status dropout_common(OpKind op, const vesrng_sharding* s, vesrng_dtype dtype, double p, uint64_t seed,
                             uint64_t offset, const void* x, const void* residual, void* y, uint8_t* mask,
                             void* hip_stream) {
  Geometry g;
  OpParams prm;
  const vesrng_status st = prepare(s, seed, offset, &g, &prm);
  if (st != VESRNG_OK) return st;
  if (!known_float_dtype(dtype)) return VESRNG_ERR_DTYPE;
  if (!(p >= 0.0 && p <= 1.0)) return VESRNG_ERR_BAD_PARAM;
  if (g.local_numel == 0) return VESRNG_OK;
  if (!x || !y || (op == kOpDropoutAdd && !residual)) return VESRNG_ERR_NULL;
  if (misaligned(x, 16) || misaligned(y, 16) || misaligned(mask, 16) || misaligned(residual, 16))
    return VESRNG_ERR_ALIGN;
  prm.dtype = dtype;
  prm.residual = residual;
  // keep = (draw >> 8) < T with T = round((1 - p) 2^24), i.e. draw <= (T << 8) - 1 for T >= 1.
  const uint64_t threshold = static_cast<uint64_t>(std::floor((1.0 - p) * 16777216.0 + 0.5));
  prm.keep_any = threshold != 0 ? 1u : 0u;
  prm.limit = threshold != 0 ? static_cast<uint32_t>((threshold << 8) - 1) : 0u;
  prm.scale = static_cast<float>(1.0 / (1.0 - p));
  return finish(launch_op(op, g, offset, prm, x, y, mask, static_cast<hipStream_t>(hip_stream)));
}

}  // namespace

extern "C" {

vesrng_status vesrng_raw_u32(const vesrng_sharding* s, uint64_t seed, uint64_t offset, uint32_t* out,
                             void* hip_stream) {
  Geometry g;
  OpParams prm;
  const vesrng_status st = prepare(s, seed, offset, &g, &prm);
  if (st != VESRNG_OK) return st;
  if (g.local_numel == 0) return VESRNG_OK;
  if (!out) return VESRNG_ERR_NULL;
  if (misaligned(out, 16)) return VESRNG_ERR_ALIGN;
  return finish(launch_op(kOpRaw, g, offset, prm, nullptr, out, nullptr, static_cast<hipStream_t>(hip_stream)));
}

vesrng_status vesrng_uniform(const vesrng_sharding* s, vesrng_dtype dtype, double low, double high,
                             uint64_t seed, uint64_t offset, void* out, void* hip_stream) {
  Geometry g;
  OpParams prm;
  const vesrng_status st = prepare(s, seed, offset, &g, &prm);
  if (st != VESRNG_OK) return st;
  if (!known_float_dtype(dtype)) return VESRNG_ERR_DTYPE;
  const float lo = static_cast<float>(low), hi = static_cast<float>(high);
  if (!(low <= high) || !std::isfinite(lo) || !std::isfinite(hi) || !std::isfinite(hi - lo))
    return VESRNG_ERR_BAD_PARAM;
  // binary16 has no finite value beyond +-65504: a wider range could not be honoured.
  if (dtype == VESRNG_F16 && (lo < -65504.0f || hi > 65504.0f)) return VESRNG_ERR_BAD_PARAM;
  if (g.local_numel == 0) return VESRNG_OK;
  if (!out) return VESRNG_ERR_NULL;
  if (misaligned(out, 16)) return VESRNG_ERR_ALIGN;
  prm.dtype = dtype;
  prm.low = lo;
  prm.width = hi - lo;
  prm.unit_range = (lo == 0.0f && hi == 1.0f) ? 1u : 0u;
  if (dtype == VESRNG_F32) prm.cap = hi > lo ? std::nextafterf(hi, lo) : hi;
  else prm.cap = hi > lo ? value_16(dtype, below_16(dtype, hi)) : hi;
  return finish(launch_op(kOpUniform, g, offset, prm, nullptr, out, nullptr, static_cast<hipStream_t>(hip_stream)));
}

vesrng_status vesrng_normal(const vesrng_sharding* s, vesrng_dtype dtype, double mean, double std,
                            uint64_t seed, uint64_t offset, void* out, void* hip_stream) {
  Geometry g;
  OpParams prm;
  const vesrng_status st = prepare(s, seed, offset, &g, &prm);
  if (st != VESRNG_OK) return st;
  if (!known_float_dtype(dtype)) return VESRNG_ERR_DTYPE;
  const float m = static_cast<float>(mean), sd = static_cast<float>(std);
  if (!(std >= 0.0) || !std::isfinite(m) || !std::isfinite(sd)) return VESRNG_ERR_BAD_PARAM;
  if (g.local_numel == 0) return VESRNG_OK;
  if (!out) return VESRNG_ERR_NULL;
  if (misaligned(out, 16)) return VESRNG_ERR_ALIGN;
  prm.dtype = dtype;
  prm.mean = m;
  prm.stddev = sd;
  return finish(launch_op(kOpNormal, g, offset, prm, nullptr, out, nullptr, static_cast<hipStream_t>(hip_stream)));
}

vesrng_status vesrng_dropout(const vesrng_sharding* s, vesrng_dtype dtype, double p, uint64_t seed,
                             uint64_t offset, const void* x, void* y, uint8_t* mask, void* hip_stream) {
  return dropout_common(kOpDropout, s, dtype, p, seed, offset, x, nullptr, y, mask, hip_stream);
}

vesrng_status vesrng_dropout_add(const vesrng_sharding* s, vesrng_dtype dtype, double p, uint64_t seed,
                                 uint64_t offset, const void* x, const void* residual, void* y, uint8_t* mask,
                                 void* hip_stream) {
  return dropout_common(kOpDropoutAdd, s, dtype, p, seed, offset, x, residual, y, mask, hip_stream);
}

vesrng_status vesrng_randint(const vesrng_sharding* s, int64_t low, int64_t high, uint64_t seed,
                             uint64_t offset, int64_t* out, void* hip_stream) {
  Geometry g;
  OpParams prm;
  const vesrng_status st = prepare(s, seed, offset, &g, &prm);
  if (st != VESRNG_OK) return st;
  if (high <= low) return VESRNG_ERR_BAD_PARAM;
  const uint64_t range = static_cast<uint64_t>(high) - static_cast<uint64_t>(low);
  if (range > (1ull << 32)) return VESRNG_ERR_BAD_PARAM;
  if (g.local_numel == 0) return VESRNG_OK;
  if (!out) return VESRNG_ERR_NULL;
  if (misaligned(out, 16)) return VESRNG_ERR_ALIGN;
  prm.base = low;
  prm.range = static_cast<uint32_t>(range);  // 2^32 -> 0
  if (prm.range != 0) {
    // q = floor(n / d) for any 32-bit n: s = ceil(log2 d), m = floor(2^32 (2^s - d) / d) + 1,
    // t = mulhi(n, m), q = (t + ((n - t) >> 1)) >> (s - 1); d = 1 is handled as s = 0.
    uint32_t sh = 0;
    while ((1ull << sh) < range) ++sh;
    prm.range_s = sh;
    prm.range_m = static_cast<uint32_t>(((1ull << 32) * ((1ull << sh) - range)) / range + 1);
  }
  return finish(launch_op(kOpRandint, g, offset, prm, nullptr, out, nullptr, static_cast<hipStream_t>(hip_stream)));
}

}  // extern "C"
