// TEST INFRASTRUCTURE ONLY (see philox.hpp).
#include "fill.hpp"

#include <cmath>
#include <cstring>
#include <limits>

#include "philox.hpp"

namespace oracle {

namespace {

uint32_t bits_of(float f) {
  uint32_t b;
  std::memcpy(&b, &f, sizeof b);
  return b;
}
float float_of(uint32_t b) {
  float f;
  std::memcpy(&f, &b, sizeof f);
  return f;
}

// The draw of global element j.
uint32_t draw_at(const Sharding& s, uint64_t seed, uint64_t offset, uint64_t j) {
  const Slot slot = slot_of(offset, j, s.virtual_threads);
  return draw_word(seed, slot, slot.word);
}

// 24 random bits as a fraction k / 2^24, exactly representable in fp32.
float fraction24(uint32_t x) { return static_cast<float>(x >> 8) * 0x1p-24f; }

}  // namespace

float float_from_bf16(uint16_t h) { return float_of(static_cast<uint32_t>(h) << 16); }

// Nearest-even rounding to bfloat16, done by comparing the candidates.  The
// candidates are the bfloat16 values whose bit patterns neighbour the
// truncation of `v` seen as fp32; all of them are exact doubles.
uint16_t bf16_from_double(double v) {
  if (std::isnan(v)) return 0x7FC0;
  const float f = static_cast<float>(v);  // only used to find the neighbourhood
  if (std::isinf(f) && std::isinf(v)) return static_cast<uint16_t>(bits_of(f) >> 16);
  const uint16_t sign = std::signbit(v) ? 0x8000 : 0;
  const double mag = std::fabs(v);
  uint32_t fb = bits_of(std::fabs(f));
  if (std::isinf(f)) fb = 0x7F7FFFFFu;  // huge finite double: start from the top of the range
  const int32_t mid = static_cast<int32_t>(fb >> 16);
  int32_t best = -1;
  double best_err = std::numeric_limits<double>::infinity();
  for (int32_t cand = mid - 1; cand <= mid + 1; ++cand) {
    if (cand < 0 || cand > 0x7F80) continue;
    const double cv = (cand == 0x7F80) ? std::ldexp(1.0, 128)  // where infinity sits for rounding
                                       : static_cast<double>(float_from_bf16(static_cast<uint16_t>(cand)));
    const double err = std::fabs(mag - cv);
    if (err < best_err || (err == best_err && (cand % 2 == 0))) {
      best_err = err;
      best = cand;
    }
  }
  return static_cast<uint16_t>(sign | static_cast<uint16_t>(best));
}

uint16_t bf16_from_float(float v) { return bf16_from_double(static_cast<double>(v)); }

// binary16: 1 sign bit, 5 exponent bits (bias 15), 10 fraction bits.
double double_from_f16(uint16_t h) {
  const int sign = h >> 15, e = (h >> 10) & 31, m = h & 1023;
  double mag;
  if (e == 31) mag = m ? std::numeric_limits<double>::quiet_NaN() : std::numeric_limits<double>::infinity();
  else if (e == 0) mag = std::ldexp(static_cast<double>(m), -24);             // subnormal: m * 2^-24
  else mag = std::ldexp(1.0 + static_cast<double>(m) / 1024.0, e - 15);      // (1 + m / 2^10) * 2^(e - 15)
  return sign ? -mag : mag;
}

// The non-negative patterns 0 .. 0x7C00 are ordered like their values, so the two
// neighbours of |v| are found by search; infinity takes part in the comparison at
// 2^16, where the next value of the format would sit.
uint16_t f16_from_double(double v) {
  if (std::isnan(v)) return 0x7E00;
  const uint16_t sign = std::signbit(v) ? 0x8000 : 0;
  const double mag = std::fabs(v);
  auto val = [](int32_t pat) { return pat == 0x7C00 ? 65536.0 : double_from_f16(static_cast<uint16_t>(pat)); };
  if (mag >= 65536.0) return static_cast<uint16_t>(sign | 0x7C00);
  int32_t lo = 0, hi = 0x7C00;  // val(lo) <= mag < val(hi)
  while (hi - lo > 1) {
    const int32_t mid = (lo + hi) / 2;
    if (val(mid) <= mag) lo = mid;
    else hi = mid;
  }
  const double below = mag - val(lo), above = val(hi) - mag;
  int32_t best;
  if (below < above) best = lo;
  else if (above < below) best = hi;
  else best = (lo % 2 == 0) ? lo : hi;
  return static_cast<uint16_t>(sign | static_cast<uint16_t>(best));
}

uint16_t round_16(DType dt, double v) { return dt == kF16 ? f16_from_double(v) : bf16_from_double(v); }
float value_16(DType dt, uint16_t h) {
  return dt == kF16 ? static_cast<float>(double_from_f16(h)) : float_from_bf16(h);  // exact either way
}

float uniform_f32(uint32_t x, float low, float high) {
  const float u = fraction24(x);
  const float width = high - low;  // rounded once
  const float scaled = u * width;  // rounded once
  float r = scaled + low;          // rounded once
  if (r >= high && high > low) r = std::nextafterf(high, low);
  return r;
}

uint16_t uniform_16(DType dt, uint32_t x, float low, float high) {
  const float r = uniform_f32(x, low, high);
  uint16_t h = round_16(dt, static_cast<double>(r));
  if (high > low && value_16(dt, h) >= high) {
    // Largest value of the format strictly below high (sign-magnitude patterns: one
    // step down is pattern - 1 above zero and pattern + 1 below it).
    uint16_t top = round_16(dt, static_cast<double>(high));
    if (value_16(dt, top) >= high) {
      const float t = value_16(dt, top);
      if (t > 0.0f) top = static_cast<uint16_t>(top - 1);
      else if (t == 0.0f) top = 0x8001;  // just below zero
      else top = static_cast<uint16_t>(top + 1);
    }
    h = top;
  }
  return h;
}

uint16_t uniform_bf16(uint32_t x, float low, float high) { return uniform_16(kBF16, x, low, high); }

double normal_f64(uint32_t xa, uint32_t xb, bool odd, double mean, double std) {
  const double pi = 3.14159265358979323846264338327950288;
  const double u1 = (static_cast<double>(xa >> 8) + 1.0) * 0x1p-24;  // (0, 1]
  const double u2 = static_cast<double>(xb >> 8) * 0x1p-24;          // [0, 1)
  const double radius = std::sqrt(-2.0 * std::log(u1));
  const double angle = 2.0 * pi * u2;
  const double n = odd ? radius * std::sin(angle) : radius * std::cos(angle);
  return mean + std * n;
}

uint32_t dropout_threshold(double p) {
  return static_cast<uint32_t>(std::floor((1.0 - p) * 16777216.0 + 0.5));
}

float dropout_scale(double p) { return static_cast<float>(1.0 / (1.0 - p)); }

void raw_u32(const Sharding& s, uint64_t seed, uint64_t offset, int64_t i_begin, int64_t i_end,
             uint32_t* out) {
  for_each_local(s, i_begin, i_end,
                 [&](int64_t i, uint64_t j) { out[i] = draw_at(s, seed, offset, j); });
}

void uniform(const Sharding& s, DType dt, double low, double high, uint64_t seed, uint64_t offset,
             int64_t i_begin, int64_t i_end, void* out) {
  const float lo = static_cast<float>(low), hi = static_cast<float>(high);
  for_each_local(s, i_begin, i_end, [&](int64_t i, uint64_t j) {
    const uint32_t x = draw_at(s, seed, offset, j);
    if (dt == kF32) static_cast<float*>(out)[i] = uniform_f32(x, lo, hi);
    else static_cast<uint16_t*>(out)[i] = uniform_16(dt, x, lo, hi);
  });
}

// An element whose draw is word w of a block uses the draw pair of its half-block:
// words (0,1) for w in {0,1}, words (2,3) for w in {2,3}; the first word of the pair
// feeds the radius, the second the angle; an even word takes the cosine.  (In the
// flat stream w = p % 4, so neighbouring positions 2k, 2k+1 share a pair.)
static double normal_at(const Sharding& s, uint64_t seed, uint64_t offset, uint64_t j, double mean, double std) {
  const Slot slot = slot_of(offset, j, s.virtual_threads);
  const uint32_t even_word = slot.word - (slot.word % 2);
  const uint32_t xa = draw_word(seed, slot, even_word);
  const uint32_t xb = draw_word(seed, slot, even_word + 1);
  return normal_f64(xa, xb, (slot.word % 2) == 1, mean, std);
}

void normal(const Sharding& s, DType dt, double mean, double std, uint64_t seed, uint64_t offset,
            int64_t i_begin, int64_t i_end, void* out) {
  for_each_local(s, i_begin, i_end, [&](int64_t i, uint64_t j) {
    const double v = normal_at(s, seed, offset, j, mean, std);
    if (dt == kF32) static_cast<float*>(out)[i] = static_cast<float>(v);
    else static_cast<uint16_t*>(out)[i] = round_16(dt, v);
  });
}

void normal_f64_values(const Sharding& s, double mean, double std, uint64_t seed, uint64_t offset,
                       int64_t i_begin, int64_t i_end, double* out) {
  for_each_local(s, i_begin, i_end, [&](int64_t i, uint64_t j) {
    out[i] = normal_at(s, seed, offset, j, mean, std);
  });
}

void dropout(const Sharding& s, DType dt, double p, uint64_t seed, uint64_t offset,
             int64_t i_begin, int64_t i_end, const void* x, void* y, uint8_t* mask) {
  const uint32_t threshold = dropout_threshold(p);
  const float scale = dropout_scale(p);
  for_each_local(s, i_begin, i_end, [&](int64_t i, uint64_t j) {
    const uint32_t r = draw_at(s, seed, offset, j);
    const bool keep = (r >> 8) < threshold;
    if (mask) mask[i] = keep ? 1 : 0;
    if (dt == kF32) {
      const float xin = static_cast<const float*>(x)[i];
      static_cast<float*>(y)[i] = keep ? xin * scale : 0.0f;
    } else {
      const float xin = value_16(dt, static_cast<const uint16_t*>(x)[i]);
      const float prod = xin * scale;  // rounded to fp32 first
      static_cast<uint16_t*>(y)[i] = keep ? round_16(dt, static_cast<double>(prod)) : uint16_t{0};
    }
  });
}

void dropout_add(const Sharding& s, DType dt, double p, uint64_t seed, uint64_t offset, int64_t i_begin,
                 int64_t i_end, const void* x, const void* residual, void* y, uint8_t* mask) {
  const uint32_t threshold = dropout_threshold(p);
  const float scale = dropout_scale(p);
  for_each_local(s, i_begin, i_end, [&](int64_t i, uint64_t j) {
    const uint32_t r = draw_at(s, seed, offset, j);
    const bool keep = (r >> 8) < threshold;
    if (mask) mask[i] = keep ? 1 : 0;
    if (dt == kF32) {
      const float prod = static_cast<const float*>(x)[i] * scale;
      const float kept = keep ? prod : 0.0f;
      static_cast<float*>(y)[i] = static_cast<const float*>(residual)[i] + kept;
    } else {
      const float prod = value_16(dt, static_cast<const uint16_t*>(x)[i]) * scale;
      const float kept = keep ? prod : 0.0f;
      const float sum = value_16(dt, static_cast<const uint16_t*>(residual)[i]) + kept;
      static_cast<uint16_t*>(y)[i] = round_16(dt, static_cast<double>(sum));
    }
  });
}

void randint(const Sharding& s, int64_t low, int64_t high, uint64_t seed, uint64_t offset,
             int64_t i_begin, int64_t i_end, int64_t* out) {
  const uint64_t range = static_cast<uint64_t>(high - low);
  for_each_local(s, i_begin, i_end, [&](int64_t i, uint64_t j) {
    const uint64_t r = draw_at(s, seed, offset, j);
    out[i] = low + static_cast<int64_t>(r % range);
  });
}

uint64_t advance_offset(const std::vector<int64_t>& global_shape, const std::vector<int64_t>& global_stride,
                        uint64_t offset, uint64_t virtual_threads) {
  uint64_t n = 1;
  for (int64_t e : global_shape) n *= static_cast<uint64_t>(e);
  uint64_t span = n;
  if (n != 0 && !global_stride.empty()) {
    uint64_t last = 0;  // flat index of the last element
    for (size_t d = 0; d < global_shape.size(); ++d)
      last += static_cast<uint64_t>(global_shape[d] - 1) * static_cast<uint64_t>(global_stride[d]);
    span = last + 1;
  }
  // With theta virtual threads every thread steps ceil(span / theta) times.
  if (virtual_threads != 0) span = (span + virtual_threads - 1) / virtual_threads;
  return offset + 4 * ((span + 3) / 4);
}

}  // namespace oracle
