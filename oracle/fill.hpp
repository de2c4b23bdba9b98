// TEST INFRASTRUCTURE ONLY (see philox.hpp).
//
// Single-device semantics (Section 5 of the paper): the value of the element
// with global flat index j depends on the seed, the offset and j alone.  A
// rank's local tensor is that function evaluated at the global indices its
// shard holds (Algorithm 1).  Everything here works one element at a time.
#pragma once
#include <cstdint>

#include "shard.hpp"

namespace oracle {

enum DType : int32_t { kF32 = 0, kBF16 = 1, kF16 = 2 };

// --- value of ONE global element -------------------------------------------

// Uniform in [low, high): top 24 bits of the draw scaled by 2^-24 (exact in
// fp32), then u * (high - low) + low as two separately rounded fp32 operations;
// a result that reaches high is pulled to the largest value below it.
float uniform_f32(uint32_t x, float low, float high);
// Same value, then rounded to bfloat16 (nearest even) with the same pull-back.
uint16_t uniform_bf16(uint32_t x, float low, float high);
// The same for either 16-bit dtype (kBF16 or kF16, IEEE binary16).
uint16_t uniform_16(DType dt, uint32_t x, float low, float high);

// Box-Muller in double.  `xa` feeds the radius, `xb` the angle; `odd` picks
// sine (odd stream position) or cosine (even).  Returns mean + std * n.
double normal_f64(uint32_t xa, uint32_t xb, bool odd, double mean, double std);

// Integer keep-threshold and fp32 scale of dropout with probability p.
uint32_t dropout_threshold(double p);
float dropout_scale(double p);

// Correctly rounded (nearest, ties to even) conversions.
uint16_t bf16_from_double(double v);
uint16_t bf16_from_float(float v);
float float_from_bf16(uint16_t h);
// IEEE binary16: the value of a bit pattern, read off the format's definition, and
// nearest-even rounding by search over the patterns.  round_16 / value_16 take either
// 16-bit dtype.
double double_from_f16(uint16_t h);
uint16_t f16_from_double(double v);
uint16_t round_16(DType dt, double v);
float value_16(DType dt, uint16_t h);

// --- a rank's local tensor, elements [i_begin, i_end) ------------------------
void raw_u32(const Sharding& s, uint64_t seed, uint64_t offset, int64_t i_begin, int64_t i_end,
             uint32_t* out);
void uniform(const Sharding& s, DType dt, double low, double high, uint64_t seed, uint64_t offset,
             int64_t i_begin, int64_t i_end, void* out);
void normal(const Sharding& s, DType dt, double mean, double std, uint64_t seed, uint64_t offset,
            int64_t i_begin, int64_t i_end, void* out);
void normal_f64_values(const Sharding& s, double mean, double std, uint64_t seed, uint64_t offset,
                       int64_t i_begin, int64_t i_end, double* out);
void dropout(const Sharding& s, DType dt, double p, uint64_t seed, uint64_t offset,
             int64_t i_begin, int64_t i_end, const void* x, void* y, uint8_t* mask);
// Dropout followed by a residual add: y = round_dtype(fl32(residual + (keep ? fl32(x * scale) : +0))).
void dropout_add(const Sharding& s, DType dt, double p, uint64_t seed, uint64_t offset, int64_t i_begin,
                 int64_t i_end, const void* x, const void* residual, void* y, uint8_t* mask);
// Integers uniform in [low, high) (high - low <= 2^32): low + draw mod (high - low).
void randint(const Sharding& s, int64_t low, int64_t high, uint64_t seed, uint64_t offset,
             int64_t i_begin, int64_t i_end, int64_t* out);

// Offset after an operator on a tensor of the given GLOBAL shape: one draw per
// stream position the whole tensor reaches (= one per element when the tensor is
// contiguous; up to the largest flat index + 1 under a global stride), rounded up
// to a whole generator block.
uint64_t advance_offset(const std::vector<int64_t>& global_shape, const std::vector<int64_t>& global_stride,
                        uint64_t offset, uint64_t virtual_threads = 0);

}  // namespace oracle
