// gfx950 kernels of the sharded random fill / fused dropout path
// (veScale Section 5, Algorithm 1, with Philox4x32-10 as the generator).
//
// Work decomposition.  Algorithm 1 walks local elements one by one.  Here a
// thread owns one generator block (4 consecutive stream positions, hence 4
// consecutive global elements) or two of them, so that one Philox call feeds
// four outputs that stay in registers.
//
//  * aligned kernels: every run of the shard starts on a block boundary and its
//    length is a multiple of the unit (4 or 8 elements); unit w covers local
//    elements [w*V, (w+1)*V) and all accesses are 16-byte vectors.  A shard that is
//    a single run may have any length: its last, partial unit is written by element.
//  * ragged kernels: any run start / length (e.g. a column shard whose first
//    column is 1366).  A thread owns one GLOBAL block and stores the lanes that
//    fall inside the run; whole blocks leave as one element-aligned vector store.
//    Used by the normal fills and the 16-bit uniform fills, and wherever runs are shorter
//    than 16 elements or the innermost global stride is not 1.
//  * tiled kernels: ragged shards of the raw, randint, fp32 uniform and dropout operators.  A
//    workgroup owns a 128-byte aligned tile of the LOCAL tensor; its threads first
//    own the GLOBAL blocks that intersect the tile and scatter their values into
//    LDS at local positions, then each thread takes an aligned unit back out of
//    LDS and stores it.  One block still feeds four outputs, and every global
//    access is an aligned 128-bit vector (wave stores that do not cover whole
//    128-byte lines run at 4.9 instead of 6.8 TB/s).
//  * chain kernel: Algorithm 1 element by element, for shards that are not boxes
//    and for the virtual-thread layout.
//
// Launches are one-shot (one unit per thread): on MI355X this sustained a higher
// rate than grid-stride loops or several units per thread.
#include <hip/hip_runtime.h>

#include <tuple>
#include <type_traits>
#include <utility>

#include "launch.hpp"
#include "philox.h"
#include "plan.h"
#include "stream_store.h"

// 1 (always, in the library): keep the argument fetch in one batch - no early exit, operator
// parameters live at kernel entry, the generator pinned above the bounds branch.  0 only in the
// measurement variant that times the kernels without it.
#ifndef VESRNG_PIN_ARGUMENT_FETCH
#define VESRNG_PIN_ARGUMENT_FETCH 1
#endif
// 0 (always, in the library): whole blocks of a ragged run leave as element-aligned vector stores.
// 1 only in the measurement variant that first realigns them to 16-byte units across lanes (measured:
// the extra instructions cost more than the aligned stores gain; the code is kept so that the
// comparison can be repeated).
#ifndef VESRNG_RAGGED_DPP_REALIGN
#define VESRNG_RAGGED_DPP_REALIGN 0
#endif
// 1 (always, in the library): shards whose runs are whole wavefronts long take the aligned kernel's form
// with the run arithmetic in scalar registers.  0 only in the measurement variant that times the per-lane form.
#ifndef VESRNG_WAVE_UNIFORM_RUNS
#define VESRNG_WAVE_UNIFORM_RUNS 1
#endif
// 0 (always, in the library): the staging kernel works its tile map out per lane.  1 only in the measurement
// variant that works it out once per wavefront in scalar registers where runs are long enough (measured: slower -
// the scalar unit, one per compute unit, then issues more instructions per wave than the vector ALUs save).
#ifndef VESRNG_TILE_WAVE_MAP
#define VESRNG_TILE_WAVE_MAP 0
#endif
// 1 (always, in the library): column-like shards whose runs all start at the same position modulo 4 take the
// short form of the staging kernel's tile map (plan.h: tile_spot_same_phase).  0 only in the measurement variant
// that times the general form on them.
// 1 (always, in the library): large aligned launches of fused dropout that also write the mask run with at most
// seven resident waves per SIMD instead of the hardware's eight (see kWaveCapLdsBytes).  0 only in the measurement
// variant that times them uncapped.
#ifndef VESRNG_CAP_MASKED_DROPOUT_WAVES
#define VESRNG_CAP_MASKED_DROPOUT_WAVES 1
#endif
// 1 (always, in the library): shards that need 64-bit indices as a whole are served piece by piece through the 32-bit
// kernels where they can be cut.  0 only in the measurement variant that times the 64-bit kernels on them.
#ifndef VESRNG_WIDE_SHARDS_IN_PIECES
#define VESRNG_WIDE_SHARDS_IN_PIECES 1
#endif
// 3 (always, in the library): shards with two and three axes of runs take kernels whose run arithmetic is written
// out for that number of axes.  1 only in the measurement variant that serves them with the loop over any number.
#ifndef VESRNG_EXACT_RUN_AXES
#define VESRNG_EXACT_RUN_AXES 3
#endif
// 1 (always, in the library): the aligned randint fill runs two threads per generator block, each storing one half.
// 0 only in the measurement variant that runs one thread per block and trades halves between neighbouring lanes.
#ifndef VESRNG_RANDINT_HALF_BLOCKS
#define VESRNG_RANDINT_HALF_BLOCKS 1
#endif
#ifndef VESRNG_TILE_SAME_PHASE
#define VESRNG_TILE_SAME_PHASE 1
#endif
// Measurement variants only: which operators may take the staging kernel.  -1 (the library): the
// measured choice below; 0: none; 1: every operator, small tile only; 2: every operator, large tile
// wherever the kernel has one.
#ifndef VESRNG_TILING
#define VESRNG_TILING -1
#endif

namespace vesrng {

namespace {
// The measurement variants of this file (one design choice flipped, built into libraries of their
// own for the benchmark) put everything into a named namespace, so that their kernels appear
// under their own names in a profiler's trace.  The library itself defines no tag.
#ifdef VESRNG_VARIANT_TAG
inline namespace VESRNG_VARIANT_TAG {
#endif

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// 16 / 8 bytes that are only 4-byte aligned: whole blocks inside a ragged run.  Vector types, so
// that each leaves as ONE store (a struct of four words is four scalar stores to the optimiser,
// which then shares the last one with the edge path and emits 12 + 4 bytes).
typedef u32x4 u32x4_align4 __attribute__((aligned(4)));
typedef u32x2 u32x2_align4 __attribute__((aligned(4)));

constexpr int kThreads = kThreadsPerGroup;
constexpr int kF32 = 0, kBF16 = 1, kF16 = 2;

// ---- conversions ---------------------------------------------------------------
// Two fp32 values rounded (nearest even) to a pair of 16-bit floats of dtype DT, low half first,
// and the exact fp32 value of either half.
template <int DT>
__device__ __forceinline__ uint32_t pack16(float lo, float hi) {
  if constexpr (DT == kF16) {
    // The values are fp32 results that get ONE more rounding.  Seen through, the compiler merges
    // the producing multiply with this conversion into a mixed-precision fma whose +0 addend
    // turns a product of -0 into +0; the empty asm keeps the two steps apart.
    asm("" : "+v"(lo));
    asm("" : "+v"(hi));
  }
  const f32x2 v = {lo, hi};
  if constexpr (DT == kBF16) return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));  // v_cvt_pk_bf16_f32
  else return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));                          // v_cvt_f16_f32 x2
}
template <int DT>
__device__ __forceinline__ float lo16(uint32_t pair) {
  if constexpr (DT == kBF16) return __uint_as_float(pair << 16);
  else return static_cast<float>(__builtin_bit_cast(f16x2, pair)[0]);
}
template <int DT>
__device__ __forceinline__ float hi16(uint32_t pair) {
  if constexpr (DT == kBF16) return __uint_as_float(pair & 0xFFFF0000u);
  else return static_cast<float>(__builtin_bit_cast(f16x2, pair)[1]);
}

__device__ __forceinline__ float fraction24(uint32_t x) {
  return static_cast<float>(x >> 8) * 0x1p-24f;  // exact
}

// Uniform in [low, high): u * width + low as two fp32 operations, held at `cap`, the largest value
// of the OUTPUT dtype below high.  Rounding to a 16-bit dtype is monotone, so capping the fp32
// value first gives what "round, then pull a result that reached high back below it" gives.
__device__ __forceinline__ float uniform_general(uint32_t x, const OpParams& prm) {
  const float r = __fadd_rn(__fmul_rn(fraction24(x), prm.width), prm.low);
  return __builtin_fminf(r, prm.cap);
}
// [0, 1): the value is u itself; only a 16-bit dtype can round it up to 1.
template <int DT>
__device__ __forceinline__ float uniform_unit(uint32_t x, const OpParams& prm) {
  const float u = fraction24(x);
  if constexpr (DT == kF32) return u;
  else return __builtin_fminf(u, prm.cap);
}

// Box-Muller on one draw pair; hardware log2 / sqrt / sin / cos (sin and cos take
// their argument in revolutions, which is exactly u2).
__device__ __forceinline__ void normal_pair(uint32_t xa, uint32_t xb, const OpParams& prm, float& even,
                                            float& odd) {
  const float u1 = __fmaf_rn(static_cast<float>(xa >> 8), 0x1p-24f, 0x1p-24f);  // ((xa >> 8) + 1) 2^-24, exact
  const float u2 = fraction24(xb);                                               // [0, 1), exact
  const float r2 = __fmul_rn(__builtin_amdgcn_logf(u1), -1.3862943611198906f);  // -2 ln u1
  const float radius = __fmul_rn(__builtin_amdgcn_sqrtf(r2), prm.stddev);       // std * sqrt(-2 ln u1)
  even = __fmaf_rn(radius, __builtin_amdgcn_cosf(u2), prm.mean);
  odd = __fmaf_rn(radius, __builtin_amdgcn_sinf(u2), prm.mean);
}

__device__ __forceinline__ bool keep_of(uint32_t x, const OpParams& prm) {
  return prm.keep_any != 0u && x <= prm.limit;
}

__device__ __forceinline__ int64_t randint_value(uint32_t x, const OpParams& prm) {
  uint32_t rem = x;
  if (prm.range != 0u) {
    uint32_t q = x;
    if (prm.range_s != 0u) {
      const uint32_t t = __umulhi(x, prm.range_m);
      q = (t + ((x - t) >> 1)) >> (prm.range_s - 1u);
    }
    rem = x - q * prm.range;
  }
  return prm.base + static_cast<int64_t>(rem);
}

// The per-element value of a whole generator block, as 32-bit patterns: fp32 bits for
// uniform and normal (whatever the output dtype), the raw draws for the operators whose
// conversion needs more than the draw (dropout needs x, randint widens to 64 bits).
template <int OP, int DT>
__device__ __forceinline__ void convert_block(const uint32_t (&d)[4], const OpParams& prm, uint32_t (&v)[4]) {
  if constexpr (OP == kOpUniform) {
    if (prm.unit_range) {  // wave-uniform; the empty asm keeps it a branch instead of four selects
      asm volatile("");
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = __float_as_uint(uniform_unit<DT>(d[e], prm));
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = __float_as_uint(uniform_general(d[e], prm));
    }
  } else if constexpr (OP == kOpNormal) {
    float n[4];
    normal_pair(d[0], d[1], prm, n[0], n[1]);
    normal_pair(d[2], d[3], prm, n[2], n[3]);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = __float_as_uint(n[e]);
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = d[e];
  }
}

template <int OP>
constexpr bool kIsDropout = (OP == kOpDropout || OP == kOpDropoutAdd);

// OP: OpKind.  DT: output dtype.  A unit is what one thread stores: V elements.
template <int OP, int DT>
struct UnitOf {
  static constexpr int kBlocks = (OP != kOpRaw && OP != kOpRandint && DT != kF32) ? 2 : 1;
  static constexpr int kElems = 4 * kBlocks;
};

// Two consecutive integers as one 16-byte store into chunk `c` (elements 2c, 2c + 1) of out.
__device__ __forceinline__ void store_randint_pair(uint32_t x0, uint32_t x1, const OpParams& prm, void* out,
                                                   uint64_t c) {
  const uint64_t r0 = static_cast<uint64_t>(randint_value(x0, prm));
  const uint64_t r1 = static_cast<uint64_t>(randint_value(x1, prm));
  const u32x4 o = {static_cast<uint32_t>(r0), static_cast<uint32_t>(r0 >> 32), static_cast<uint32_t>(r1),
                   static_cast<uint32_t>(r1 >> 32)};
  stream_store(o, static_cast<u32x4*>(out) + c);
}

// Writes unit number `u` of the local tensor (elements [u*V, (u+1)*V)) from the V values
// made by convert_block; dropout also consumes the 16 bytes of x loaded for the unit.
template <int OP, int DT>
__device__ __forceinline__ void emit_unit(const uint32_t (&v)[UnitOf<OP, DT>::kElems], const OpParams& prm,
                                          u32x4 xv, u32x4 rv, uint64_t u, void* out, uint8_t* mask) {
  constexpr int NB = UnitOf<OP, DT>::kBlocks;
  if constexpr (OP == kOpRandint) {
    store_randint_pair(v[0], v[1], prm, out, 2 * u);
    store_randint_pair(v[2], v[3], prm, out, 2 * u + 1);
  } else if constexpr (kIsDropout<OP>) {
    constexpr bool kAdd = (OP == kOpDropoutAdd);
    u32x4 y;
    if constexpr (DT == kF32) {
      uint32_t m = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool keep = keep_of(v[e], prm);
        const float prod = __fmul_rn(__uint_as_float(xv[e]), prm.scale);
        const float kept = keep ? prod : 0.0f;
        y[e] = __float_as_uint(kAdd ? __fadd_rn(__uint_as_float(rv[e]), kept) : kept);
        m |= (keep ? 1u : 0u) << (8 * e);
      }
      stream_store(y, static_cast<u32x4*>(out) + u);
      if (mask) stream_store(m, reinterpret_cast<uint32_t*>(mask) + u);
    } else {
      u32x2 m = {0u, 0u};
#pragma unroll
      for (int b = 0; b < NB; ++b) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {  // two packed pairs per block
          const uint32_t pair = xv[2 * b + h];
          const bool k0 = keep_of(v[4 * b + 2 * h], prm), k1 = keep_of(v[4 * b + 2 * h + 1], prm);
          const float p0 = __fmul_rn(lo16<DT>(pair), prm.scale);
          const float p1 = __fmul_rn(hi16<DT>(pair), prm.scale);
          // Select before rounding: a dropped element becomes +0 whatever x held.
          float y0 = k0 ? p0 : 0.0f, y1 = k1 ? p1 : 0.0f;
          if constexpr (kAdd) {
            y0 = __fadd_rn(lo16<DT>(rv[2 * b + h]), y0);
            y1 = __fadd_rn(hi16<DT>(rv[2 * b + h]), y1);
          }
          y[2 * b + h] = pack16<DT>(y0, y1);
          m[b] |= ((k0 ? 1u : 0u) | (k1 ? 0x100u : 0u)) << (16 * h);
        }
      }
      stream_store(y, static_cast<u32x4*>(out) + u);
      if (mask) stream_store(m, reinterpret_cast<u32x2*>(mask) + u);
    }
  } else {
    u32x4 o;
    if constexpr (OP == kOpRaw || DT == kF32) {
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = v[e];
    } else {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float a = __uint_as_float(v[2 * q]), b = __uint_as_float(v[2 * q + 1]);
        o[q] = pack16<DT>(a, b);
      }
    }
    stream_store(o, static_cast<u32x4*>(out) + u);
  }
}

// Writes ONE local element `i` from its convert_block value (edges of ragged shards).
template <int OP, int DT>
__device__ __forceinline__ void emit_element(uint32_t v, const OpParams& prm, const void* xin, int64_t i, void* out,
                                             uint8_t* mask) {
  if constexpr (OP == kOpRaw) {
    static_cast<uint32_t*>(out)[i] = v;
  } else if constexpr (OP == kOpRandint) {
    static_cast<int64_t*>(out)[i] = randint_value(v, prm);
  } else if constexpr (kIsDropout<OP>) {
    constexpr bool kAdd = (OP == kOpDropoutAdd);
    const bool keep = keep_of(v, prm);
    if constexpr (DT == kF32) {
      const float x = static_cast<const float*>(xin)[i];
      const float kept = keep ? __fmul_rn(x, prm.scale) : 0.0f;
      static_cast<float*>(out)[i] = kAdd ? __fadd_rn(static_cast<const float*>(prm.residual)[i], kept) : kept;
    } else {
      const uint32_t x = static_cast<const uint16_t*>(xin)[i];
      float kept = keep ? __fmul_rn(lo16<DT>(x), prm.scale) : 0.0f;
      if constexpr (kAdd) {
        const uint32_t r = static_cast<const uint16_t*>(prm.residual)[i];
        kept = __fadd_rn(lo16<DT>(r), kept);
      }
      static_cast<uint16_t*>(out)[i] = static_cast<uint16_t>(pack16<DT>(kept, 0.0f));
    }
    if (mask) mask[i] = keep ? 1 : 0;
  } else if constexpr (DT == kF32) {
    static_cast<uint32_t*>(out)[i] = v;
  } else {
    const float a = __uint_as_float(v);
    const uint32_t pair = pack16<DT>(a, a);
    static_cast<uint16_t*>(out)[i] = static_cast<uint16_t>(pair);
  }
}

// Makes the operator's scalar parameters live at the point of call, so that they are fetched
// with the first batch of kernel arguments instead of in a second, dependent round after the
// generator (the compiler otherwise loads them where the conversion first needs them).
template <int OP>
__device__ __forceinline__ void touch_params(const OpParams& prm) {
#if !VESRNG_PIN_ARGUMENT_FETCH
  (void)prm;
  return;
#endif
  if constexpr (OP == kOpUniform)
    asm volatile("" ::"s"(prm.width), "s"(prm.low), "s"(prm.cap), "s"(prm.unit_range));
  else if constexpr (OP == kOpNormal)
    asm volatile("" ::"s"(prm.mean), "s"(prm.stddev));
  else if constexpr (kIsDropout<OP>)
    asm volatile("" ::"s"(prm.scale), "s"(prm.limit), "s"(prm.keep_any));
  else if constexpr (OP == kOpRandint)
    asm volatile("" ::"s"(prm.range), "s"(prm.range_m), "s"(prm.range_s));
}

// ---- locating work ---------------------------------------------------------------
// (run_position, locate and the tile map live in plan.h: the host evaluates them too.)
// The part of global block `bi` of a run that belongs to the run.
template <typename IT>
struct BlockSpan {
  uint32_t first, last;  // lanes [first, last) are inside the run (last = 0: none)
  typename SignedOf<IT>::type li0;  // local flat index of lane 0 (may lie before the run: only valid lanes are used)
  bool any;
};
template <typename IT>
__device__ __forceinline__ BlockSpan<IT> block_span(const PlanT<IT>& plan, IT run, IT bi, uint64_t run_pos) {
  using ST = typename SignedOf<IT>::type;
  const uint32_t phase = static_cast<uint32_t>(run_pos) & 3u;
  // Elements of the run from this block's lane 0 onwards.  Not positive only when runs differ
  // in phase and units_per_run is the upper bound over phases.
  const ST remaining = static_cast<ST>(phase + plan.run_len) - static_cast<ST>(4 * bi);
  BlockSpan<IT> s;
  s.any = remaining > 0;
  s.first = (bi == 0) ? phase : 0u;
  s.last = remaining < 4 ? static_cast<uint32_t>(remaining > 0 ? remaining : 0) : 4u;
  s.li0 = static_cast<ST>(run * plan.run_len + 4 * bi) - static_cast<ST>(phase);
  return s;
}

// ---- aligned kernels -----------------------------------------------------------
// The value the wave's first active lane holds, as a wave-uniform (scalar) value.
__device__ __forceinline__ __attribute__((unused)) uint32_t first_lane(uint32_t x) {
  return static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(x)));
}

// WAVE: every run is a whole number of wavefronts long (units_per_run is a multiple of 64), so the 64
// units of a wave lie in ONE run: the run's number, its stream position and the 64-bit stride products
// are the same for all lanes and are worked out once per wave in scalar registers; a lane only adds
// its slot.  (All of it costs vector-ALU issue slots otherwise, and the 16-bit fills and the normal
// fills are bound by exactly those.)
template <int OP, int DT, typename IT, int NOUT, bool WAVE>
__global__ void __launch_bounds__(kThreads)
aligned_kernel(const PlanT<IT> plan, const OpParams prm, const void* xin, void* out, uint8_t* mask) {
  constexpr int NB = UnitOf<OP, DT>::kBlocks;
  constexpr int V = UnitOf<OP, DT>::kElems;
  static_assert(!(WAVE && NOUT == 0), "a single run needs no run arithmetic at all");
  // Threads past the end compute unit 0 again and skip the stores: no early exit, so all
  // kernel arguments are fetched in one batch at the top.
  touch_params<OP>(prm);
#if VESRNG_PIN_ARGUMENT_FETCH
  asm volatile("" ::"s"(out), "s"(mask));
#endif
  // randint writes 32 bytes per generator block.  Lane by lane that would be two stores of 16 bytes at a 32-byte
  // stride, which run at a third of the contiguous rate (2.35 TB/s).  The library runs TWO threads per block: thread
  // t computes block t / 2 - the generator is cheap next to 16 bytes of HBM traffic - and stores the half t % 2 (two
  // integers, 16 bytes): one store instruction per thread, a wave's kilobyte contiguous: 7.3 TB/s on a contiguous
  // shard, 6.85 with runs.  The form it replaced (measurement variant only) keeps one thread per block: the lane pair
  // (2k, 2k+1) of a wave computes blocks k and 32 + k of the wave's 64 and the two trade halves across lanes, so that
  // either of a thread's TWO store instructions writes 1 KiB without gaps: 5.9 TB/s, the rate of every kernel here
  // that issues two 16-byte stores per thread.
  const uint32_t lane = threadIdx.x & 63u;
  constexpr bool kHalf = (OP == kOpRandint) && (VESRNG_RANDINT_HALF_BLOCKS != 0) && !WAVE;
  if constexpr (kHalf) {
    const uint64_t t64 = static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x;
    const bool on = (t64 >> 1) < plan.total_units;
    const uint64_t w = on ? (t64 >> 1) : 0;
    IT run, unit;
    uint64_t run_pos;
    locate<NOUT>(plan, static_cast<IT>(w), run, unit, run_pos);
    uint32_t d[4];
    philox_block((run_pos + static_cast<uint64_t>(unit) * V) >> 2, prm.key0, prm.key1, d);
    asm volatile("" : "+v"(d[0]), "+v"(d[1]), "+v"(d[2]), "+v"(d[3]));
    if (!on) return;
    const bool hi = (t64 & 1u) != 0u;
    store_randint_pair(hi ? d[2] : d[0], hi ? d[3] : d[1], prm, out, t64);
    return;
  }
  const uint32_t slot = (OP == kOpRandint) ? (lane >> 1) + ((lane & 1u) << 5) : lane;  // the wave's unit this lane takes
  uint64_t wave_base, w64, block0;
  bool live;
  if constexpr (WAVE) {
    wave_base = static_cast<uint64_t>(blockIdx.x) * kThreads + (first_lane(threadIdx.x >> 6) << 6);  // scalar
    live = wave_base < plan.total_units;  // total_units is a multiple of 64 here: the whole wave or none of it
    const uint64_t base = live ? wave_base : 0;
    const IT run = plan.units_div.div(static_cast<IT>(base));
    const IT unit0 = static_cast<IT>(base) - run * plan.units_per_run;
    const uint64_t start = run_position<NOUT>(plan, run) + static_cast<uint64_t>(unit0) * V;  // of the wave's first unit
    block0 = (start >> 2) + slot * static_cast<uint32_t>(V / 4);
    w64 = base + slot;
  } else {
    const uint64_t t0 = static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x;
    wave_base = t0 - lane;
    const uint64_t t64 = wave_base + slot;
    live = t64 < plan.total_units;
#if !VESRNG_PIN_ARGUMENT_FETCH
    if constexpr (OP != kOpRandint)
      if (!live) return;  // measurement variant: the plain early exit
#endif
    w64 = live ? t64 : 0;
    IT run, unit;
    uint64_t run_pos;
    locate<NOUT>(plan, static_cast<IT>(w64), run, unit, run_pos);
    block0 = (run_pos + static_cast<uint64_t>(unit) * V) >> 2;
  }

  // A shard that is ONE run (contiguous in the global tensor) may end inside a unit: its last
  // unit is then written element by element, and its 16-byte load would pass the end of x.
  bool partial = false;
  uint32_t tail = 0;
  if constexpr (NOUT == 0) {
    tail = static_cast<uint32_t>(plan.run_len) & static_cast<uint32_t>(V - 1);
    partial = tail != 0u && w64 + 1 == plan.total_units;
  }

  // Dropout: issue the load before the generator so that it overlaps the ALU work.
  u32x4 xv = {0u, 0u, 0u, 0u}, rv = {0u, 0u, 0u, 0u};
  if constexpr (kIsDropout<OP>)
    if (!partial) xv = __builtin_nontemporal_load(static_cast<const u32x4*>(xin) + w64);
  if constexpr (OP == kOpDropoutAdd)
    if (!partial) rv = __builtin_nontemporal_load(static_cast<const u32x4*>(prm.residual) + w64);
  __builtin_amdgcn_sched_barrier(0);  // the loads are issued here, not moved down to their first use

  uint32_t d[NB][4];
#pragma unroll
  for (int b = 0; b < NB; ++b) philox_block(block0 + b, prm.key0, prm.key1, d[b]);
  // Keep the generator (and the argument loads it needs) ahead of the bounds branch: without
  // this the compiler sinks everything below the branch and fetches the arguments in two
  // dependent rounds.
#if VESRNG_PIN_ARGUMENT_FETCH
#pragma unroll
  for (int b = 0; b < NB; ++b) asm volatile("" : "+v"(d[b][0]), "+v"(d[b][1]), "+v"(d[b][2]), "+v"(d[b][3]));
  if constexpr (kIsDropout<OP>) asm volatile("" : "+v"(xv));
  if constexpr (OP == kOpDropoutAdd) asm volatile("" : "+v"(rv));
#endif
  if constexpr (OP == kOpRandint) {
    // All 64 lanes are still active here.  The even lane holds block k, the odd lane block
    // 32 + k; each hands the half its partner stores to the neighbouring lane (quad_perm
    // [1,0,3,2]).  Store A covers blocks 0..31 of the wave, store B blocks 32..63.
    const bool odd = (lane & 1u) != 0u;
    const uint32_t give0 = odd ? d[0][0] : d[0][2], give1 = odd ? d[0][1] : d[0][3];
    const uint32_t got0 = static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(give0), 0xB1, 0xF, 0xF, false));
    const uint32_t got1 = static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(give1), 0xB1, 0xF, 0xF, false));
    const uint64_t block_a = wave_base + (lane >> 1);  // the block whose half this lane writes in store A
    const uint64_t chunk = 2 * wave_base + lane;
    if (block_a < plan.total_units)
      store_randint_pair(odd ? got0 : d[0][0], odd ? got1 : d[0][1], prm, out, chunk);
    if (block_a + 32 < plan.total_units)
      store_randint_pair(odd ? d[0][2] : got0, odd ? d[0][3] : got1, prm, out, chunk + 64);
    return;
  }
  if (!live) return;

  uint32_t v[V];
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    uint32_t vb[4];
    convert_block<OP, DT>(d[b], prm, vb);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[4 * b + e] = vb[e];
  }
  if (partial) {
#pragma unroll
    for (int e = 0; e < V - 1; ++e)
      if (static_cast<uint32_t>(e) < tail)
        emit_element<OP, DT>(v[e], prm, xin, static_cast<int64_t>(w64 * V + e), out, mask);
    return;
  }
  emit_unit<OP, DT>(v, prm, xv, rv, w64, out, mask);
}

// ---- tiled kernels ---------------------------------------------------------------
// UPT: aligned units a thread takes out of the tile in stage B (the tile is up to kThreads * UPT
// units).  WAVE (measurement variant only): runs have at least 64 blocks and stage A works the tile map out
// once per wavefront in scalar registers (plan.h: tile_wave) instead of once per lane.
// How stage A of the staging kernel finds where a generator block lands (plan.h).
constexpr int kTileMapBlock = 0;      // per block, any box-shaped shard
constexpr int kTileMapWave = 1;       // per wavefront (measurement variant only)
constexpr int kTileMapSamePhase = 2;  // per block, short form: one axis of runs, one phase, 32-bit indices

template <int OP, int DT, typename IT, int NOUT, int UPT, int MAP>
__global__ void __launch_bounds__(kThreads)
tiled_kernel(const PlanT<IT> plan, const OpParams prm, const TileArgs<IT> ta, const void* xin, void* out,
             uint8_t* mask) {
  constexpr int V = UnitOf<OP, DT>::kElems;
  // One 32-bit value per local element of the tile, plus a slot that swallows the lanes of
  // edge blocks that fall outside the tile or the run (cheaper than predicated LDS writes).
  constexpr int kDummy = kThreads * V * UPT;
  __shared__ __attribute__((aligned(16))) uint32_t tile[kThreads * V * UPT + 4];

  const uint64_t tile_elems = static_cast<uint64_t>(ta.tile_units) * V;
  const uint64_t i0 = static_cast<uint64_t>(blockIdx.x) * tile_elems;  // first local element of the tile
  const uint64_t i1 = (i0 + tile_elems < ta.local_numel) ? i0 + tile_elems : ta.local_numel;
  const int32_t lim = static_cast<int32_t>(i1 - i0);

  // Generator blocks that intersect [i0, i1): flattened (run, block) numbers wa .. wa + count - 1.
  const IT wa = tile_block_of<NOUT>(plan, ta, i0);
  const IT count = tile_block_of<NOUT>(plan, ta, i1 - 1) - wa + 1;

  // Stage A: one block per thread (one pass for 4-byte units, two for bfloat16 units).
  for (IT k = threadIdx.x; k < count; k += kThreads) {
    TileSpot spot;
    if constexpr (MAP == kTileMapWave) {
      // Lane 0 of the wave holds the wave's first block number (lanes run out at the top end only).
      const uint64_t k64 = static_cast<uint64_t>(k);
      const uint64_t kw = (static_cast<uint64_t>(first_lane(static_cast<uint32_t>(k64 >> 32))) << 32) |
                          first_lane(static_cast<uint32_t>(k64));
      spot = tile_spot_of_lane(tile_wave<NOUT>(plan, i0, lim, static_cast<IT>(wa + static_cast<IT>(kw))), threadIdx.x & 63u);
    } else if constexpr (MAP == kTileMapSamePhase) {
      spot = tile_spot_same_phase(plan, ta, i0, lim, wa + k);
    } else {
      spot = tile_spot<NOUT>(plan, i0, lim, static_cast<IT>(wa + k));
    }
    uint32_t d[4], v[4];
    philox_block(spot.block, prm.key0, prm.key1, d);
    convert_block<OP, DT>(d, prm, v);
    // Word e of this block sits at tile position rel + e.  A word is written when it is inside
    // both the run and the tile; the other words of edge blocks (and the dead slots of runs that
    // differ in phase) go to the dummy slot.
    const int32_t rel = spot.rel, lo = spot.lo, hi = spot.hi;
    if (rel >= lo && rel + 4 <= hi) {
      // Interior block (nearly all of them): four writes off one address.
#pragma unroll
      for (int e = 0; e < 4; ++e) tile[rel + e] = v[e];
    } else {
      const uint32_t width = static_cast<uint32_t>(hi - lo);  // hi > lo: the run intersects the tile
      const uint32_t base = static_cast<uint32_t>(rel - lo);
#pragma unroll
      for (int e = 0; e < 4; ++e) tile[(base + e < width) ? rel + e : kDummy] = v[e];
    }
  }
  __syncthreads();

  // Stage B: one aligned unit per thread out of LDS.
  if constexpr (OP == kOpRandint) {
    // 16-byte chunks (two integers), consecutive threads on consecutive chunks: every store
    // instruction of a wave writes 1 KiB without gaps.  local_numel is even here or the last
    // element is written alone.
    const uint32_t chunks = (static_cast<uint32_t>(lim) + 1u) >> 1;
    for (uint32_t c = threadIdx.x; c < chunks; c += kThreads) {
      if (2 * c + 1 < static_cast<uint32_t>(lim))
        store_randint_pair(tile[2 * c], tile[2 * c + 1], prm, out, (i0 >> 1) + c);
      else
        static_cast<int64_t*>(out)[i0 + 2 * c] = randint_value(tile[2 * c], prm);
    }
    return;
  }
  // Indices relative to the tile fit 32 bits; the tile's first unit is the same for all threads.
  const uint64_t u0 = static_cast<uint64_t>(blockIdx.x) * ta.tile_units;
  const uint32_t whole = static_cast<uint32_t>(lim) / static_cast<uint32_t>(V);  // whole units of the tile
  for (uint32_t t = threadIdx.x; t < whole; t += kThreads) {
    uint32_t v[V];
#pragma unroll
    for (int q = 0; q < V / 4; ++q) {
      const u32x4 w = *reinterpret_cast<const u32x4*>(&tile[t * V + 4 * q]);
#pragma unroll
      for (int e = 0; e < 4; ++e) v[4 * q + e] = w[e];
    }
    const uint64_t u = u0 + t;
    u32x4 xv = {0u, 0u, 0u, 0u}, rv = {0u, 0u, 0u, 0u};
    if constexpr (kIsDropout<OP>) xv = __builtin_nontemporal_load(static_cast<const u32x4*>(xin) + u);
    if constexpr (OP == kOpDropoutAdd) rv = __builtin_nontemporal_load(static_cast<const u32x4*>(prm.residual) + u);
    emit_unit<OP, DT>(v, prm, xv, rv, u, out, mask);
  }
  // The last unit of a shard whose size is not a multiple of the unit (only the shard's last tile has one).
  if (threadIdx.x == (whole & (kThreads - 1)))
    for (uint32_t i = whole * V; i < static_cast<uint32_t>(lim); ++i)
      emit_element<OP, DT>(tile[i], prm, xin, static_cast<int64_t>(i0 + i), out, mask);
}

// ---- ragged / general kernels ----------------------------------------------------
template <int OP, int DT, typename IT, int NOUT>
__global__ void __launch_bounds__(kThreads)
ragged_kernel(const PlanT<IT> plan, const OpParams prm, const void* xin, void* out, uint8_t* mask) {
  touch_params<OP>(prm);
  const uint64_t t64 = static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x;
  const bool in_range = t64 < plan.total_units;
  const IT w = in_range ? static_cast<IT>(t64) : 0;
  IT run, bi;  // bi: block number inside the run
  uint64_t run_pos;
  locate<NOUT>(plan, w, run, bi, run_pos);
  const BlockSpan<IT> s = block_span(plan, run, bi, run_pos);

  uint32_t d[4];
  philox_block((run_pos >> 2) + bi, prm.key0, prm.key1, d);
#if VESRNG_PIN_ARGUMENT_FETCH
  asm volatile("" : "+v"(d[0]), "+v"(d[1]), "+v"(d[2]), "+v"(d[3]));  // see aligned_kernel
#endif
  if (!in_range || !s.any) return;

  uint32_t v[4];
  convert_block<OP, DT>(d, prm, v);
  // All four values exist before the stores are chosen: otherwise the compiler shares the
  // last value's conversion between the whole-block and the edge path and splits the
  // whole-block store into 12 + 4 bytes.
  asm volatile("" : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]));
  const int64_t li0 = static_cast<int64_t>(s.li0);
#if VESRNG_RAGGED_DPP_REALIGN
  // A wave whose 64 blocks are whole and lie in ONE run holds 256 consecutive local elements that
  // start m = li0 mod 4 elements past a 16-byte boundary.  Instead of 64 element-aligned stores the
  // lanes realign: lane l assembles the aligned unit that starts inside its block from its own
  // last m words and the first 4 - m words of lane l + 1's block (one DPP wave shift per word),
  // lanes 0 .. 62 store aligned vectors, and the m + (4 - m) words at the wave's two ends leave
  // word by word.  m is wave-uniform here, so the three shifts are scalar branches, not selects.
  if constexpr (OP == kOpRaw || ((OP == kOpUniform || OP == kOpNormal) && DT == kF32)) {
    const uint64_t run64 = static_cast<uint64_t>(run);
    const uint32_t run_lo = static_cast<uint32_t>(run64), run_hi = static_cast<uint32_t>(run64 >> 32);
    const bool same = (s.first == 0u && s.last == 4u) && run_lo == first_lane(run_lo) && run_hi == first_lane(run_hi);
    if (__builtin_amdgcn_ballot_w64(same) == ~0ull) {
      const uint32_t m = first_lane(static_cast<uint32_t>(li0) & 3u);
      uint32_t* const dst = static_cast<uint32_t*>(out) + li0;
      if (m == 0u) {
        __builtin_nontemporal_store(u32x4{v[0], v[1], v[2], v[3]}, reinterpret_cast<u32x4*>(dst));
        return;
      }
      const uint32_t lane = threadIdx.x & 63u;
      // next[e]: word e of the block of lane l + 1 (lane 63 keeps its own: not used there).
      uint32_t next[3];
#pragma unroll
      for (int e = 0; e < 3; ++e)
        next[e] = static_cast<uint32_t>(__builtin_amdgcn_update_dpp(static_cast<int>(v[e]), static_cast<int>(v[e]), 0x130,
                                                                    0xF, 0xF, false));
      u32x4 unit;
      if (m == 1u) unit = u32x4{v[3], next[0], next[1], next[2]};
      else if (m == 2u) unit = u32x4{v[2], v[3], next[0], next[1]};
      else unit = u32x4{v[1], v[2], v[3], next[0]};
      if (lane != 63u) __builtin_nontemporal_store(unit, reinterpret_cast<u32x4*>(dst + (4u - m)));
      if (lane == 0u) {
#pragma unroll
        for (uint32_t e = 0; e < 3u; ++e)
          if (e < 4u - m) dst[e] = v[e];
      }
      if (lane == 63u) {
#pragma unroll
        for (uint32_t e = 1; e < 4u; ++e)
          if (e >= 4u - m) dst[e] = v[e];
      }
      return;
    }
  }
#endif
  // Whole blocks of the fills leave as one store that is only element-aligned.
  if constexpr (OP == kOpRaw || OP == kOpUniform || OP == kOpNormal) {
    if (s.first == 0u && s.last == 4u) {
      if constexpr (OP == kOpRaw || DT == kF32) {
        __builtin_nontemporal_store(u32x4{v[0], v[1], v[2], v[3]}, reinterpret_cast<u32x4_align4*>(static_cast<uint32_t*>(out) + li0));
        return;
      } else if ((li0 & 1) == 0) {
        const float a = __uint_as_float(v[0]), b = __uint_as_float(v[1]);
        const float c = __uint_as_float(v[2]), e = __uint_as_float(v[3]);
        const uint32_t p01 = pack16<DT>(a, b), p23 = pack16<DT>(c, e);
        __builtin_nontemporal_store(u32x2{p01, p23}, reinterpret_cast<u32x2_align4*>(static_cast<uint16_t*>(out) + li0));
        return;
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 4; ++e)
    if (static_cast<uint32_t>(e) >= s.first && static_cast<uint32_t>(e) < s.last)
      emit_element<OP, DT>(v[e], prm, xin, li0 + e, out, mask);
}

template <typename Tuple, size_t... I>
void fill_pointers(Tuple& values, void** ptrs, std::index_sequence<I...>) {
  ((ptrs[I] = &std::get<I>(values)), ...);
}

// ---- chain kernel: Algorithm 1 element by element ----------------------------------
// For shards that are not boxes, and for the virtual-thread layout.  One thread per local
// element: decode, map every coordinate back through the placements, one generator block
// per element, word picked.  theta == 0: flat stream (position offset + j).  theta > 0:
// Algorithm 1's "virtualize thread index and offset" to the letter - virtual thread
// tau = j mod theta, virtual offset beta = offset + j / theta, counter
// (lo32 q, hi32 q, lo32 tau, hi32 tau) with q = beta / 4, word beta mod 4.
template <int OP, int DT>
__global__ void __launch_bounds__(kThreads)
chain_kernel(const ChainPlan cp, const uint64_t offset, const uint64_t theta, const uint32_t theta32,
             const uint32_t small, const uint64_t local_numel, const OpParams prm, const void* xin, void* out,
             uint8_t* mask) {
  const uint64_t i = static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (i >= local_numel) return;
  // Wave-uniform choice: the common small plans (<= 4 dimensions, <= 2 placements each, 32-bit
  // extents) take the unrolled map; anything else the general one.
  const uint64_t j = small ? chain_global_index_fixed<4, 2, uint32_t>(cp, static_cast<uint32_t>(i))
                           : chain_global_index(cp, i);
  uint32_t d[4];
  uint32_t word;
  if (theta == 0) {
    const uint64_t p = offset + j;
    philox_block(p >> 2, prm.key0, prm.key1, d);
    word = static_cast<uint32_t>(p) & 3u;
  } else {
    // theta32: theta and every global index are below 2^32, so the division can be a 32-bit one.
    const uint64_t step = theta32 ? static_cast<uint64_t>(static_cast<uint32_t>(j) / static_cast<uint32_t>(theta))
                                  : j / theta;
    const uint64_t tau = j - step * theta;
    const uint64_t beta = offset + step;
    const uint64_t q = beta >> 2;
    philox_rounds(static_cast<uint32_t>(q), static_cast<uint32_t>(q >> 32), static_cast<uint32_t>(tau),
                  static_cast<uint32_t>(tau >> 32), prm.key0, prm.key1, d);
    word = static_cast<uint32_t>(beta) & 3u;
  }
  // Only one word of the block is this element's: pick the draw (for a normal, its pair) first
  // and convert that alone.  The conversions are the ones convert_block applies.
  uint32_t value;
  if constexpr (OP == kOpNormal) {
    const bool upper = (word & 2u) != 0u;
    float even, odd;
    normal_pair(upper ? d[2] : d[0], upper ? d[3] : d[1], prm, even, odd);
    value = __float_as_uint((word & 1u) ? odd : even);
  } else {
    const uint32_t x = word == 0u ? d[0] : word == 1u ? d[1] : word == 2u ? d[2] : d[3];
    if constexpr (OP == kOpUniform)
      value = __float_as_uint(prm.unit_range ? uniform_unit<DT>(x, prm) : uniform_general(x, prm));
    else
      value = x;
  }
  emit_element<OP, DT>(value, prm, xin, static_cast<int64_t>(i), out, mask);
}

// ---- virtual-thread layout, one generator call per four outputs ---------------------
// Thread (g, c) owns column c (V consecutive virtual threads tau = c V .. c V + V - 1) of step
// group g: V generator blocks, whose word k belongs to step 4 g + k, i.e. to the aligned unit
// that starts at global index (4 g + k) Theta + c V.  Units outside the shard are skipped; the
// shard's last unit may be partial.
template <int OP, int DT>
__global__ void __launch_bounds__(kThreads)
theta_kernel(const ThetaPlan tp, const OpParams prm, const void* xin, void* out, uint8_t* mask) {
  constexpr int V = UnitOf<OP, DT>::kElems;
  touch_params<OP>(prm);
  const uint64_t t = static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (t >= tp.total_threads) return;
  const uint32_t gi = tp.cols_div.div(static_cast<uint32_t>(t));
  const uint64_t c = static_cast<uint32_t>(t) - gi * static_cast<uint32_t>(tp.cols);
  const uint64_t group = tp.group0 + gi;
  const uint64_t block = tp.block0 + group;      // the same for all V virtual threads
  const uint64_t tau0 = c * V;

  // The four units of this thread: step 4 group + k starts at global index (4 group + k) Theta + tau0.
  uint64_t unit[4];
  bool inside[4], whole[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const uint64_t j = (4 * group + static_cast<uint64_t>(k)) * tp.theta + tau0;
    // origin and j are multiples of V: a unit lies wholly below the shard or starts inside/above it.
    const uint64_t i = j - tp.origin;
    inside[k] = j >= tp.origin && i < tp.local_numel;
    whole[k] = inside[k] && i + V <= tp.local_numel;
    unit[k] = inside[k] ? i / V : 0;
  }
  u32x4 xv[4], rv[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    xv[k] = u32x4{0u, 0u, 0u, 0u};
    rv[k] = u32x4{0u, 0u, 0u, 0u};
    if constexpr (kIsDropout<OP>)
      if (whole[k]) xv[k] = __builtin_nontemporal_load(static_cast<const u32x4*>(xin) + unit[k]);
    if constexpr (OP == kOpDropoutAdd)
      if (whole[k]) rv[k] = __builtin_nontemporal_load(static_cast<const u32x4*>(prm.residual) + unit[k]);
  }

  // cv[e][k]: converted value of word k of virtual thread tau0 + e (for a normal the pairs are the
  // words (0,1) and (2,3) of a block, i.e. steps 4 g, 4 g + 1 and 4 g + 2, 4 g + 3 of one thread).
  uint32_t cv[V][4];
#pragma unroll
  for (int e = 0; e < V; ++e) {
    const uint64_t tau = tau0 + static_cast<uint64_t>(e);
    uint32_t d[4];
    philox_rounds(static_cast<uint32_t>(block), static_cast<uint32_t>(block >> 32), static_cast<uint32_t>(tau),
                  static_cast<uint32_t>(tau >> 32), prm.key0, prm.key1, d);
    convert_block<OP, DT>(d, prm, cv[e]);
  }
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    if (!inside[k]) continue;
    uint32_t v[V];
#pragma unroll
    for (int e = 0; e < V; ++e) v[e] = cv[e][k];
    if (whole[k]) {
      emit_unit<OP, DT>(v, prm, xv[k], rv[k], unit[k], out, mask);
    } else {
      const uint64_t i0 = unit[k] * V;
#pragma unroll
      for (int e = 0; e < V - 1; ++e)
        if (i0 + static_cast<uint64_t>(e) < tp.local_numel)
          emit_element<OP, DT>(v[e], prm, xin, static_cast<int64_t>(i0 + e), out, mask);
    }
  }
}

// Enqueues `kernel` and returns the launch's own status (hipGetLastError would also report,
// and clear, an error some other code left behind).
// `unused_lds_bytes` of dynamic LDS that the kernel never touches limit how many workgroups a compute unit holds
// at once (160 KiB of LDS per compute unit).
template <typename... Params, typename... Args>
hipError_t enqueue_with_lds(void (*kernel)(Params...), dim3 grid, dim3 block, size_t unused_lds_bytes, hipStream_t stream,
                            Args... args) {
  static_assert(sizeof...(Params) == sizeof...(Args), "one argument per kernel parameter");
  std::tuple<std::remove_cv_t<Params>...> values{args...};
  void* ptrs[sizeof...(Params)];
  fill_pointers(values, ptrs, std::index_sequence_for<Params...>{});
  return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, unused_lds_bytes, stream);
}
template <typename... Params, typename... Args>
hipError_t enqueue(void (*kernel)(Params...), dim3 grid, dim3 block, hipStream_t stream, Args... args) {
  return enqueue_with_lds(kernel, grid, block, 0, stream, args...);
}

// Seven resident waves per SIMD instead of eight for fused dropout WITH a mask, on launches that stream far more than
// the last-level cache holds: a workgroup is four waves, one per SIMD, so a compute unit holds eight workgroups; 21 KiB
// of untouched dynamic LDS each let seven fit in its 160 KiB.  Measured in one run on 2^29-element shards: bf16 dropout
// with mask 6.52 -> 6.67 TB/s, fp32 with mask 6.53 -> 6.64; six waves gain less (6.65), five lose a tenth.  The same
// cap costs the kernels with ONE store stream (fills, dropout without mask: -0.3 to -1.7 %) and the launches that fit
// the cache (-0.7 % on 17 M elements), so only these take it.
constexpr size_t kWaveCapLdsBytes = 21 * 1024;
constexpr uint64_t kWaveCapMinUnits = 1ull << 23;

template <int OP, int DT>
hipError_t launch_chain(const Geometry& g, uint64_t offset, const OpParams& prm, const void* x, void* out,
                        uint8_t* mask, hipStream_t stream) {
  const uint64_t n = static_cast<uint64_t>(g.local_numel);
  const uint64_t blocks = (n + kThreads - 1) / kThreads;
  if (blocks > 0x7FFFFFFFull) return hipErrorInvalidConfiguration;
  const uint32_t theta32 = ((g.virtual_threads | g.max_global_index) >> 32) == 0 ? 1u : 0u;
  uint32_t small = (g.chain.fits32 && g.chain.ndim <= 4) ? 1u : 0u;
  for (int d = 0; d < g.chain.ndim; ++d)
    if (g.chain.nsteps[d] > 2) small = 0u;
  return enqueue(chain_kernel<OP, DT>, dim3(static_cast<uint32_t>(blocks)), dim3(kThreads), stream, g.chain, offset,
                 g.virtual_threads, theta32, small, n, prm, x, out, mask);
}

// ---- dispatch --------------------------------------------------------------------
// Which kernel a shard takes is decided on the host by choose_launch (geometry.cpp); the traits
// below say what each operator can use.
// Which ragged shards take the staging kernel, operator by operator (measured on column shards of 0.7 M to 358 M
// elements with runs of 100 to 3414 elements, GPU-side time per launch in graph replays):
//  * raw, randint, fused dropout, fp32 uniform: every shard with runs of 16 elements and more.  Staging doubles the rate
//    of bf16 dropout (5.9 vs 2.4 TB/s) and lifts the raw fill from 4.8 to 6.1-6.7 and the fp32 uniform fill to 5.9-6.3.
//  * fp32 normal: shards below 2^24 elements (10-20 % less time from 0.7 M to 11 M elements - C2's 5.6 M: 7.3 -> 6.0 us -,
//    level from 22 M on, where the kernel without staging stays: both are bound by instruction issue there).
//  * 16-bit uniform and normal: shards of 2^21 .. 2^25 elements with runs of 256 elements and more (5-26 % less time;
//    below, the launch is too small to matter and staging costs a barrier; above, two generator blocks per 16 bytes
//    make both forms issue-bound and the kernel without staging is 3-10 % ahead; short runs lose up to 10 %).
#if VESRNG_TILING == -1
template <int OP, int DT>
constexpr bool kTileable = true;
template <int OP, int DT>
constexpr uint64_t kTileMinElems = ((OP == kOpUniform || OP == kOpNormal) && DT != kF32) ? (1ull << 21) : 0;
template <int OP, int DT>
constexpr uint64_t kTileMaxElems = (OP == kOpNormal && DT == kF32)                          ? (1ull << 24)
                                   : ((OP == kOpUniform || OP == kOpNormal) && DT != kF32) ? (1ull << 25)
                                                                                            : 0;  // 0: no upper limit
template <int OP, int DT>
constexpr uint64_t kTileMinRunLen = ((OP == kOpUniform || OP == kOpNormal) && DT != kF32) ? 256 : 16;
#else
template <int OP, int DT>
constexpr bool kTileable = (VESRNG_TILING != 0);
template <int OP, int DT>
constexpr uint64_t kTileMinElems = 0;
template <int OP, int DT>
constexpr uint64_t kTileMaxElems = 0;
template <int OP, int DT>
constexpr uint64_t kTileMinRunLen = 16;
#endif
// Four aligned units per thread in the store stage (a four times larger tile): the fills of 4-byte elements gain from
// it on all but small shards (measured with the short tile map: raw 3.7-5.3 -> 4.0-6.6 TB/s, fp32 uniform 3.6-5.1 ->
// 3.9-6.3, fp32 normal 6.4 -> 6.1 us on C2's shard); on small shards the four times fewer workgroups no longer fill
// the chip.  Dropout and randint, which issue more memory instructions per unit, lose with the large tile and keep
// one unit; the 16-bit fills have no large form (their unit is already two generator blocks).
template <int OP, int DT>
constexpr bool kBigTileable = (VESRNG_TILING == -1 || VESRNG_TILING == 2) &&
                              ((OP == kOpRaw || OP == kOpUniform || OP == kOpNormal) && UnitOf<OP, DT>::kElems == 4);
// Smallest shard that takes the big tile (measured: level at 2.8 M elements, 6 % ahead at 5.6 M).
#ifdef VESRNG_BIG_TILE_MIN_ELEMS  // measurement variants only: force one tile size
template <int OP>
constexpr uint64_t kBigTileMinElems = VESRNG_BIG_TILE_MIN_ELEMS;
#else
template <int OP>
constexpr uint64_t kBigTileMinElems = 1ull << 22;
#endif

template <int OP, int DT, typename IT, int NOUT, int UPT>
hipError_t launch_tiled(const PlanT<IT>& plan, uint64_t tile_units, uint64_t local_numel, dim3 grid, dim3 block,
                        const OpParams& prm, const void* x, void* out, uint8_t* mask, hipStream_t stream) {
  const TileArgs<IT> ta = make_tile_args(plan, tile_units, local_numel);
  if constexpr (VESRNG_TILE_WAVE_MAP != 0)
    if (static_cast<uint64_t>(plan.units_per_run) >= kTileWaveMinBlocks)
      return enqueue(tiled_kernel<OP, DT, IT, NOUT, UPT, kTileMapWave>, grid, block, stream, plan, prm, ta, x, out,
                     mask);
  if constexpr (VESRNG_TILE_SAME_PHASE != 0 && NOUT == 1 && std::is_same<IT, uint32_t>::value)
    if (ta.same_phase)
      return enqueue(tiled_kernel<OP, DT, IT, NOUT, UPT, kTileMapSamePhase>, grid, block, stream, plan, prm, ta, x, out,
                     mask);
  return enqueue(tiled_kernel<OP, DT, IT, NOUT, UPT, kTileMapBlock>, grid, block, stream, plan, prm, ta, x, out, mask);
}

template <int OP, int DT, typename IT, int NOUT>
hipError_t launch_nout(Flavour flavour, const PlanT<IT>& plan, uint64_t tile_units, uint64_t local_numel,
                       const OpParams& prm, const void* x, void* out, uint8_t* mask, hipStream_t stream) {
  constexpr uint64_t V = UnitOf<OP, DT>::kElems;
  uint64_t blocks;
  if (flavour == kTiled || flavour == kTiledBig)
    blocks = (local_numel + tile_units * V - 1) / (tile_units * V);
  else if (OP == kOpRandint && VESRNG_RANDINT_HALF_BLOCKS != 0 && flavour == kAligned)
    blocks = (2 * plan.total_units + kThreads - 1) / kThreads;
  else
    blocks = (plan.total_units + kThreads - 1) / kThreads;
  if (blocks == 0) return hipSuccess;
  if (blocks > 0x7FFFFFFFull) return hipErrorInvalidConfiguration;
  const dim3 grid(static_cast<uint32_t>(blocks)), block(kThreads);
  switch (flavour) {
    case kAligned: {
      size_t cap = 0;
      if constexpr (kIsDropout<OP> && VESRNG_CAP_MASKED_DROPOUT_WAVES != 0)
        if (mask != nullptr && plan.total_units >= kWaveCapMinUnits) cap = kWaveCapLdsBytes;
      if constexpr (NOUT != 0 && VESRNG_WAVE_UNIFORM_RUNS != 0 && !(OP == kOpRandint && VESRNG_RANDINT_HALF_BLOCKS != 0))
        if (plan.wave_runs)
          return enqueue_with_lds(aligned_kernel<OP, DT, IT, NOUT, true>, grid, block, cap, stream, plan, prm, x, out,
                                  mask);
      return enqueue_with_lds(aligned_kernel<OP, DT, IT, NOUT, false>, grid, block, cap, stream, plan, prm, x, out,
                              mask);
    }
    case kTiled:
      if constexpr (kTileable<OP, DT>)
        return launch_tiled<OP, DT, IT, NOUT, 1>(plan, tile_units, local_numel, grid, block, prm, x, out, mask, stream);
      break;
    case kTiledBig:
      if constexpr (kBigTileable<OP, DT>)
        return launch_tiled<OP, DT, IT, NOUT, kBigTileUnits>(plan, tile_units, local_numel, grid, block, prm, x, out, mask,
                                                             stream);
      break;
    case kRagged:
      return enqueue(ragged_kernel<OP, DT, IT, NOUT>, grid, block, stream, plan, prm, x, out, mask);
  }
  return hipErrorInvalidValue;
}

// `n`: local elements the launch covers (the whole shard, or one piece of it).
template <int OP, int DT, typename IT>
hipError_t launch_typed(Flavour flavour, const Geometry& g, const RunShape& rs, uint64_t n, uint64_t offset,
                        uint64_t units_per_run, uint64_t tile_units, const OpParams& prm, const void* x, void* out,
                        uint8_t* mask, hipStream_t stream) {
  const PlanT<IT> plan = make_plan<IT>(g, rs, offset, units_per_run);
  switch (plan.n_outer) {
    case 0: return launch_nout<OP, DT, IT, 0>(flavour, plan, tile_units, n, prm, x, out, mask, stream);
    case 1: return launch_nout<OP, DT, IT, 1>(flavour, plan, tile_units, n, prm, x, out, mask, stream);
    case 2:
      if constexpr (VESRNG_EXACT_RUN_AXES >= 2)
        return launch_nout<OP, DT, IT, 2>(flavour, plan, tile_units, n, prm, x, out, mask, stream);
      break;
    case 3:
      if constexpr (VESRNG_EXACT_RUN_AXES >= 3)
        return launch_nout<OP, DT, IT, 3>(flavour, plan, tile_units, n, prm, x, out, mask, stream);
      break;
    default: break;
  }
  return launch_nout<OP, DT, IT, kAnyAxes>(flavour, plan, tile_units, n, prm, x, out, mask, stream);
}

template <int OP, int DT>
hipError_t launch_dt(const Geometry& g, uint64_t offset, const OpParams& prm, const void* x, void* out,
                     uint8_t* mask, hipStream_t stream) {
  if (g.boxed && g.virtual_threads != 0) {
    ThetaPlan tp;
    if (plan_theta(g, run_shape(g), offset, UnitOf<OP, DT>::kElems, &tp)) {
      const uint64_t blocks = (tp.total_threads + kThreads - 1) / kThreads;
      if (blocks > 0x7FFFFFFFull) return hipErrorInvalidConfiguration;
      return enqueue(theta_kernel<OP, DT>, dim3(static_cast<uint32_t>(blocks)), dim3(kThreads), stream, tp, prm, x, out,
                     mask);
    }
  }
  if (!g.boxed || g.virtual_threads != 0) return launch_chain<OP, DT>(g, offset, prm, x, out, mask, stream);
  const RunShape rs = run_shape(g);
  LaunchTraits traits;
  traits.unit_elems = UnitOf<OP, DT>::kElems;
  traits.tileable = kTileable<OP, DT>;
  traits.big_tileable = kBigTileable<OP, DT>;
  traits.big_tile_min_elems = kBigTileMinElems<OP>;
  traits.tile_min_elems = kTileMinElems<OP, DT>;
  traits.tile_max_elems = kTileMaxElems<OP, DT>;
  traits.tile_min_run_len = kTileMinRunLen<OP, DT>;
  traits.whole_blocks_only = (OP == kOpRandint);
  const LaunchChoice c = choose_launch(g, rs, offset, traits);
  const uint64_t n = static_cast<uint64_t>(g.local_numel);
  if (!c.wide)
    return launch_typed<OP, DT, uint32_t>(c.flavour, g, rs, n, offset, c.units_per_run, c.tile_units, prm, x, out, mask, stream);
  // A shard that needs 64-bit indices as a whole: piece by piece through the 32-bit kernels where it can be cut
  // (geometry.hpp: Pieces), one launch per piece, each on its own part of every buffer.
  Pieces pc;
  if (VESRNG_WIDE_SHARDS_IN_PIECES != 0 && plan_pieces(rs, c.units_per_run, &pc)) {
    constexpr uint64_t out_bytes = (OP == kOpRandint) ? 8 : (OP == kOpRaw || DT == kF32) ? 4 : 2;
    constexpr uint64_t x_bytes = (DT == kF32) ? 4 : 2;
    for (uint64_t row = 0; row < pc.extent; row += pc.rows_per_piece) {
      const uint64_t rows = (pc.extent - row < pc.rows_per_piece) ? pc.extent - row : pc.rows_per_piece;
      const uint64_t first = row * pc.per_index;  // first local element of the piece
      OpParams piece_prm = prm;
      if (prm.residual) piece_prm.residual = static_cast<const char*>(prm.residual) + first * x_bytes;
      const hipError_t e = launch_typed<OP, DT, uint32_t>(
          c.flavour, g, piece_shape(rs, rows), rows * pc.per_index, offset + row * pc.stride, c.units_per_run, c.tile_units,
          piece_prm, x ? static_cast<const char*>(x) + first * x_bytes : nullptr, static_cast<char*>(out) + first * out_bytes,
          mask ? mask + first : nullptr, stream);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  return launch_typed<OP, DT, uint64_t>(c.flavour, g, rs, n, offset, c.units_per_run, c.tile_units, prm, x, out, mask, stream);
}

// The floating-point operators, by output dtype.
template <int OP>
hipError_t launch_float(const Geometry& g, uint64_t offset, const OpParams& prm, const void* x, void* out,
                        uint8_t* mask, hipStream_t stream) {
  switch (prm.dtype) {
    case kF32: return launch_dt<OP, kF32>(g, offset, prm, x, out, mask, stream);
    case kBF16: return launch_dt<OP, kBF16>(g, offset, prm, x, out, mask, stream);
    case kF16: return launch_dt<OP, kF16>(g, offset, prm, x, out, mask, stream);
  }
  return hipErrorInvalidValue;
}

#ifdef VESRNG_VARIANT_TAG
}  // inline namespace
#endif
}  // namespace

hipError_t launch_op(OpKind op, const Geometry& g, uint64_t offset, const OpParams& prm, const void* x, void* out,
                     uint8_t* mask, hipStream_t stream) {
  if (g.local_numel == 0) return hipSuccess;
  switch (op) {
    case kOpRaw: return launch_dt<kOpRaw, kF32>(g, offset, prm, x, out, mask, stream);
    case kOpRandint: return launch_dt<kOpRandint, kF32>(g, offset, prm, x, out, mask, stream);
    case kOpUniform: return launch_float<kOpUniform>(g, offset, prm, x, out, mask, stream);
    case kOpNormal: return launch_float<kOpNormal>(g, offset, prm, x, out, mask, stream);
    case kOpDropout: return launch_float<kOpDropout>(g, offset, prm, x, out, mask, stream);
    case kOpDropoutAdd: return launch_float<kOpDropoutAdd>(g, offset, prm, x, out, mask, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace vesrng
