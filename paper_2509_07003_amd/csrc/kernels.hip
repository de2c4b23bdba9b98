// gfx950 kernels of the sharded random fill / fused dropout path
// (veScale Section 5, Algorithm 1, with Philox4x32-10 as the generator).
//
// Work decomposition.  Algorithm 1 walks local elements one by one.  Here a
// thread owns one generator block (4 consecutive stream positions, hence 4
// consecutive global elements) or two of them, so that one Philox call feeds
// four outputs that stay in registers and leave as one 128-bit store.
//
//  * aligned kernels: every run of the shard starts on a block boundary and its
//    length is a multiple of the unit (4 or 8 elements); unit w covers local
//    elements [w*V, (w+1)*V) and all accesses are 16-byte vectors.
//  * ragged kernels: any run start / length; a thread still owns one global
//    block and stores only the lanes that fall inside the run (e.g. a column
//    shard whose first column is 1366).  They also serve as the general path.
//
// The launch is one-shot (one unit per thread): on MI355X this sustained a higher
// store rate than a grid-stride loop over the same bytes.
#include <hip/hip_runtime.h>

#include "launch.hpp"
#include "plan.h"

namespace vesrng {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
// 16 bytes that are only 4-byte aligned: row starts of a ragged fp32 shard.
struct __attribute__((packed, aligned(4))) U32x4Unaligned {
  uint32_t a, b, c, d;
};

constexpr int kThreads = 256;
constexpr int kF32 = 0, kBF16 = 1;

// ---- generator ---------------------------------------------------------------
// a ^ b ^ c in one instruction (v_bitop3_b32, truth table 0x96); the compiler emits two
// v_xor_b32 for the plain expression, and the XORs are half of Philox's instructions.
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
  return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// Philox4x32-10 on counter (lo32 b, hi32 b, 0, 0), key (k0, k1).
__device__ __forceinline__ void philox_block(uint64_t b, uint32_t k0, uint32_t k1, uint32_t (&w)[4]) {
  uint32_t c0 = static_cast<uint32_t>(b), c1 = static_cast<uint32_t>(b >> 32), c2 = 0u, c3 = 0u;
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = static_cast<uint64_t>(0xD2511F53u) * c0;
    const uint64_t p1 = static_cast<uint64_t>(0xCD9E8D57u) * c2;
    const uint32_t n0 = xor3(static_cast<uint32_t>(p1 >> 32), c1, k0);
    const uint32_t n2 = xor3(static_cast<uint32_t>(p0 >> 32), c3, k1);
    c1 = static_cast<uint32_t>(p1);
    c3 = static_cast<uint32_t>(p0);
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;  // wave-uniform: lives in scalar registers
    k1 += 0xBB67AE85u;
  }
  w[0] = c0;
  w[1] = c1;
  w[2] = c2;
  w[3] = c3;
}

// ---- conversions ---------------------------------------------------------------
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));  // v_cvt_pk_bf16_f32, RNE
}
__device__ __forceinline__ float bf16_lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t pair) { return __uint_as_float(pair & 0xFFFF0000u); }

__device__ __forceinline__ float fraction24(uint32_t x) {
  return static_cast<float>(x >> 8) * 0x1p-24f;  // exact
}

__device__ __forceinline__ float uniform_value(uint32_t x, const OpParams& prm) {
  const float scaled = __fmul_rn(fraction24(x), prm.width);
  const float r = __fadd_rn(scaled, prm.low);
  return r >= prm.high ? prm.top_f32 : r;
}

// bfloat16 bits of one uniform (upper guard applied after rounding).
__device__ __forceinline__ uint32_t uniform_bf16_pair(uint32_t xa, uint32_t xb, const OpParams& prm) {
  uint32_t pair = pack_bf16(uniform_value(xa, prm), uniform_value(xb, prm));
  if (bf16_lo(pair) >= prm.high) pair = (pair & 0xFFFF0000u) | prm.top_bf16;
  if (bf16_hi(pair) >= prm.high) pair = (pair & 0x0000FFFFu) | (prm.top_bf16 << 16);
  return pair;
}

// Box-Muller on one draw pair; hardware log2 / sqrt / sin / cos (sin and cos take
// their argument in revolutions, which is exactly u2).
__device__ __forceinline__ void normal_pair(uint32_t xa, uint32_t xb, const OpParams& prm, float& even,
                                            float& odd) {
  const float u1 = (static_cast<float>(xa >> 8) + 1.0f) * 0x1p-24f;  // (0, 1], exact
  const float u2 = fraction24(xb);                                    // [0, 1), exact
  const float r2 = __fmul_rn(__builtin_amdgcn_logf(u1), -1.3862943611198906f);  // -2 ln u1
  const float radius = __builtin_amdgcn_sqrtf(r2);
  const float c = __builtin_amdgcn_cosf(u2);
  const float s = __builtin_amdgcn_sinf(u2);
  even = __fmaf_rn(__fmul_rn(radius, c), prm.stddev, prm.mean);
  odd = __fmaf_rn(__fmul_rn(radius, s), prm.stddev, prm.mean);
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

// ---- aligned kernels -----------------------------------------------------------
// OP: OpKind.  DT: output dtype.  One thread = one unit of V elements.
template <int OP, int DT>
struct UnitOf {
  static constexpr int kBlocks = (OP != kOpRaw && OP != kOpRandint && DT == kBF16) ? 2 : 1;
  static constexpr int kElems = 4 * kBlocks;
};

// Position (stream position of the first element) of work unit `w`.  NOUT is the number
// of run-enumerating axes known at compile time (0, 1) or 2 for "any number": the common
// shards (a contiguous slice; one strided axis of runs) then need no loop and no loads
// that depend on a loop counter.
template <int NOUT, typename IT>
__device__ __forceinline__ void locate(const PlanT<IT>& plan, IT w, IT& run, IT& unit, uint64_t& run_pos) {
  if constexpr (NOUT == 0) {
    run = 0;
    unit = w;
    run_pos = plan.pos0;
  } else {
    run = plan.units_div.div(w);
    unit = w - run * plan.units_per_run;
    if constexpr (NOUT == 1)
      run_pos = plan.pos0 + static_cast<uint64_t>(run) * plan.outer_stride[0];
    else
      run_pos = plan.pos0 + run_offset(plan, run);
  }
}

template <int OP, int DT, typename IT, int NOUT>
__global__ void __launch_bounds__(kThreads)
aligned_kernel(const PlanT<IT> plan, const OpParams prm, const void* xin, void* out, uint8_t* mask) {
  constexpr int NB = UnitOf<OP, DT>::kBlocks;
  constexpr int V = UnitOf<OP, DT>::kElems;
  // Threads past the end compute unit 0 again and skip the stores: no early exit, so all
  // kernel arguments are fetched in one batch at the top.
  const uint64_t t64 = static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x;
  const bool live = t64 < plan.total_units;
  const uint64_t w64 = live ? t64 : 0;
  const IT w = static_cast<IT>(w64);
  IT run, unit;
  uint64_t run_pos;
  locate<NOUT>(plan, w, run, unit, run_pos);
  const uint64_t block0 = (run_pos + static_cast<uint64_t>(unit) * V) >> 2;

  // Dropout: issue the load before the generator so that it overlaps the ALU work.
  u32x4 xv = {0u, 0u, 0u, 0u};
  if constexpr (OP == kOpDropout) xv = __builtin_nontemporal_load(static_cast<const u32x4*>(xin) + w64);

  uint32_t d[NB][4];
#pragma unroll
  for (int b = 0; b < NB; ++b) philox_block(block0 + b, prm.key0, prm.key1, d[b]);
  // Keep the generator (and the argument loads it needs) ahead of the bounds branch: without
  // this the compiler sinks everything below the branch and fetches the arguments in two
  // dependent rounds.
#pragma unroll
  for (int b = 0; b < NB; ++b) asm volatile("" : "+v"(d[b][0]), "+v"(d[b][1]), "+v"(d[b][2]), "+v"(d[b][3]));
  if constexpr (OP == kOpDropout) asm volatile("" : "+v"(xv));
  if (!live) return;

  if constexpr (OP == kOpRaw) {
    const u32x4 v = {d[0][0], d[0][1], d[0][2], d[0][3]};
    __builtin_nontemporal_store(v, static_cast<u32x4*>(out) + w64);
  } else if constexpr (OP == kOpRandint) {
    int64_t r[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) r[e] = randint_value(d[0][e], prm);
    u32x4 lo = {static_cast<uint32_t>(r[0]), static_cast<uint32_t>(static_cast<uint64_t>(r[0]) >> 32),
                static_cast<uint32_t>(r[1]), static_cast<uint32_t>(static_cast<uint64_t>(r[1]) >> 32)};
    u32x4 hi = {static_cast<uint32_t>(r[2]), static_cast<uint32_t>(static_cast<uint64_t>(r[2]) >> 32),
                static_cast<uint32_t>(r[3]), static_cast<uint32_t>(static_cast<uint64_t>(r[3]) >> 32)};
    __builtin_nontemporal_store(lo, static_cast<u32x4*>(out) + 2 * w64);
    __builtin_nontemporal_store(hi, static_cast<u32x4*>(out) + 2 * w64 + 1);
  } else if constexpr (OP == kOpUniform) {
    u32x4 v;
    if constexpr (DT == kF32) {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = __float_as_uint(uniform_value(d[0][e], prm));
    } else {
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        v[2 * b] = uniform_bf16_pair(d[b][0], d[b][1], prm);
        v[2 * b + 1] = uniform_bf16_pair(d[b][2], d[b][3], prm);
      }
    }
    __builtin_nontemporal_store(v, static_cast<u32x4*>(out) + w64);
  } else if constexpr (OP == kOpNormal) {
    u32x4 v;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      float n[4];
      normal_pair(d[b][0], d[b][1], prm, n[0], n[1]);
      normal_pair(d[b][2], d[b][3], prm, n[2], n[3]);
      if constexpr (DT == kF32) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = __float_as_uint(n[e]);
      } else {
        v[2 * b] = pack_bf16(n[0], n[1]);
        v[2 * b + 1] = pack_bf16(n[2], n[3]);
      }
    }
    __builtin_nontemporal_store(v, static_cast<u32x4*>(out) + w64);
  } else if constexpr (OP == kOpDropout) {
    u32x4 y;
    if constexpr (DT == kF32) {
      uint32_t m = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool keep = keep_of(d[0][e], prm);
        const float prod = __fmul_rn(__uint_as_float(xv[e]), prm.scale);
        y[e] = keep ? __float_as_uint(prod) : 0u;
        m |= (keep ? 1u : 0u) << (8 * e);
      }
      __builtin_nontemporal_store(y, static_cast<u32x4*>(out) + w64);
      if (mask) __builtin_nontemporal_store(m, reinterpret_cast<uint32_t*>(mask) + w64);
    } else {
      u32x2 m = {0u, 0u};
#pragma unroll
      for (int b = 0; b < NB; ++b) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {  // two packed pairs per block
          const uint32_t pair = xv[2 * b + h];
          const bool k0 = keep_of(d[b][2 * h], prm), k1 = keep_of(d[b][2 * h + 1], prm);
          const float p0 = __fmul_rn(bf16_lo(pair), prm.scale);
          const float p1 = __fmul_rn(bf16_hi(pair), prm.scale);
          // Select before rounding: a dropped element becomes +0 whatever x held.
          y[2 * b + h] = pack_bf16(k0 ? p0 : 0.0f, k1 ? p1 : 0.0f);
          m[b] |= ((k0 ? 1u : 0u) | (k1 ? 0x100u : 0u)) << (16 * h);
        }
      }
      __builtin_nontemporal_store(y, static_cast<u32x4*>(out) + w64);
      if (mask) __builtin_nontemporal_store(m, reinterpret_cast<u32x2*>(mask) + w64);
    }
  }
}

// ---- ragged / general kernels ----------------------------------------------------
template <typename IT>
struct SignedOf;
template <>
struct SignedOf<uint32_t> {
  using type = int32_t;
};
template <>
struct SignedOf<uint64_t> {
  using type = int64_t;
};

template <int OP, int DT, typename IT, int NOUT>
__global__ void __launch_bounds__(kThreads)
ragged_kernel(const PlanT<IT> plan, const OpParams prm, const void* xin, void* out, uint8_t* mask) {
  using ST = typename SignedOf<IT>::type;
  const uint64_t t64 = static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x;
  const bool in_range = t64 < plan.total_units;
  const IT w = in_range ? static_cast<IT>(t64) : 0;
  IT run, bi;  // bi: block number inside the run
  uint64_t run_pos;
  locate<NOUT>(plan, w, run, bi, run_pos);
  const uint32_t phase = static_cast<uint32_t>(run_pos) & 3u;
  // Elements of the run from this block's lane 0 onwards (lane 0 may lie before the run).
  // Not positive only when runs differ in phase and units_per_run is the upper bound.
  const ST remaining = static_cast<ST>(phase + plan.run_len) - static_cast<ST>(4 * bi);
  const bool live = in_range && remaining > 0;
  // Lanes [first, last) of this block belong to the run.
  const uint32_t first = (bi == 0) ? phase : 0u;
  const uint32_t last = remaining < 4 ? static_cast<uint32_t>(remaining) : 4u;
  // Local flat index of lane 0 (negative for the very first block of a shard with phase > 0:
  // only valid lanes are touched).
  const int64_t li0 = static_cast<int64_t>(static_cast<ST>(run * plan.run_len + 4 * bi) - static_cast<ST>(phase));

  uint32_t d[4];
  philox_block((run_pos >> 2) + bi, prm.key0, prm.key1, d);
  asm volatile("" : "+v"(d[0]), "+v"(d[1]), "+v"(d[2]), "+v"(d[3]));  // see aligned_kernel
  if (!live) return;

  const bool full = (first == 0u) && (last == 4u);
  if constexpr (OP == kOpRaw) {
    uint32_t* o = static_cast<uint32_t*>(out) + li0;
    if (full) {
      *reinterpret_cast<U32x4Unaligned*>(o) = U32x4Unaligned{d[0], d[1], d[2], d[3]};
    } else {
#pragma unroll
      for (uint32_t e = 0; e < 4; ++e)
        if (e >= first && e < last) o[e] = d[e];
    }
  } else if constexpr (OP == kOpRandint) {
    int64_t* o = static_cast<int64_t*>(out) + li0;
#pragma unroll
    for (uint32_t e = 0; e < 4; ++e)
      if (e >= first && e < last) o[e] = randint_value(d[e], prm);
  } else if constexpr (OP == kOpUniform || OP == kOpNormal) {
    float v[4];
    if constexpr (OP == kOpUniform) {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = uniform_value(d[e], prm);
    } else {
      normal_pair(d[0], d[1], prm, v[0], v[1]);
      normal_pair(d[2], d[3], prm, v[2], v[3]);
    }
    if constexpr (DT == kF32) {
      float* o = static_cast<float*>(out) + li0;
      if (full) {
        *reinterpret_cast<U32x4Unaligned*>(o) = U32x4Unaligned{__float_as_uint(v[0]), __float_as_uint(v[1]),
                                                               __float_as_uint(v[2]), __float_as_uint(v[3])};
      } else {
#pragma unroll
        for (uint32_t e = 0; e < 4; ++e)
          if (e >= first && e < last) o[e] = v[e];
      }
    } else {
      uint32_t p01, p23;
      if constexpr (OP == kOpUniform) {
        p01 = uniform_bf16_pair(d[0], d[1], prm);
        p23 = uniform_bf16_pair(d[2], d[3], prm);
      } else {
        p01 = pack_bf16(v[0], v[1]);
        p23 = pack_bf16(v[2], v[3]);
      }
      const uint16_t h[4] = {static_cast<uint16_t>(p01), static_cast<uint16_t>(p01 >> 16),
                             static_cast<uint16_t>(p23), static_cast<uint16_t>(p23 >> 16)};
      uint16_t* o = static_cast<uint16_t*>(out) + li0;
#pragma unroll
      for (uint32_t e = 0; e < 4; ++e)
        if (e >= first && e < last) o[e] = h[e];
    }
  } else if constexpr (OP == kOpDropout) {
    if constexpr (DT == kF32) {
      const float* xi = static_cast<const float*>(xin) + li0;
      float* o = static_cast<float*>(out) + li0;
      float xv[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (uint32_t e = 0; e < 4; ++e)
        if (e >= first && e < last) xv[e] = xi[e];
#pragma unroll
      for (uint32_t e = 0; e < 4; ++e)
        if (e >= first && e < last) {
          const bool keep = keep_of(d[e], prm);
          o[e] = keep ? __fmul_rn(xv[e], prm.scale) : 0.0f;
          if (mask) mask[li0 + e] = keep ? 1 : 0;
        }
    } else {
      const uint16_t* xi = static_cast<const uint16_t*>(xin) + li0;
      uint16_t* o = static_cast<uint16_t*>(out) + li0;
      uint16_t xv[4] = {0, 0, 0, 0};
#pragma unroll
      for (uint32_t e = 0; e < 4; ++e)
        if (e >= first && e < last) xv[e] = xi[e];
#pragma unroll
      for (uint32_t e = 0; e < 4; ++e)
        if (e >= first && e < last) {
          const bool keep = keep_of(d[e], prm);
          const float prod = __fmul_rn(__uint_as_float(static_cast<uint32_t>(xv[e]) << 16), prm.scale);
          o[e] = static_cast<uint16_t>(pack_bf16(keep ? prod : 0.0f, 0.0f));
          if (mask) mask[li0 + e] = keep ? 1 : 0;
        }
    }
  }
}

// ---- dispatch --------------------------------------------------------------------
template <int OP, int DT, typename IT, int NOUT>
hipError_t launch_nout(bool aligned, const PlanT<IT>& plan, const OpParams& prm, const void* x, void* out,
                       uint8_t* mask, hipStream_t stream) {
  const uint64_t blocks = (plan.total_units + kThreads - 1) / kThreads;
  if (blocks == 0) return hipSuccess;
  if (blocks > 0x7FFFFFFFull) return hipErrorInvalidConfiguration;
  const dim3 grid(static_cast<uint32_t>(blocks)), block(kThreads);
  if (aligned)
    hipLaunchKernelGGL((aligned_kernel<OP, DT, IT, NOUT>), grid, block, 0, stream, plan, prm, x, out, mask);
  else
    hipLaunchKernelGGL((ragged_kernel<OP, DT, IT, NOUT>), grid, block, 0, stream, plan, prm, x, out, mask);
  return hipGetLastError();
}

template <int OP, int DT, typename IT>
hipError_t launch_typed(bool aligned, const Geometry& g, const RunShape& rs, uint64_t offset, uint64_t units_per_run,
                        const OpParams& prm, const void* x, void* out, uint8_t* mask, hipStream_t stream) {
  const PlanT<IT> plan = make_plan<IT>(g, rs, offset, units_per_run);
  switch (plan.n_outer) {
    case 0: return launch_nout<OP, DT, IT, 0>(aligned, plan, prm, x, out, mask, stream);
    case 1: return launch_nout<OP, DT, IT, 1>(aligned, plan, prm, x, out, mask, stream);
    default: return launch_nout<OP, DT, IT, 2>(aligned, plan, prm, x, out, mask, stream);
  }
}

template <int OP, int DT>
hipError_t launch_dt(const Geometry& g, uint64_t offset, const OpParams& prm, const void* x, void* out,
                     uint8_t* mask, hipStream_t stream) {
  const RunShape rs = run_shape(g);
  constexpr uint64_t V = UnitOf<OP, DT>::kElems;
  const uint64_t pos0 = offset + g.origin;
  const bool aligned = rs.phases_equal && (pos0 % 4 == 0) && (rs.run_len % V == 0);
  // Ragged: one unit per generator block a run can touch; with unequal phases the
  // count is the upper bound over phases 0..3.
  const uint64_t phase_max = rs.phases_equal ? (pos0 % 4) : 3;
  const uint64_t units = aligned ? rs.run_len / V : (phase_max + rs.run_len + 3) / 4;
  if (fits_32bit(rs, units))
    return launch_typed<OP, DT, uint32_t>(aligned, g, rs, offset, units, prm, x, out, mask, stream);
  return launch_typed<OP, DT, uint64_t>(aligned, g, rs, offset, units, prm, x, out, mask, stream);
}

}  // namespace

hipError_t launch_op(OpKind op, const Geometry& g, uint64_t offset, const OpParams& prm, const void* x, void* out,
                     uint8_t* mask, hipStream_t stream) {
  if (g.local_numel == 0) return hipSuccess;
  const bool bf16 = prm.dtype == kBF16;
  switch (op) {
    case kOpRaw:
      return launch_dt<kOpRaw, kF32>(g, offset, prm, x, out, mask, stream);
    case kOpRandint:
      return launch_dt<kOpRandint, kF32>(g, offset, prm, x, out, mask, stream);
    case kOpUniform:
      return bf16 ? launch_dt<kOpUniform, kBF16>(g, offset, prm, x, out, mask, stream)
                  : launch_dt<kOpUniform, kF32>(g, offset, prm, x, out, mask, stream);
    case kOpNormal:
      return bf16 ? launch_dt<kOpNormal, kBF16>(g, offset, prm, x, out, mask, stream)
                  : launch_dt<kOpNormal, kF32>(g, offset, prm, x, out, mask, stream);
    case kOpDropout:
      return bf16 ? launch_dt<kOpDropout, kBF16>(g, offset, prm, x, out, mask, stream)
                  : launch_dt<kOpDropout, kF32>(g, offset, prm, x, out, mask, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace vesrng
