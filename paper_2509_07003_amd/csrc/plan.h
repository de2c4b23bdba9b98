// Decode plan: what the host hands to a kernel so that it can evaluate the
// local-to-global index map of Algorithm 1 (veScale, Section 5) without reading
// any metadata from memory.
//
// The rank's shard is described as a row-major box of "runs": the innermost
// axis is a run of `run_len` elements that are consecutive both in the local
// tensor and in the flattened global tensor; the outer axes enumerate the runs,
// each with its own global stride.  Algorithm 1's per-element mixed-radix decode
// (i' mod upsilon_d, i' / upsilon_d, sum of c_d * pi_d) is performed once per
// run-unit instead of once per element, with divisions by launch constants
// turned into multiply-shift.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define VESRNG_HD __host__ __device__ inline __attribute__((always_inline))
#else
#define VESRNG_HD inline
#endif

namespace vesrng {

constexpr int kMaxOuter = 16;

// 32x32 -> high 32 bits.
VESRNG_HD uint32_t mul_hi_u32(uint32_t a, uint32_t b) {
  return static_cast<uint32_t>((static_cast<uint64_t>(a) * b) >> 32);
}

// Division of a dividend n < 2^31 by a fixed divisor 1 <= d <= 2^31 with one
// high multiply: q = (mulhi(n, m) + n) >> s, where s = ceil(log2 d) and
// m = floor(2^32 (2^s - d) / d) + 1 (round-up method of Granlund & Montgomery).
// n < 2^31 keeps the sum inside 32 bits.
struct Div32 {
  uint32_t d, m, s;
  VESRNG_HD uint32_t div(uint32_t n) const { return (mul_hi_u32(n, m) + n) >> s; }
};

inline Div32 make_div32(uint32_t d) {
  Div32 r;
  r.d = d;
  uint32_t s = 0;
  while ((1ull << s) < d) ++s;
  r.s = s;
  r.m = static_cast<uint32_t>(((1ull << 32) * ((1ull << s) - d)) / d + 1);
  return r;
}

// Same interface on 64-bit indices, for shards too large for the 32-bit path.  The compiler's own 64-bit division
// checks at run time whether both operands fit 32 bits and then divides in 32 bits, which they do for every shard
// below 2^32 units; a multiply-shift form for full 64-bit dividends (one 64 x 64 -> high 64 multiply, four shifts
// and adds) was measured 4-12 % slower on shards of 2^30 .. 2^31 elements and is not used.
struct Div64 {
  uint64_t d;
  VESRNG_HD uint64_t div(uint64_t n) const { return n / d; }
};

template <typename IT>
struct DivOf;
template <>
struct DivOf<uint32_t> {
  using type = Div32;
  static Div32 make(uint64_t d) { return make_div32(static_cast<uint32_t>(d)); }
};
template <>
struct DivOf<uint64_t> {
  using type = Div64;
  static Div64 make(uint64_t d) { return Div64{d}; }
};

template <typename IT>
struct PlanT {
  using Div = typename DivOf<IT>::type;
  uint64_t pos0;        // stream position of local element 0: offset + its global flat index
  uint64_t total_units; // units_per_run * number of runs
  IT run_len;           // elements per run
  IT units_per_run;     // work units one run is cut into
  Div units_div;        // divides by units_per_run
  int32_t n_outer;      // axes that enumerate runs; axis 0 varies fastest
  int32_t wave_runs;    // units_per_run is a multiple of 64: the 64 units of a wavefront lie in ONE run, so the
                        // run's number, position and strides can be worked out once per wave in scalar registers
  IT outer_extent[kMaxOuter];
  Div outer_div[kMaxOuter];
  uint64_t outer_stride[kMaxOuter]; // global stride of the axis, in elements
};

// Global offset (in elements, relative to local element 0) of run number `o`.
template <typename IT>
VESRNG_HD uint64_t run_offset(const PlanT<IT>& p, IT o) {
  uint64_t off = 0;
#if defined(__HIPCC__)
#pragma unroll 1
#endif
  for (int k = 0; k + 1 < p.n_outer; ++k) {
    const IT q = p.outer_div[k].div(o);
    const IT c = o - q * p.outer_extent[k];
    off += static_cast<uint64_t>(c) * p.outer_stride[k];
    o = q;
  }
  if (p.n_outer > 0) off += static_cast<uint64_t>(o) * p.outer_stride[p.n_outer - 1];
  return off;
}

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

// Stream position of the first element of run `run`.  NOUT is the number of run-enumerating axes known at
// compile time (0 to 3) or 4 for "any number": the common shards (a contiguous slice; one strided axis of
// runs; two or three, as double sharding of a tensor of three to five dimensions gives - Table 5's grid) need
// no loop and no argument loads that depend on a loop counter, so their constants arrive with the rest of the
// kernel's arguments.
constexpr int kAnyAxes = 4;
template <int NOUT, typename IT>
VESRNG_HD uint64_t run_position(const PlanT<IT>& plan, IT run) {
  if constexpr (NOUT == 0) {
    return plan.pos0;
  } else if constexpr (NOUT == 1) {
    return plan.pos0 + static_cast<uint64_t>(run) * plan.outer_stride[0];
  } else if constexpr (NOUT == 2) {
    const IT c1 = plan.outer_div[0].div(run);
    const IT c0 = run - c1 * plan.outer_extent[0];
    return plan.pos0 + static_cast<uint64_t>(c0) * plan.outer_stride[0] + static_cast<uint64_t>(c1) * plan.outer_stride[1];
  } else if constexpr (NOUT == 3) {
    const IT q0 = plan.outer_div[0].div(run);
    const IT c0 = run - q0 * plan.outer_extent[0];
    const IT c2 = plan.outer_div[1].div(q0);
    const IT c1 = q0 - c2 * plan.outer_extent[1];
    return plan.pos0 + static_cast<uint64_t>(c0) * plan.outer_stride[0] + static_cast<uint64_t>(c1) * plan.outer_stride[1] +
           static_cast<uint64_t>(c2) * plan.outer_stride[2];
  } else {
    return plan.pos0 + run_offset(plan, run);
  }
}

// Work unit w -> (run, unit inside the run, stream position of the run).
template <int NOUT, typename IT>
VESRNG_HD void locate(const PlanT<IT>& plan, IT w, IT& run, IT& unit, uint64_t& run_pos) {
  if constexpr (NOUT == 0) {
    run = 0;
    unit = w;
  } else {
    run = plan.units_div.div(w);
    unit = w - run * plan.units_per_run;
  }
  run_pos = run_position<NOUT>(plan, run);
}

// ---- tile map of the staging kernel ---------------------------------------------
// A workgroup of the staging kernel owns a tile of the LOCAL tensor (elements [i0, i0 + lim))
// and first computes the GLOBAL generator blocks that intersect it.  plan.units_per_run counts
// the blocks a run can touch; a block is named by its flattened number run * units_per_run + bi.
template <typename IT>
struct TileArgs {
  typename PlanT<IT>::Div run_len_div;  // divides by the run length
  IT tile_units;                        // aligned units of the local tensor per tile
  uint64_t local_numel;
  // The short form of the tile map (tile_spot_same_phase below) and its two constants.
  uint32_t same_phase;  // 1: the short form applies
  uint32_t dblock;      // stride / 4 - units_per_run
  uint32_t drel;        // run_len - 4 * units_per_run modulo 2^32 (zero or a small negative number)
};

// Fills the tile arguments for a plan whose units_per_run counts generator blocks per run.  The short form
// of the map needs: 32-bit indices, ONE axis of runs, a stride between runs that is a multiple of four
// (so every run starts at the same position modulo 4 and units_per_run is exact for every run) and at
// least units_per_run blocks long, with a difference that fits 32 bits.
template <typename IT>
inline TileArgs<IT> make_tile_args(const PlanT<IT>& plan, uint64_t tile_units, uint64_t local_numel) {
  TileArgs<IT> ta{};
  ta.run_len_div = DivOf<IT>::make(plan.run_len);
  ta.tile_units = static_cast<IT>(tile_units);
  ta.local_numel = local_numel;
  if (sizeof(IT) == 4 && plan.n_outer == 1 && plan.outer_stride[0] % 4 == 0) {
    const uint64_t s4 = plan.outer_stride[0] >> 2, upr = static_cast<uint64_t>(plan.units_per_run);
    if (s4 >= upr && s4 - upr <= 0xFFFFFFFFull) {
      ta.same_phase = 1;
      ta.dblock = static_cast<uint32_t>(s4 - upr);
      ta.drel = static_cast<uint32_t>(plan.run_len) - 4u * static_cast<uint32_t>(upr);
    }
  }
  return ta;
}
// A run of at least 64 blocks lets stage A work out the tile map once per wavefront (tile_wave).
constexpr uint64_t kTileWaveMinBlocks = 64;

// Flattened number of the generator block that holds local element i.
template <int NOUT, typename IT>
VESRNG_HD IT tile_block_of(const PlanT<IT>& plan, const TileArgs<IT>& ta, uint64_t i) {
  const IT ii = static_cast<IT>(i);
  const IT run = ta.run_len_div.div(ii);
  const IT c = ii - run * plan.run_len;
  const uint32_t phase = static_cast<uint32_t>(run_position<NOUT>(plan, run)) & 3u;
  return run * plan.units_per_run + ((c + phase) >> 2);
}

// Where generator block w lands in the tile, in tile coordinates (local index minus i0): word e of
// the block sits at rel + e, and is written when lo <= rel + e < hi, the part of the block's run
// that lies inside the tile.  The run itself may start far before the tile and end far after it
// (a run of 2^32 elements and more is possible), so its bounds are clamped to the tile in the index
// type BEFORE they are narrowed; rel lies within a block of the tile by construction.
struct TileSpot {
  uint64_t block;   // generator block number in the stream
  int32_t rel, lo, hi;
};
template <int NOUT, typename IT>
VESRNG_HD TileSpot tile_spot(const PlanT<IT>& plan, uint64_t i0, int32_t lim, IT w) {
  using ST = typename SignedOf<IT>::type;
  IT run, bi;
  uint64_t run_pos;
  locate<NOUT>(plan, w, run, bi, run_pos);
  const ST run_lo = static_cast<ST>(run * plan.run_len) - static_cast<ST>(i0);
  const ST run_hi = run_lo + static_cast<ST>(plan.run_len);
  const ST zero = 0, top = static_cast<ST>(lim);
  TileSpot s;
  s.block = (run_pos >> 2) + bi;
  s.rel = static_cast<int32_t>(run_lo + static_cast<ST>(4 * bi) - static_cast<ST>(static_cast<uint32_t>(run_pos) & 3u));
  s.lo = static_cast<int32_t>(run_lo > zero ? (run_lo < top ? run_lo : top) : zero);
  s.hi = static_cast<int32_t>(run_hi < top ? (run_hi > zero ? run_hi : zero) : top);
  return s;
}

// The short form of the same map, for the shards make_tile_args marks (a column shard of a matrix whose
// row length is a multiple of four is the common one).  With one phase for all runs, run r starts at
// stream position pos0 + r * stride = 4 * (pos0 / 4 + r * stride / 4) + phase, so block w = r * upr + bi is
//   block = pos0 / 4 + r * (stride / 4 - upr) + w,      rel = 4 w + r * (run_len - 4 upr) - (i0 + phase),
// one division and two multiply-adds per block in 32-bit registers (rel modulo 2^32: its value lies within a
// block of the tile).  upr is exact for every run, so each block number of a tile belongs to a run that
// intersects the tile: run_lo < lim and run_hi > 0, and one-sided clamps give the same lo and hi.
VESRNG_HD TileSpot tile_spot_same_phase(const PlanT<uint32_t>& plan, const TileArgs<uint32_t>& ta, uint64_t i0,
                                        int32_t lim, uint32_t w) {
  const uint32_t run = plan.units_div.div(w);
  const uint32_t i032 = static_cast<uint32_t>(i0);
  const int32_t run_lo = static_cast<int32_t>(run * plan.run_len - i032);
  const int32_t run_hi = run_lo + static_cast<int32_t>(plan.run_len);
  TileSpot s;
  s.block = (plan.pos0 >> 2) + static_cast<uint64_t>(run) * ta.dblock + w;
  s.rel = static_cast<int32_t>(4u * w + run * ta.drel - (i032 + (static_cast<uint32_t>(plan.pos0) & 3u)));
  s.lo = run_lo > 0 ? run_lo : 0;
  s.hi = run_hi < lim ? run_hi : lim;
  return s;
}

// The same map worked out once per WAVEFRONT.  In stage A the 64 lanes of a wave take 64 consecutive
// flattened block numbers wf .. wf + 63.  When a run has at least 64 blocks these lie in at most two runs:
// `split` lanes in the run of block wf, the rest at the start of the next run.  Everything that depends on
// the run - its stream position, its bounds clamped to the tile, the division that finds it - is the same
// for all lanes of a part and is computed here from wave-uniform values (on the GPU: in scalar registers);
// a lane then only selects its part and adds its offset (tile_spot_of_lane).  rel_a / rel_b are the tile
// positions of the FIRST block of each part, which lie within a block of the tile, so they fit 32 bits
// whatever the run length.
struct TileWave {
  uint64_t block_a, block_b;  // generator block of lane 0 / of lane `split`
  uint32_t split;             // lanes below belong to part a (>= 64: the whole wave)
  int32_t rel_a, lo_a, hi_a, rel_b, lo_b, hi_b;
};
template <int NOUT, typename IT>
VESRNG_HD TileWave tile_wave(const PlanT<IT>& plan, uint64_t i0, int32_t lim, IT wf) {
  using ST = typename SignedOf<IT>::type;
  const ST zero = 0, top = static_cast<ST>(lim);
  IT run, bi;
  uint64_t pos_a;
  locate<NOUT>(plan, wf, run, bi, pos_a);
  const uint64_t pos_b = run_position<NOUT>(plan, static_cast<IT>(run + 1));
  const IT left = plan.units_per_run - bi;  // blocks of this run from bi on
  TileWave t;
  t.split = left < 64 ? static_cast<uint32_t>(left) : 64u;
  const ST lo_a = static_cast<ST>(run * plan.run_len) - static_cast<ST>(i0), hi_a = lo_a + static_cast<ST>(plan.run_len);
  const ST lo_b = hi_a, hi_b = hi_a + static_cast<ST>(plan.run_len);  // the local tensor is run after run
  t.block_a = (pos_a >> 2) + bi;
  t.block_b = pos_b >> 2;
  t.rel_a = static_cast<int32_t>(lo_a + static_cast<ST>(4 * bi) - static_cast<ST>(static_cast<uint32_t>(pos_a) & 3u));
  t.rel_b = static_cast<int32_t>(lo_b - static_cast<ST>(static_cast<uint32_t>(pos_b) & 3u));
  t.lo_a = static_cast<int32_t>(lo_a > zero ? (lo_a < top ? lo_a : top) : zero);
  t.hi_a = static_cast<int32_t>(hi_a < top ? (hi_a > zero ? hi_a : zero) : top);
  t.lo_b = static_cast<int32_t>(lo_b > zero ? (lo_b < top ? lo_b : top) : zero);
  t.hi_b = static_cast<int32_t>(hi_b < top ? (hi_b > zero ? hi_b : zero) : top);
  return t;
}
VESRNG_HD TileSpot tile_spot_of_lane(const TileWave& t, uint32_t lane) {
  const bool b = lane >= t.split;
  const uint32_t off = b ? lane - t.split : lane;
  TileSpot s;
  s.block = (b ? t.block_b : t.block_a) + off;
  s.rel = (b ? t.rel_b : t.rel_a) + static_cast<int32_t>(4u * off);
  s.lo = b ? t.lo_b : t.lo_a;
  s.hi = b ? t.hi_b : t.hi_a;
  return s;
}

// ---- chain plan: the general index map ---------------------------------------
// When a rank's indices along some tensor dimension do not form a box (an
// interleaved dimension that is cut again across group boundaries), the map
// from a local index to a global index along that dimension is evaluated by
// undoing the placements one by one, last applied first:
//   Shard:            c -> start + c
//   InterleavedShard: c = g * len + t  ->  g * per + start + t
// (start, len) is the rank's chunk of a list (Shard) or of every group
// (InterleavedShard); per is the group length before the cut.  This is Algorithm 1
// element by element: decode i over the local shape, map each coordinate, dot with
// the global stride.
constexpr int kMaxDims = 8;
constexpr int kMaxSteps = 8;

struct ChainStep {
  int64_t interleaved;  // 0: Shard, 1: InterleavedShard
  int64_t start, len, per;
};

struct ChainPlan {
  int32_t ndim;
  int32_t fits32;  // the local element count and every global extent are below 2^32
  int32_t nsteps[kMaxDims];
  int64_t local_shape[kMaxDims];
  int64_t stride[kMaxDims];  // global stride pi, in elements
  ChainStep steps[kMaxDims][kMaxSteps];
};

// Global flat index j of local flat index i.  T is the type the decode divides in: uint32_t
// when p.fits32 (every coordinate then fits 32 bits; a 32-bit division costs a fifth of a
// 64-bit one on the GPU), uint64_t otherwise.  The dot product with the stride is 64-bit.
template <typename T>
VESRNG_HD uint64_t chain_global_index_as(const ChainPlan& p, T i) {
  uint64_t j = 0;
  for (int d = p.ndim - 1; d >= 0; --d) {
    const T n = static_cast<T>(p.local_shape[d]);
    const T q = i / n;
    T c = i - q * n;
    i = q;
    for (int m = p.nsteps[d] - 1; m >= 0; --m) {
      const ChainStep& st = p.steps[d][m];
      if (st.interleaved) {
        const T len = static_cast<T>(st.len);
        const T g = c / len;
        c = g * static_cast<T>(st.per) + static_cast<T>(st.start) + (c - g * len);
      } else {
        c += static_cast<T>(st.start);
      }
    }
    j += static_cast<uint64_t>(c) * static_cast<uint64_t>(p.stride[d]);
  }
  return j;
}

// The same map with compile-time loop bounds (ndim <= ND, at most NS placements per dimension),
// so that a kernel fetches the whole plan in one batch instead of one dependent scalar load
// after another inside data-dependent loops.
template <int ND, int NS, typename T>
VESRNG_HD uint64_t chain_global_index_fixed(const ChainPlan& p, T i) {
  uint64_t j = 0;
#if defined(__HIPCC__)
#pragma unroll
#endif
  for (int d = ND - 1; d >= 0; --d) {
    if (d < p.ndim) {
      const T n = static_cast<T>(p.local_shape[d]);
      const T q = i / n;
      T c = i - q * n;
      i = q;
#if defined(__HIPCC__)
#pragma unroll
#endif
      for (int m = NS - 1; m >= 0; --m) {
        if (m < p.nsteps[d]) {
          const ChainStep& st = p.steps[d][m];
          if (st.interleaved) {
            const T len = static_cast<T>(st.len);
            const T g = c / len;
            c = g * static_cast<T>(st.per) + static_cast<T>(st.start) + (c - g * len);
          } else {
            c += static_cast<T>(st.start);
          }
        }
      }
      j += static_cast<uint64_t>(c) * static_cast<uint64_t>(p.stride[d]);
    }
  }
  return j;
}

VESRNG_HD uint64_t chain_global_index(const ChainPlan& p, uint64_t i) {
  return p.fits32 ? chain_global_index_as<uint32_t>(p, static_cast<uint32_t>(i))
                  : chain_global_index_as<uint64_t>(p, i);
}

}  // namespace vesrng
