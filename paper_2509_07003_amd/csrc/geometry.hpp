// Host side of the sharded-RNG path: validates a sharding description and
// turns it into closed-form shard geometry (veScale Section 2.2: device mesh,
// placements, local tensor; Algorithm 1's metadata upsilon, omega, pi, rho).
#pragma once
#include <cstddef>
#include <cstdint>

#include "../../include/vesrng.h"
#include "plan.h"

namespace vesrng {

// A vector with inline storage: shard descriptions are tiny (at most 8 dimensions, a few axes
// each) and are rebuilt on every call, so nothing here touches the heap.
template <typename T, int N>
struct SmallVec {
  T item[N];
  int count = 0;
  size_t size() const { return static_cast<size_t>(count); }
  bool empty() const { return count == 0; }
  bool full() const { return count == N; }
  void clear() { count = 0; }
  T& operator[](size_t k) { return item[k]; }
  const T& operator[](size_t k) const { return item[k]; }
  T& back() { return item[count - 1]; }
  const T& back() const { return item[count - 1]; }
  const T* begin() const { return item; }
  const T* end() const { return item + count; }
  void push_back(const T& v) { item[count++] = v; }
  void assign(size_t n, const T& v) {
    count = static_cast<int>(n);
    for (int k = 0; k < count; ++k) item[k] = v;
  }
  void insert_at(size_t pos, const T& v) {
    for (size_t k = static_cast<size_t>(count); k > pos; --k) item[k] = item[k - 1];
    item[pos] = v;
    ++count;
  }
};
constexpr int kMaxSubs = 12;                    // axes of one tensor dimension
constexpr int kMaxAxes = kMaxDims * kMaxSubs;   // axes of a whole shard before merging

// One axis of the shard seen as a box in the flattened global tensor.
struct Axis {
  int64_t extent;
  int64_t stride;  // global stride in elements
};

struct Geometry {
  SmallVec<int64_t, kMaxDims> local_shape;  // per tensor dimension
  int64_t local_numel = 0;
  uint64_t global_numel = 0;         // product of the global shape
  uint64_t max_global_index = 0;     // largest global flat index of the whole tensor
  uint64_t origin = 0;               // global flat index of local element 0
  SmallVec<Axis, kMaxAxes> axes;     // outermost first; local tensor is row-major over them,
                                     // extent-1 axes dropped, mergeable neighbours merged
  uint64_t virtual_threads = 0;      // Algorithm 1's global thread count Theta; 0 = flat stream
  bool boxed = true;                 // false: the shard is not a box; only `chain` describes it
  ChainPlan chain{};                 // always filled: the placement-by-placement index map
};

// Returns VESRNG_OK and fills `g`, or the status that describes what is wrong.
vesrng_status build_geometry(const vesrng_sharding* s, Geometry* g);

// Shape of the work a kernel launch covers.
struct RunShape {
  uint64_t run_len = 1;              // innermost axis if its global stride is 1, else 1
  SmallVec<Axis, kMaxAxes> outer;    // innermost outer axis first
  uint64_t n_runs = 1;
  bool phases_equal = true;          // every run starts at the same position modulo 4
};
RunShape run_shape(const Geometry& g);

// Fills a kernel plan.  `units_per_run` is chosen by the caller (it depends on the
// kernel flavour); pos0 = offset + origin.
template <typename IT>
PlanT<IT> make_plan(const Geometry& g, const RunShape& rs, uint64_t offset, uint64_t units_per_run);

// True when every quantity of the plan fits the 32-bit index path.
bool fits_32bit(const RunShape& rs, uint64_t units_per_run);

// ---- which kernel a boxed shard takes ------------------------------------------
// kAligned: every run starts on a generator-block boundary and is whole units long (or the
// shard is a single run).  kTiled / kTiledBig: ragged shard staged through LDS, one or
// kBigTileUnits aligned units per thread.  kRagged: one global block per thread, stored
// in place.
enum Flavour { kAligned, kTiled, kTiledBig, kRagged };
constexpr int kThreadsPerGroup = 256;
constexpr int kBigTileUnits = 4;

// What the operator / dtype instantiation of the kernels can use.
struct LaunchTraits {
  uint64_t unit_elems = 4;          // elements per aligned unit (4, or 8 for the 16-bit floating-point operators)
  bool tileable = false;            // has a staging kernel
  bool big_tileable = false;        // ... and its large-tile form
  uint64_t big_tile_min_elems = 0;  // smallest shard that takes the large tile
  // Shards the staging kernels serve at all: local element counts in [tile_min_elems, tile_max_elems) (0 = no
  // upper limit) with runs of at least tile_min_run_len elements; the rest keeps the kernel without staging.
  uint64_t tile_min_elems = 0;
  uint64_t tile_max_elems = 0;
  uint64_t tile_min_run_len = 16;
  bool whole_blocks_only = false;   // the aligned kernel cannot finish a partial last unit (randint)
};
struct LaunchChoice {
  Flavour flavour = kRagged;
  uint64_t units_per_run = 0;  // aligned: units of unit_elems; otherwise generator blocks a run can touch
  uint64_t tile_units = 0;     // staging kernels: aligned units per tile
  bool wide = false;           // 64-bit index instantiation
};
LaunchChoice choose_launch(const Geometry& g, const RunShape& rs, uint64_t offset, const LaunchTraits& traits);

// ---- shards whose indices need 64 bits, cut into pieces that do not -----------------
// A shard of 2^30 elements and more takes the 64-bit index instantiation of the kernels, whose index arithmetic
// costs the instruction-bound operators up to a third of their rate.  When the shard has at least one axis of
// runs it can instead be served piece by piece: the outermost axis of runs is the slowest local dimension, so
// `rows` consecutive indices of it are a contiguous part of the local tensor and a shard of the same kind
// (same run length, strides, phases), `rows` times `per_index` elements long, whose first element sits `stride`
// stream positions per index further on.  rows_per_piece is a multiple of 32, so that every piece starts on a
// 128-byte line of every buffer whatever the element size.
struct Pieces {
  uint64_t rows_per_piece = 0;  // indices of the outermost run axis per piece (the last piece may be shorter)
  uint64_t per_index = 0;       // local elements per index of that axis
  uint64_t extent = 0;          // extent of that axis
  uint64_t stride = 0;          // its global stride, in elements
};
// Fills `p` and returns true when the shard can be cut so that every piece fits the 32-bit index path.
bool plan_pieces(const RunShape& rs, uint64_t units_per_run, Pieces* p);
// The run shape of `rows` indices of the outermost run axis.
RunShape piece_shape(const RunShape& rs, uint64_t rows);

// ---- the virtual-thread layout with one generator call per four outputs ------------
// Algorithm 1's (tau, beta) virtualisation puts element j at virtual thread tau = j mod Theta,
// step s = j / Theta; word s mod 4 of block (offset / 4 + s / 4, tau).  The four words of one
// block therefore belong to the elements j, j + Theta, j + 2 Theta, j + 3 Theta of one step group
// (4 g <= s < 4 g + 4).  When the shard is ONE run [origin, origin + n) of the flattened global
// tensor, Theta and origin are multiples of the unit and the run is many step groups long, a
// thread can own the unit-wide column c of a step group g: unit_elems generator blocks feed its
// four aligned units, one per step, and neighbouring threads write neighbouring units.
struct ThetaPlan {
  uint64_t theta = 0;          // Theta
  uint64_t cols = 0;           // Theta / unit_elems: threads per step group
  Div32 cols_div{};            // divides by cols (thread numbers and cols are below 2^31)
  uint64_t group0 = 0;         // first step group that holds an element of the shard
  uint64_t origin = 0;         // global flat index of local element 0
  uint64_t local_numel = 0;
  uint64_t block0 = 0;         // offset / 4: generator block of step group 0
  uint64_t total_threads = 0;  // (number of step groups) * cols
};
// Fills `tp` and returns true when the shard qualifies; otherwise the element-wise kernel serves it.
bool plan_theta(const Geometry& g, const RunShape& rs, uint64_t offset, uint64_t unit_elems, ThetaPlan* tp);

// Largest tile (in units, a multiple of 8 so that tiles start on 128-byte lines) whose
// generator blocks fit the workgroup's passes; 0 = runs too short for tiling.
uint64_t pick_tile_units(uint64_t run_len, uint64_t unit_elems, uint64_t per_thread, bool phases_equal);

}  // namespace vesrng
