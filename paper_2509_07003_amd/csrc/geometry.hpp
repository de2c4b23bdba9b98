// Host side of the sharded-RNG path: validates a sharding description and
// turns it into closed-form shard geometry (veScale Section 2.2: device mesh,
// placements, local tensor; Algorithm 1's metadata upsilon, omega, pi, rho).
#pragma once
#include <cstdint>
#include <vector>

#include "../../include/vesrng.h"
#include "plan.h"

namespace vesrng {

// One axis of the shard seen as a box in the flattened global tensor.
struct Axis {
  int64_t extent;
  int64_t stride;  // global stride in elements
};

struct Geometry {
  std::vector<int64_t> local_shape;  // per tensor dimension
  int64_t local_numel = 0;
  uint64_t global_numel = 0;         // product of the global shape
  uint64_t max_global_index = 0;     // largest global flat index of the whole tensor
  uint64_t origin = 0;               // global flat index of local element 0
  std::vector<Axis> axes;            // outermost first; local tensor is row-major over them,
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
  std::vector<Axis> outer;           // innermost outer axis first
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

}  // namespace vesrng
