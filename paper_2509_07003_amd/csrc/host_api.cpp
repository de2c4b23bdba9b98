// C ABI of the library, the entry points that never touch the GPU: shard geometry
// (Algorithm 1's upsilon and rho from the mesh and placements of Section 2.2), the offset
// every rank advances to after an operator (Section 5, design (f)), the i -> j map evaluated
// on the host by the kernels' own decode plan, and the status strings.  No HIP here: this
// file and geometry.cpp also build with a plain host compiler (the sanitizer build of the tests).
#include "../../include/vesrng.h"

#include <limits>

#include "geometry.hpp"

using namespace vesrng;

namespace {
template <typename IT>
uint64_t position_of_run(const vesrng::PlanT<IT>& plan, IT run) {
  switch (plan.n_outer) {
    case 0: return vesrng::run_position<0>(plan, run);
    case 1: return vesrng::run_position<1>(plan, run);
    case 2: return vesrng::run_position<2>(plan, run);
    case 3: return vesrng::run_position<3>(plan, run);
    default: return vesrng::run_position<vesrng::kAnyAxes>(plan, run);
  }
}
}  // namespace

extern "C" {

vesrng_status vesrng_local_shape(const vesrng_sharding* s, int64_t* local_shape, int64_t* local_numel) {
  if (!s || !local_numel) return VESRNG_ERR_NULL;
  Geometry g;
  const vesrng_status st = build_geometry(s, &g);
  if (st != VESRNG_OK) return st;
  if (local_shape)
    for (size_t d = 0; d < g.local_shape.size(); ++d) local_shape[d] = g.local_shape[d];
  *local_numel = g.local_numel;
  return VESRNG_OK;
}

vesrng_status vesrng_advance_offset(const vesrng_sharding* s, uint64_t offset, uint64_t* new_offset) {
  if (!s || !new_offset) return VESRNG_ERR_NULL;
  if (offset % 4 != 0) return VESRNG_ERR_OFFSET_ALIGN;
  // Only the global shape matters: use a one-rank view of the same tensor.
  vesrng_sharding whole = *s;
  whole.mesh_ndim = 0;
  whole.mesh_shape = nullptr;
  whole.placements = nullptr;
  whole.mesh_coord = nullptr;
  Geometry g;
  const vesrng_status st = build_geometry(&whole, &g);
  if (st != VESRNG_OK) return st;
  // Draws consumed: one per position up to the last global element; with theta virtual
  // threads each thread steps ceil(span / theta) times.
  uint64_t span = g.global_numel == 0 ? 0 : g.max_global_index + 1;
  if (s->virtual_threads != 0) span = (span + s->virtual_threads - 1) / s->virtual_threads;
  const uint64_t step = 4 * ((span + 3) / 4);
  if (offset > std::numeric_limits<uint64_t>::max() - step) return VESRNG_ERR_OVERFLOW;
  *new_offset = offset + step;
  return VESRNG_OK;
}

vesrng_status vesrng_global_index(const vesrng_sharding* s, int64_t n, const int64_t* local_index,
                                  uint64_t* global_index) {
  if (!s || (n > 0 && (!local_index || !global_index))) return VESRNG_ERR_NULL;
  Geometry g;
  const vesrng_status st = build_geometry(s, &g);
  if (st != VESRNG_OK) return st;
  if (!g.boxed) {
    for (int64_t k = 0; k < n; ++k) {
      if (local_index[k] < 0 || local_index[k] >= g.local_numel) return VESRNG_ERR_BAD_PARAM;
      global_index[k] = chain_global_index(g.chain, static_cast<uint64_t>(local_index[k]));
    }
    return VESRNG_OK;
  }
  const RunShape rs = run_shape(g);
  // Same plan types and decode routines as the kernels, compiled for the host, chosen as the kernels' launcher
  // chooses them (the forms written out for one and two axes of runs, the loop for more).
  const bool narrow = fits_32bit(rs, rs.run_len);
  const PlanT<uint32_t> p32 = narrow ? make_plan<uint32_t>(g, rs, 0, rs.run_len) : PlanT<uint32_t>{};
  const PlanT<uint64_t> p64 = make_plan<uint64_t>(g, rs, 0, rs.run_len);
  for (int64_t k = 0; k < n; ++k) {
    const int64_t i = local_index[k];
    if (i < 0 || i >= g.local_numel) return VESRNG_ERR_BAD_PARAM;
    if (narrow) {
      const uint32_t w = static_cast<uint32_t>(i);
      const uint32_t run = p32.units_div.div(w);
      global_index[k] = position_of_run(p32, run) + (w - run * p32.units_per_run);
    } else {
      const uint64_t w = static_cast<uint64_t>(i);
      const uint64_t run = p64.units_div.div(w);
      global_index[k] = position_of_run(p64, run) + (w - run * p64.units_per_run);
    }
  }
  return VESRNG_OK;
}

vesrng_status vesrng_global_index_general(const vesrng_sharding* s, int64_t n, const int64_t* local_index,
                                          uint64_t* global_index) {
  if (!s || (n > 0 && (!local_index || !global_index))) return VESRNG_ERR_NULL;
  Geometry g;
  const vesrng_status st = build_geometry(s, &g);
  if (st != VESRNG_OK) return st;
  for (int64_t k = 0; k < n; ++k) {
    if (local_index[k] < 0 || local_index[k] >= g.local_numel) return VESRNG_ERR_BAD_PARAM;
    global_index[k] = chain_global_index(g.chain, static_cast<uint64_t>(local_index[k]));
  }
  return VESRNG_OK;
}

const char* vesrng_status_string(vesrng_status st) {
  switch (st) {
    case VESRNG_OK: return "ok";
    case VESRNG_ERR_NULL: return "a required pointer is NULL";
    case VESRNG_ERR_BAD_SHAPE: return "bad global shape";
    case VESRNG_ERR_BAD_MESH: return "bad mesh shape";
    case VESRNG_ERR_BAD_COORD: return "mesh coordinate out of range";
    case VESRNG_ERR_BAD_PLACEMENT: return "bad placement";
    case VESRNG_ERR_OFFSET_ALIGN: return "offset must be a multiple of 4";
    case VESRNG_ERR_BAD_PARAM: return "bad operator parameter";
    case VESRNG_ERR_DTYPE: return "unsupported dtype";
    case VESRNG_ERR_UNSUPPORTED: return "sharding beyond the supported number of placements per dimension";
    case VESRNG_ERR_OVERFLOW: return "stream position or stride overflow";
    case VESRNG_ERR_HIP: return "HIP launch failed";
    case VESRNG_ERR_ALIGN: return "device pointer not 16-byte aligned";
  }
  return "unknown status";
}

}  // extern "C"
