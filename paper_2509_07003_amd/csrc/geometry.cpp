#include "geometry.hpp"

#include <algorithm>

namespace vesrng {

namespace {

constexpr uint64_t kMaxNumel = 1ull << 62;

// The global indices a rank holds along ONE tensor dimension, kept as a
// row-major box: index(t_0, .., t_{m-1}) = origin + sum t_k * step_k, local
// order = row-major over (t_0 .. t_{m-1}).  A fresh dimension is one axis of
// step 1; InterleavedShard adds an axis.
struct Sub {
  int64_t extent;
  int64_t step;
};
struct DimBox {
  SmallVec<Sub, kMaxSubs> subs;  // outermost first
  int64_t origin = 0;
  int64_t length() const {
    int64_t n = 1;
    for (const Sub& s : subs) n *= s.extent;
    return n;
  }
};

// Keeps entries [start, start + len) of the row-major list of subs[from..].
// Possible in closed form when the range is whole rows of the leading axis or
// lies inside one of its rows.
bool slice(DimBox& box, size_t from, int64_t start, int64_t len) {
  if (len == 0) {
    box.subs.assign(1, Sub{0, 1});
    return true;
  }
  if (from + 1 == box.subs.size()) {
    box.origin += start * box.subs[from].step;
    box.subs[from].extent = len;
    return true;
  }
  int64_t inner = 1;
  for (size_t k = from + 1; k < box.subs.size(); ++k) inner *= box.subs[k].extent;
  if (start % inner == 0 && len % inner == 0) {
    box.origin += (start / inner) * box.subs[from].step;
    box.subs[from].extent = len / inner;
    return true;
  }
  if (start / inner == (start + len - 1) / inner) {
    box.origin += (start / inner) * box.subs[from].step;
    box.subs[from].extent = 1;
    return slice(box, from + 1, start % inner, len);
  }
  return false;
}

// Start and length of chunk `which` when `n` entries are cut into `parts`
// consecutive chunks of ceil(n / parts).
void chunk_range(int64_t n, int64_t parts, int64_t which, int64_t* start, int64_t* len) {
  const int64_t q = (n + parts - 1) / parts;
  const int64_t b = std::min(n, q * which);
  const int64_t e = std::min(n, q * (which + 1));
  *start = b;
  *len = e - b;
}

vesrng_status apply_shard(DimBox& box, int64_t parts, int64_t which) {
  int64_t start, len;
  chunk_range(box.length(), parts, which, &start, &len);
  return slice(box, 0, start, len) ? VESRNG_OK : VESRNG_ERR_UNSUPPORTED;
}

vesrng_status apply_interleaved(DimBox& box, int64_t groups, int64_t parts, int64_t which) {
  const int64_t n = box.length();
  if (groups < 1 || n % groups != 0) return VESRNG_ERR_BAD_PLACEMENT;
  if (n == 0) return VESRNG_OK;
  // Make the leading axes enumerate exactly `groups` groups.
  int64_t remaining = groups;
  size_t k = 0;
  while (remaining > 1) {
    if (k >= box.subs.size()) return VESRNG_ERR_UNSUPPORTED;
    const int64_t e = box.subs[k].extent;
    if (e % remaining == 0) {
      const int64_t per = e / remaining;
      const int64_t step = box.subs[k].step;
      box.subs[k] = Sub{remaining, step * per};
      if (box.subs.full()) return VESRNG_ERR_UNSUPPORTED;
      box.subs.insert_at(k + 1, Sub{per, step});
      remaining = 1;
      ++k;
    } else if (remaining % e == 0) {
      remaining /= e;
      ++k;
    } else {
      return VESRNG_ERR_UNSUPPORTED;
    }
  }
  if (k == box.subs.size()) {
    if (box.subs.full()) return VESRNG_ERR_UNSUPPORTED;
    box.subs.push_back(Sub{1, 1});  // groups of one entry
  }
  int64_t start, len;
  chunk_range(n / groups, parts, which, &start, &len);
  if (len == 0) {
    box.subs.assign(1, Sub{0, 1});
    return VESRNG_OK;
  }
  return slice(box, k, start, len) ? VESRNG_OK : VESRNG_ERR_UNSUPPORTED;
}

}  // namespace

vesrng_status build_geometry(const vesrng_sharding* s, Geometry* g) {
  if (!s || !g) return VESRNG_ERR_NULL;
  if (s->ndim < 0 || s->ndim > kMaxDims) return VESRNG_ERR_BAD_SHAPE;
  if (s->mesh_ndim < 0 || s->mesh_ndim > kMaxDims) return VESRNG_ERR_BAD_MESH;
  if (s->ndim > 0 && !s->global_shape) return VESRNG_ERR_NULL;
  if (s->mesh_ndim > 0 && (!s->mesh_shape || !s->placements || !s->mesh_coord)) return VESRNG_ERR_NULL;

  const int nd = s->ndim;
  uint64_t numel = 1;
  bool empty = false;
  for (int d = 0; d < nd; ++d) {
    const int64_t e = s->global_shape[d];
    if (e < 0) return VESRNG_ERR_BAD_SHAPE;
    if (e == 0) empty = true;
  }
  if (!empty)
    for (int d = 0; d < nd; ++d) {
      const uint64_t e = static_cast<uint64_t>(s->global_shape[d]);
      if (numel > kMaxNumel / e) return VESRNG_ERR_BAD_SHAPE;
      numel *= e;
    }
  else
    numel = 0;

  // Global strides (Algorithm 1's pi) and the largest flat index they reach.
  SmallVec<int64_t, kMaxDims> pi;
  pi.assign(static_cast<size_t>(nd), 1);
  if (s->global_stride) {
    for (int d = 0; d < nd; ++d) {
      if (s->global_stride[d] <= 0) return VESRNG_ERR_OVERFLOW;
      pi[static_cast<size_t>(d)] = s->global_stride[d];
    }
  } else {
    for (int d = nd - 1; d > 0; --d)
      pi[static_cast<size_t>(d) - 1] =
          pi[static_cast<size_t>(d)] * std::max<int64_t>(1, s->global_shape[d]);
  }
  uint64_t max_index = 0;
  if (!empty)
    for (int d = 0; d < nd; ++d) {
      const uint64_t span = static_cast<uint64_t>(s->global_shape[d] - 1);
      const uint64_t st = static_cast<uint64_t>(pi[static_cast<size_t>(d)]);
      if (span != 0 && st > (kMaxNumel - max_index) / span) return VESRNG_ERR_OVERFLOW;
      max_index += span * st;
    }

  for (int m = 0; m < s->mesh_ndim; ++m) {
    if (s->mesh_shape[m] < 1) return VESRNG_ERR_BAD_MESH;
  }
  for (int m = 0; m < s->mesh_ndim; ++m) {
    if (s->mesh_coord[m] < 0 || s->mesh_coord[m] >= s->mesh_shape[m]) return VESRNG_ERR_BAD_COORD;
  }
  for (int m = 0; m < s->mesh_ndim; ++m) {
    const vesrng_placement& pl = s->placements[m];
    if (pl.kind == VESRNG_REPLICATE) continue;
    if (pl.kind != VESRNG_SHARD && pl.kind != VESRNG_INTERLEAVED_SHARD) return VESRNG_ERR_BAD_PLACEMENT;
    if (pl.dim < 0 || pl.dim >= nd) return VESRNG_ERR_BAD_PLACEMENT;
    if (pl.kind == VESRNG_INTERLEAVED_SHARD && pl.interleave < 1) return VESRNG_ERR_BAD_PLACEMENT;
  }

  // Two descriptions are built side by side: the chain of placements per dimension (always
  // possible) and the box form the fast kernels need (dropped as soon as a cut has no box).
  SmallVec<DimBox, kMaxDims> boxes;
  boxes.assign(static_cast<size_t>(nd), DimBox{});
  SmallVec<int64_t, kMaxDims> length;
  length.assign(static_cast<size_t>(nd), 0);
  for (int d = 0; d < nd; ++d) {
    boxes[static_cast<size_t>(d)].subs.assign(1, Sub{s->global_shape[d], 1});
    length[static_cast<size_t>(d)] = s->global_shape[d];
  }
  // One virtual thread is the flat stream itself (tau = 0, beta = offset + j): the fast kernels serve it.
  g->virtual_threads = s->virtual_threads == 1 ? 0 : s->virtual_threads;
  g->boxed = true;
  g->chain = ChainPlan{};
  g->chain.ndim = nd;
  for (int m = 0; m < s->mesh_ndim; ++m) {
    const vesrng_placement& pl = s->placements[m];
    if (pl.kind == VESRNG_REPLICATE) continue;
    const size_t d = static_cast<size_t>(pl.dim);
    const int64_t parts = s->mesh_shape[m], which = s->mesh_coord[m];
    int64_t& n = length[d];
    ChainStep step{};
    if (pl.kind == VESRNG_SHARD) {
      chunk_range(n, parts, which, &step.start, &step.len);
      n = step.len;
    } else {
      if (n % pl.interleave != 0) return VESRNG_ERR_BAD_PLACEMENT;
      step.interleaved = 1;
      step.per = n / pl.interleave;
      chunk_range(step.per, parts, which, &step.start, &step.len);
      n = step.len * pl.interleave;
    }
    if (g->chain.nsteps[d] >= kMaxSteps) return VESRNG_ERR_UNSUPPORTED;
    g->chain.steps[d][g->chain.nsteps[d]++] = step;
    if (g->boxed) {
      const vesrng_status st = pl.kind == VESRNG_SHARD ? apply_shard(boxes[d], parts, which)
                                                       : apply_interleaved(boxes[d], pl.interleave, parts, which);
      if (st == VESRNG_ERR_UNSUPPORTED) g->boxed = false;
      else if (st != VESRNG_OK) return st;
    }
  }

  g->local_shape.assign(static_cast<size_t>(nd), 0);
  g->local_numel = 1;
  for (int d = 0; d < nd; ++d) {
    g->local_shape[static_cast<size_t>(d)] = length[static_cast<size_t>(d)];
    g->local_numel *= length[static_cast<size_t>(d)];
    g->chain.local_shape[d] = length[static_cast<size_t>(d)];
    g->chain.stride[d] = pi[static_cast<size_t>(d)];
  }
  g->chain.fits32 = (static_cast<uint64_t>(g->local_numel) >> 32) == 0 ? 1 : 0;
  for (int d = 0; d < nd; ++d)
    if ((static_cast<uint64_t>(s->global_shape[d]) >> 32) != 0) g->chain.fits32 = 0;
  g->global_numel = numel;
  g->max_global_index = max_index;
  g->origin = 0;
  g->axes.clear();
  if (g->local_numel == 0 || !g->boxed) return VESRNG_OK;

  SmallVec<Axis, kMaxAxes> raw;
  for (int d = 0; d < nd; ++d) {
    const DimBox& box = boxes[static_cast<size_t>(d)];
    const int64_t st = pi[static_cast<size_t>(d)];
    g->origin += static_cast<uint64_t>(box.origin) * static_cast<uint64_t>(st);
    for (const Sub& sub : box.subs)
      if (sub.extent != 1) raw.push_back(Axis{sub.extent, sub.step * st});
  }
  // Merge neighbours that form one longer arithmetic progression.
  for (const Axis& a : raw) {
    if (!g->axes.empty() && g->axes.back().stride == a.extent * a.stride)
      g->axes.back() = Axis{g->axes.back().extent * a.extent, a.stride};
    else
      g->axes.push_back(a);
  }
  if (g->axes.size() > static_cast<size_t>(kMaxOuter)) g->boxed = false;  // the chain still describes it
  return VESRNG_OK;
}

RunShape run_shape(const Geometry& g) {
  RunShape rs;
  size_t n_outer = g.axes.size();
  if (!g.axes.empty() && g.axes.back().stride == 1) {
    rs.run_len = static_cast<uint64_t>(g.axes.back().extent);
    --n_outer;
  }
  for (size_t k = n_outer; k-- > 0;) {
    rs.outer.push_back(g.axes[k]);
    rs.n_runs *= static_cast<uint64_t>(g.axes[k].extent);
    if (g.axes[k].stride % 4 != 0) rs.phases_equal = false;
  }
  return rs;
}

bool fits_32bit(const RunShape& rs, uint64_t units_per_run) {
  // 2^30 rather than 2^31: the kernels also form small signed differences of these values.
  const uint64_t lim = 1ull << 30;
  if (rs.run_len >= lim || units_per_run >= lim) return false;
  if (rs.n_runs >= lim || rs.n_runs * units_per_run >= lim) return false;
  // Local flat indices are formed as run * run_len + k in the index type.
  if (rs.n_runs * rs.run_len >= lim) return false;
  for (const Axis& a : rs.outer)
    if (static_cast<uint64_t>(a.extent) >= lim) return false;
  return true;
}

// A tile of T elements cut by B run boundaries touches at most T/4 + 1.5 (B + 1) blocks, plus one
// dead slot per boundary when runs differ in phase; they must fit `passes` rounds of the workgroup.
uint64_t pick_tile_units(uint64_t run_len, uint64_t unit_elems, uint64_t per_thread, bool phases_equal) {
  const uint64_t passes = unit_elems / 4 * per_thread;
  for (uint64_t q = kThreadsPerGroup * per_thread; q >= 32; q -= 8) {
    const uint64_t t = q * unit_elems;
    const uint64_t b = (t + run_len - 1) / run_len;
    const uint64_t blocks = t / 4 + (3 * (b + 1) + 1) / 2 + (phases_equal ? 0 : b) + 1;
    if (blocks <= passes * kThreadsPerGroup) return q;
  }
  return 0;
}

LaunchChoice choose_launch(const Geometry& g, const RunShape& rs, uint64_t offset, const LaunchTraits& traits) {
  const uint64_t V = traits.unit_elems;
  const uint64_t pos0 = offset + g.origin;
  LaunchChoice c;
  // Aligned: every run starts on a block boundary and is whole units long - or the shard is a
  // single run, whose last unit the aligned kernel finishes element by element (not randint,
  // whose lanes trade halves of whole blocks).
  if (rs.phases_equal && (pos0 % 4 == 0) &&
      (rs.run_len % V == 0 || (rs.n_runs == 1 && !traits.whole_blocks_only))) {
    c.flavour = kAligned;
  } else if (rs.run_len >= 16 && rs.run_len >= traits.tile_min_run_len &&
             static_cast<uint64_t>(g.local_numel) >= traits.tile_min_elems &&
             (traits.tile_max_elems == 0 || static_cast<uint64_t>(g.local_numel) < traits.tile_max_elems)) {
    if (traits.big_tileable && static_cast<uint64_t>(g.local_numel) >= traits.big_tile_min_elems) {
      c.tile_units = pick_tile_units(rs.run_len, V, kBigTileUnits, rs.phases_equal);
      if (c.tile_units != 0) c.flavour = kTiledBig;
    }
    if (c.flavour == kRagged && traits.tileable) {
      c.tile_units = pick_tile_units(rs.run_len, V, 1, rs.phases_equal);
      if (c.tile_units != 0) c.flavour = kTiled;
    }
  }
  // Aligned: units of V elements.  Otherwise: one unit per generator block a run can touch;
  // with unequal phases the count is the upper bound over phases 0..3.
  const uint64_t phase_max = rs.phases_equal ? (pos0 % 4) : 3;
  c.units_per_run = c.flavour == kAligned ? (rs.run_len + V - 1) / V : (phase_max + rs.run_len + 3) / 4;
  c.wide = !fits_32bit(rs, c.units_per_run);
  return c;
}

RunShape piece_shape(const RunShape& rs, uint64_t rows) {
  RunShape piece = rs;
  const uint64_t extent = static_cast<uint64_t>(rs.outer.back().extent);
  piece.outer.back().extent = static_cast<int64_t>(rows);
  piece.n_runs = rs.n_runs / extent * rows;
  return piece;
}

bool plan_pieces(const RunShape& rs, uint64_t units_per_run, Pieces* p) {
  if (rs.outer.empty()) return false;
  const Axis top = rs.outer.back();
  p->extent = static_cast<uint64_t>(top.extent);
  p->stride = static_cast<uint64_t>(top.stride);
  p->per_index = rs.n_runs / p->extent * rs.run_len;
  // Bounded by elements first (fits_32bit's limit), then checked in full: units per run exceed elements per run
  // only for runs shorter than a unit, which the second test catches.
  uint64_t rows = ((1ull << 30) - 1) / p->per_index;
  rows -= rows % 32;
  while (rows >= 32 && !fits_32bit(piece_shape(rs, rows), units_per_run)) rows -= 32;
  if (rows < 32) return false;
  p->rows_per_piece = rows;
  return true;
}

bool plan_theta(const Geometry& g, const RunShape& rs, uint64_t offset, uint64_t unit_elems, ThetaPlan* tp) {
  const uint64_t theta = g.virtual_threads, n = static_cast<uint64_t>(g.local_numel), V = unit_elems;
  if (theta == 0 || !g.boxed || n == 0) return false;
  if (rs.n_runs != 1 || rs.run_len != n) return false;          // one run only
  if (theta % V != 0 || g.origin % V != 0) return false;        // units must not straddle threads or steps
  // Step groups at the shard's two ends are only partly inside it; their threads still run.
  // Below 16 step groups' worth of elements that waste exceeds a third: leave it to the element-wise kernel.
  if (theta > (1ull << 40) || n / 64 < theta) return false;
  const uint64_t first_step = g.origin / theta, last_step = (g.origin + n - 1) / theta;
  tp->theta = theta;
  tp->cols = theta / V;
  tp->group0 = first_step / 4;
  const uint64_t groups = last_step / 4 - tp->group0 + 1;
  tp->total_threads = groups * tp->cols;
  // Thread numbers are split into (group, column) with one 32-bit multiply-shift division; shards beyond that
  // (2^35 fp32 elements and more) are left to the element-wise kernel.
  if (tp->total_threads >= (1ull << 31) || tp->cols >= (1ull << 31)) return false;
  tp->cols_div = make_div32(static_cast<uint32_t>(tp->cols));
  tp->origin = g.origin;
  tp->local_numel = n;
  tp->block0 = offset / 4;
  return true;
}

template <typename IT>
PlanT<IT> make_plan(const Geometry& g, const RunShape& rs, uint64_t offset, uint64_t units_per_run) {
  PlanT<IT> p{};
  p.pos0 = offset + g.origin;
  p.total_units = units_per_run * rs.n_runs;
  p.run_len = static_cast<IT>(rs.run_len);
  p.units_per_run = static_cast<IT>(units_per_run);
  p.units_div = DivOf<IT>::make(units_per_run);
  p.n_outer = static_cast<int32_t>(rs.outer.size());
  p.wave_runs = (units_per_run % 64 == 0) ? 1 : 0;
  for (size_t k = 0; k < rs.outer.size(); ++k) {
    p.outer_extent[k] = static_cast<IT>(rs.outer[k].extent);
    p.outer_div[k] = DivOf<IT>::make(static_cast<uint64_t>(rs.outer[k].extent));
    p.outer_stride[k] = static_cast<uint64_t>(rs.outer[k].stride);
  }
  for (size_t k = rs.outer.size(); k < static_cast<size_t>(kMaxOuter); ++k) {
    p.outer_extent[k] = 1;
    p.outer_div[k] = DivOf<IT>::make(1);
    p.outer_stride[k] = 0;
  }
  return p;
}

template PlanT<uint32_t> make_plan<uint32_t>(const Geometry&, const RunShape&, uint64_t, uint64_t);
template PlanT<uint64_t> make_plan<uint64_t>(const Geometry&, const RunShape&, uint64_t, uint64_t);

}  // namespace vesrng
