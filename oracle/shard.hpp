// TEST INFRASTRUCTURE ONLY (see philox.hpp).
//
// Shard geometry by simulation.  The paper's Algorithm 1 (Section 5) takes the
// local shape, the global shape and stride and the shard's coordinate in the
// global tensor as metadata "got from DTensor"; Section 2.2 defines that
// metadata as a device mesh plus one placement per mesh dimension.  The oracle
// does not derive closed forms: it starts from the list of all indices of each
// tensor dimension and literally cuts it, mesh dimension by mesh dimension.
#pragma once
#include <cstdint>
#include <stdexcept>
#include <vector>

namespace oracle {

enum PlacementKind : int32_t { kReplicate = 0, kShard = 1, kInterleavedShard = 2 };

struct Placement {
  int32_t kind;
  int32_t dim;         // tensor dimension that is cut (Shard / InterleavedShard)
  int32_t interleave;  // number of groups (InterleavedShard only)
};

struct Sharding {
  std::vector<int64_t> global_shape;
  std::vector<int64_t> global_stride;  // empty = row-major contiguous
  std::vector<int32_t> mesh_shape;
  std::vector<Placement> placements;   // one per mesh dimension, dim 0 applied first
  std::vector<int32_t> mesh_coord;
  uint64_t virtual_threads = 0;        // Algorithm 1's global thread count; 0 = one flat stream
};

// For every tensor dimension, the global indices this rank holds, in local order.
std::vector<std::vector<int64_t>> index_lists(const Sharding& s);

// Row-major strides of a shape (in elements).
std::vector<int64_t> row_major_strides(const std::vector<int64_t>& shape);

// Visits every local element in local row-major order, handing out its local
// flat index i and its global flat index j (Algorithm 1's i -> j map).  Only the
// range [i_begin, i_end) is visited.
template <class F>
void for_each_local(const Sharding& s, int64_t i_begin, int64_t i_end, F&& visit) {
  const std::vector<std::vector<int64_t>> lists = index_lists(s);
  const std::vector<int64_t> stride =
      s.global_stride.empty() ? row_major_strides(s.global_shape) : s.global_stride;
  const size_t nd = lists.size();
  int64_t numel = 1;
  for (const auto& l : lists) numel *= static_cast<int64_t>(l.size());
  if (i_end > numel) i_end = numel;
  if (i_begin >= i_end) return;
  // Coordinates of i_begin, innermost dimension fastest.
  std::vector<int64_t> c(nd, 0);
  int64_t rest = i_begin;
  for (size_t d = nd; d-- > 0;) {
    const int64_t n = static_cast<int64_t>(lists[d].size());
    c[d] = rest % n;
    rest /= n;
  }
  for (int64_t i = i_begin; i < i_end; ++i) {
    uint64_t j = 0;
    for (size_t d = 0; d < nd; ++d)
      j += static_cast<uint64_t>(lists[d][c[d]]) * static_cast<uint64_t>(stride[d]);
    visit(i, j);
    for (size_t d = nd; d-- > 0;) {  // odometer step
      if (++c[d] < static_cast<int64_t>(lists[d].size())) break;
      c[d] = 0;
    }
  }
}

}  // namespace oracle
