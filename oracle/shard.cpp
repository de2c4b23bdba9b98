// TEST INFRASTRUCTURE ONLY (see philox.hpp).
#include "shard.hpp"

#include <string>

namespace oracle {

namespace {

// Cuts `list` into `parts` consecutive chunks of ceil(n / parts) entries (the
// last non-empty chunk may be shorter, the ones after it empty) and returns
// chunk number `which`.  This is the uneven-split rule of the DTensor model the
// paper builds on (Section 2.2).
std::vector<int64_t> chunk(const std::vector<int64_t>& list, int64_t parts, int64_t which) {
  const int64_t n = static_cast<int64_t>(list.size());
  const int64_t q = (n + parts - 1) / parts;
  std::vector<int64_t> out;
  for (int64_t t = 0; t < n; ++t)
    if (t / (q == 0 ? 1 : q) == which) out.push_back(list[t]);
  return out;
}

}  // namespace

std::vector<int64_t> row_major_strides(const std::vector<int64_t>& shape) {
  std::vector<int64_t> st(shape.size(), 1);
  for (size_t d = shape.size(); d-- > 1;) st[d - 1] = st[d] * shape[d];
  return st;
}

std::vector<std::vector<int64_t>> index_lists(const Sharding& s) {
  const size_t nd = s.global_shape.size();
  const size_t md = s.mesh_shape.size();
  if (s.placements.size() != md || s.mesh_coord.size() != md)
    throw std::invalid_argument("one placement and one coordinate per mesh dimension");
  std::vector<std::vector<int64_t>> lists(nd);
  for (size_t d = 0; d < nd; ++d) {
    if (s.global_shape[d] < 0) throw std::invalid_argument("negative extent");
    lists[d].resize(static_cast<size_t>(s.global_shape[d]));
    for (int64_t t = 0; t < s.global_shape[d]; ++t) lists[d][static_cast<size_t>(t)] = t;
  }
  for (size_t m = 0; m < md; ++m) {
    const int64_t parts = s.mesh_shape[m];
    const int64_t which = s.mesh_coord[m];
    if (parts < 1) throw std::invalid_argument("mesh extent < 1");
    if (which < 0 || which >= parts) throw std::invalid_argument("mesh coordinate out of range");
    const Placement& pl = s.placements[m];
    if (pl.kind == kReplicate) continue;
    if (pl.kind != kShard && pl.kind != kInterleavedShard)
      throw std::invalid_argument("placement has no per-element value (Partial or unknown)");
    if (pl.dim < 0 || static_cast<size_t>(pl.dim) >= nd)
      throw std::invalid_argument("sharded tensor dimension out of range");
    std::vector<int64_t>& list = lists[static_cast<size_t>(pl.dim)];
    if (pl.kind == kShard) {
      list = chunk(list, parts, which);
    } else {
      // InterleavedShard (Appendix A): the dimension is seen as `interleave`
      // consecutive groups; every group is cut like Shard and the rank keeps its
      // chunk of every group, in group order.
      const int64_t groups = pl.interleave;
      const int64_t n = static_cast<int64_t>(list.size());
      if (groups < 1 || n % groups != 0)
        throw std::invalid_argument("interleave must divide the dimension");
      const int64_t per = n / groups;
      std::vector<int64_t> kept;
      for (int64_t g = 0; g < groups; ++g) {
        std::vector<int64_t> group(list.begin() + g * per, list.begin() + (g + 1) * per);
        const std::vector<int64_t> mine = chunk(group, parts, which);
        kept.insert(kept.end(), mine.begin(), mine.end());
      }
      list = kept;
    }
  }
  return lists;
}

}  // namespace oracle
