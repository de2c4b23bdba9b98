// Test driver for the HOST code of the library (no GPU, no HIP): built by the tests with
// g++ -fsanitize=address,undefined from csrc/geometry.cpp and csrc/host_api.cpp, so that the
// fixed-capacity index surgery of the shard geometry and the kernels' decode plan run under the
// sanitizers on the whole brute-force grid.  It also evaluates the staging kernel's tile map
// (plan.h: tile_block_of / tile_spot, the very functions the kernel calls) for chosen tiles, so
// that a test can check "every tile slot is written exactly once, with the right stream
// position" for shards far too large to generate, e.g. a single run of more than 2^32 elements.
//
// Protocol: one request per input line, whitespace-separated integers after a letter.
//   sharding := ndim shape[ndim] has_stride (stride[ndim])? mesh_ndim mesh_shape[m]
//               (kind dim interleave)[m] coord[m] virtual_threads
//   G sharding max_print
//       -> "G status ndim local_shape[ndim] numel" and, when status == 0 and numel <= max_print,
//          " J j(0) .. j(numel-1)" from vesrng_global_index and " K ..." from
//          vesrng_global_index_general; then " A status new_offset" of vesrng_advance_offset(0).
//   T sharding offset unit_elems tileable big_tileable big_min_elems whole_blocks_only tile_min_elems tile_max_elems
//     tile_min_run_len ntiles tile[ntiles]
//       -> "T status flavour wide units_per_run tile_units n_tiles_total short=0|1" (short: the short form of the
//          tile map applies and was walked next to the general one) and per requested tile
//          " | i0 lim count dummy_writes pos(0) .. pos(lim-1)": the stream position whose value
//          lands in each slot; -1 = never written, -2 = written twice.
#include <cstdint>
#include <cstdio>
#include <iostream>
#include <sstream>
#include <string>
#include <vector>

#include "../include/vesrng.h"
#include "../paper_2509_07003_amd/csrc/geometry.hpp"

using namespace vesrng;

namespace {

struct Desc {
  std::vector<int64_t> shape, stride;
  std::vector<int32_t> mesh, coord;
  std::vector<vesrng_placement> pls;
  vesrng_sharding s{};
};

bool read_sharding(std::istringstream& in, Desc& d) {
  int nd = 0, has_stride = 0, md = 0;
  if (!(in >> nd)) return false;
  d.shape.resize(static_cast<size_t>(nd > 0 ? nd : 0));
  for (auto& v : d.shape) in >> v;
  in >> has_stride;
  if (has_stride) {
    d.stride.resize(d.shape.size());
    for (auto& v : d.stride) in >> v;
  }
  in >> md;
  d.mesh.resize(static_cast<size_t>(md > 0 ? md : 0));
  for (auto& v : d.mesh) in >> v;
  d.pls.resize(d.mesh.size());
  for (auto& p : d.pls) in >> p.kind >> p.dim >> p.interleave;
  d.coord.resize(d.mesh.size());
  for (auto& v : d.coord) in >> v;
  uint64_t theta = 0;
  in >> theta;
  d.s.ndim = nd;
  d.s.global_shape = d.shape.data();
  d.s.global_stride = has_stride ? d.stride.data() : nullptr;
  d.s.mesh_ndim = md;
  d.s.mesh_shape = d.mesh.data();
  d.s.placements = d.pls.data();
  d.s.mesh_coord = d.coord.data();
  d.s.virtual_threads = theta;
  return static_cast<bool>(in);
}

void geometry_request(std::istringstream& in) {
  Desc d;
  int64_t max_print = 0;
  if (!read_sharding(in, d) || !(in >> max_print)) {
    std::printf("G parse-error\n");
    return;
  }
  std::vector<int64_t> local(d.shape.size() + 1, 0);
  int64_t numel = 0;
  const vesrng_status st = vesrng_local_shape(&d.s, local.data(), &numel);
  std::printf("G %d %d", static_cast<int>(st), d.s.ndim);
  if (st == VESRNG_OK) {
    for (int k = 0; k < d.s.ndim; ++k) std::printf(" %lld", static_cast<long long>(local[static_cast<size_t>(k)]));
    std::printf(" %lld", static_cast<long long>(numel));
    if (numel <= max_print) {
      std::vector<int64_t> idx(static_cast<size_t>(numel));
      for (int64_t i = 0; i < numel; ++i) idx[static_cast<size_t>(i)] = i;
      std::vector<uint64_t> j(static_cast<size_t>(numel) + 1);
      const vesrng_status a = vesrng_global_index(&d.s, numel, idx.data(), j.data());
      std::printf(" J %d", static_cast<int>(a));
      for (int64_t i = 0; i < numel; ++i) std::printf(" %llu", static_cast<unsigned long long>(j[static_cast<size_t>(i)]));
      const vesrng_status b = vesrng_global_index_general(&d.s, numel, idx.data(), j.data());
      std::printf(" K %d", static_cast<int>(b));
      for (int64_t i = 0; i < numel; ++i) std::printf(" %llu", static_cast<unsigned long long>(j[static_cast<size_t>(i)]));
    }
  }
  uint64_t next = 0;
  const vesrng_status adv = vesrng_advance_offset(&d.s, 0, &next);
  std::printf(" A %d %llu\n", static_cast<int>(adv), static_cast<unsigned long long>(next));
}

// Stage A of the staging kernel for one tile, on the host: which stream position lands in which slot.
template <typename IT, int NOUT>
void emulate_tile(const PlanT<IT>& plan, const TileArgs<IT>& ta, uint64_t unit_elems, uint64_t tile) {
  const uint64_t tile_elems = static_cast<uint64_t>(ta.tile_units) * unit_elems;
  const uint64_t i0 = tile * tile_elems;
  const uint64_t i1 = (i0 + tile_elems < ta.local_numel) ? i0 + tile_elems : ta.local_numel;
  const int32_t lim = static_cast<int32_t>(i1 - i0);
  const IT wa = tile_block_of<NOUT>(plan, ta, i0);
  const IT count = tile_block_of<NOUT>(plan, ta, i1 - 1) - wa + 1;
  std::vector<long long> slot(static_cast<size_t>(lim), -1);
  long long dummy = 0;
  // The per-wavefront form of the map (64 consecutive block numbers share one tile_wave; used by a measurement
  // variant of the kernel where runs have at least 64 blocks) is walked next to the per-lane form the library
  // uses: where both exist they must agree field by field.
  const bool wave = static_cast<uint64_t>(plan.units_per_run) >= kTileWaveMinBlocks;
  TileWave tw{};
  for (IT k = 0; k < count; ++k) {
    TileSpot spot = tile_spot<NOUT>(plan, i0, lim, static_cast<IT>(wa + k));
    if (wave) {
      if (k % 64 == 0) tw = tile_wave<NOUT>(plan, i0, lim, static_cast<IT>(wa + k));
      const TileSpot ws = tile_spot_of_lane(tw, static_cast<uint32_t>(k % 64));
      // Dead slots beyond a run's last block may differ in where they point, never in being outside [lo, hi).
      const bool live_a = spot.rel + 4 > spot.lo && spot.rel < spot.hi, live_b = ws.rel + 4 > ws.lo && ws.rel < ws.hi;
      if (live_a != live_b || (live_a && (ws.block != spot.block || ws.rel != spot.rel || ws.lo != spot.lo || ws.hi != spot.hi)))
        std::printf(" | OUT-OF-TILE wave-map-mismatch-at-block-%llu", static_cast<unsigned long long>(k));
      spot = ws;
    }
    // The short form of the map, where the library would take it: the same four fields for every block.
    if constexpr (NOUT == 1 && sizeof(IT) == 4) {
      if (ta.same_phase) {
        const TileSpot sp = tile_spot_same_phase(plan, ta, i0, lim, static_cast<IT>(wa + k));
        if (sp.block != spot.block || sp.rel != spot.rel || sp.lo != spot.lo || sp.hi != spot.hi)
          std::printf(" | OUT-OF-TILE short-map-mismatch-at-block-%llu", static_cast<unsigned long long>(k));
        spot = sp;
      }
    }
    // The kernel's own choice between the interior path and the edge path.
    const int32_t rel = spot.rel, lo = spot.lo, hi = spot.hi;
    for (int e = 0; e < 4; ++e) {
      bool inside;
      if (rel >= lo && rel + 4 <= hi) {
        inside = true;
      } else {
        const uint32_t width = static_cast<uint32_t>(hi - lo), base = static_cast<uint32_t>(rel - lo);
        inside = base + static_cast<uint32_t>(e) < width;
      }
      if (!inside) {
        ++dummy;
        continue;
      }
      const long long at = static_cast<long long>(rel) + e;
      if (at < 0 || at >= lim) {  // an out-of-range LDS write in the kernel: report it as such
        std::printf(" | OUT-OF-TILE %lld", at);
        continue;
      }
      long long& s = slot[static_cast<size_t>(at)];
      s = (s == -1) ? static_cast<long long>(spot.block * 4 + static_cast<uint64_t>(e)) : -2;
    }
  }
  std::printf(" | %llu %d %llu %lld", static_cast<unsigned long long>(i0), lim, static_cast<unsigned long long>(count), dummy);
  for (long long s : slot) std::printf(" %lld", s);
}

template <typename IT>
void tiles_typed(const Geometry& g, const RunShape& rs, uint64_t offset, const LaunchChoice& c, uint64_t unit_elems,
                 const std::vector<uint64_t>& tiles) {
  const PlanT<IT> plan = make_plan<IT>(g, rs, offset, c.units_per_run);
  const TileArgs<IT> ta = make_tile_args(plan, c.tile_units, static_cast<uint64_t>(g.local_numel));
  std::printf(" short=%u", ta.same_phase);
  for (uint64_t t : tiles) {
    switch (plan.n_outer) {
      case 0: emulate_tile<IT, 0>(plan, ta, unit_elems, t); break;
      case 1: emulate_tile<IT, 1>(plan, ta, unit_elems, t); break;
      case 2: emulate_tile<IT, 2>(plan, ta, unit_elems, t); break;
      case 3: emulate_tile<IT, 3>(plan, ta, unit_elems, t); break;
      default: emulate_tile<IT, kAnyAxes>(plan, ta, unit_elems, t); break;
    }
  }
}

void tile_request(std::istringstream& in) {
  Desc d;
  uint64_t offset = 0, ntiles = 0;
  LaunchTraits traits;
  int tileable = 0, big = 0, whole = 0;
  if (!read_sharding(in, d) ||
      !(in >> offset >> traits.unit_elems >> tileable >> big >> traits.big_tile_min_elems >> whole >> traits.tile_min_elems >>
        traits.tile_max_elems >> traits.tile_min_run_len >> ntiles)) {
    std::printf("T parse-error\n");
    return;
  }
  traits.tileable = tileable != 0;
  traits.big_tileable = big != 0;
  traits.whole_blocks_only = whole != 0;
  std::vector<uint64_t> tiles(ntiles);
  for (auto& t : tiles) in >> t;
  Geometry g;
  const vesrng_status st = build_geometry(&d.s, &g);
  if (st != VESRNG_OK || !g.boxed || g.local_numel == 0) {
    std::printf("T %d not-a-box-or-empty\n", static_cast<int>(st));
    return;
  }
  const RunShape rs = run_shape(g);
  const LaunchChoice c = choose_launch(g, rs, offset, traits);
  uint64_t total = 0;
  if (c.flavour == kTiled || c.flavour == kTiledBig) {
    const uint64_t per = c.tile_units * traits.unit_elems;
    total = (static_cast<uint64_t>(g.local_numel) + per - 1) / per;
  }
  std::printf("T 0 %d %d %llu %llu %llu", static_cast<int>(c.flavour), c.wide ? 1 : 0,
              static_cast<unsigned long long>(c.units_per_run), static_cast<unsigned long long>(c.tile_units),
              static_cast<unsigned long long>(total));
  if (total != 0) {
    for (auto& t : tiles)
      if (t >= total) t = total - 1;
    if (c.wide) tiles_typed<uint64_t>(g, rs, offset, c, traits.unit_elems, tiles);
    else tiles_typed<uint32_t>(g, rs, offset, c, traits.unit_elems, tiles);
  }
  std::printf("\n");
}

}  // namespace

// "D d n(0) n(1) ..." -> "D q64(0) q64(1) ... | q32 ..." : the kernels' divisions by the launch constant d (64-bit form on
// every n; the multiply-shift 32-bit form on the n below 2^31 when d <= 2^31, the range it is specified for).
void division_request(std::istringstream& in) {
  uint64_t d = 0, n = 0;
  in >> d;
  std::vector<uint64_t> ns;
  while (in >> n) ns.push_back(n);
  const Div64 wide = DivOf<uint64_t>::make(d);
  std::printf("D");
  for (uint64_t x : ns) std::printf(" %llu", static_cast<unsigned long long>(wide.div(x)));
  std::printf(" |");
  if (d <= (1ull << 31)) {
    const Div32 narrow = DivOf<uint32_t>::make(d);
    for (uint64_t x : ns)
      if (x < (1ull << 31)) std::printf(" %u", narrow.div(static_cast<uint32_t>(x)));
  }
  std::printf("\n");
}

// "P sharding offset unit_elems" -> "P wide cut rows_per_piece per_index extent stride pieces_fit": how the library cuts a
// shard that needs 64-bit indices into pieces for the 32-bit kernels (cut = 0: it cannot, the 64-bit kernels serve it).
void pieces_request(std::istringstream& in) {
  Desc d;
  uint64_t offset = 0;
  LaunchTraits traits;
  if (!read_sharding(in, d) || !(in >> offset >> traits.unit_elems)) {
    std::printf("P parse-error\n");
    return;
  }
  traits.tileable = traits.big_tileable = true;
  Geometry g;
  if (build_geometry(&d.s, &g) != VESRNG_OK || !g.boxed || g.local_numel == 0) {
    std::printf("P not-a-box-or-empty\n");
    return;
  }
  const RunShape rs = run_shape(g);
  const LaunchChoice c = choose_launch(g, rs, offset, traits);
  Pieces pc;
  const bool cut = plan_pieces(rs, c.units_per_run, &pc);
  int fit = 1;
  if (cut) {
    const uint64_t last = pc.extent % pc.rows_per_piece;
    fit = fits_32bit(piece_shape(rs, pc.rows_per_piece), c.units_per_run) &&
          (last == 0 || fits_32bit(piece_shape(rs, last), c.units_per_run));
  }
  std::printf("P %d %d %llu %llu %llu %llu %d\n", c.wide ? 1 : 0, cut ? 1 : 0, static_cast<unsigned long long>(pc.rows_per_piece),
              static_cast<unsigned long long>(pc.per_index), static_cast<unsigned long long>(pc.extent),
              static_cast<unsigned long long>(pc.stride), fit);
}

int main() {
  std::string line;
  while (std::getline(std::cin, line)) {
    if (line.empty()) continue;
    std::istringstream in(line.substr(1));
    if (line[0] == 'G') geometry_request(in);
    else if (line[0] == 'T') tile_request(in);
    else if (line[0] == 'D') division_request(in);
    else if (line[0] == 'P') pieces_request(in);
    else std::printf("? unknown request\n");
  }
  return 0;
}
