// TEST INFRASTRUCTURE ONLY (see philox.hpp).
//
// Flat C entry points so that the Python tests can call the oracle through
// ctypes.  All pointers are host memory.  Every function returns 0 on success
// and -1 when the description is invalid (the message goes to `err`).
// `threads` > 1 splits the local index range into contiguous slices, one per
// std::thread; the per-element code is the same either way.
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <functional>
#include <thread>

#include "fill.hpp"
#include "philox.hpp"
#include "shard.hpp"

using namespace oracle;

namespace {

// Identity of the sources this library was built from (passed by oracle/build.py); the Python
// front end finds it by scanning the file and rebuilds a stale library.
#ifdef ORACLE_BUILD_ID
__attribute__((used)) const char kOracleBuildId[] = "ORACLE_BUILD_ID=" ORACLE_BUILD_ID;
#endif

struct FlatSharding {
  int32_t ndim;
  const int64_t* global_shape;
  const int64_t* global_stride;  // may be null: row-major contiguous
  int32_t mesh_ndim;
  const int32_t* mesh_shape;
  const int32_t* placement_kind;        // [mesh_ndim]
  const int32_t* placement_dim;         // [mesh_ndim]
  const int32_t* placement_interleave;  // [mesh_ndim]
  const int32_t* mesh_coord;
  uint64_t virtual_threads;
};

Sharding unflatten(const FlatSharding* f) {
  Sharding s;
  s.global_shape.assign(f->global_shape, f->global_shape + f->ndim);
  if (f->global_stride) s.global_stride.assign(f->global_stride, f->global_stride + f->ndim);
  s.mesh_shape.assign(f->mesh_shape, f->mesh_shape + f->mesh_ndim);
  s.mesh_coord.assign(f->mesh_coord, f->mesh_coord + f->mesh_ndim);
  s.virtual_threads = f->virtual_threads;
  for (int m = 0; m < f->mesh_ndim; ++m)
    s.placements.push_back(Placement{f->placement_kind[m], f->placement_dim[m], f->placement_interleave[m]});
  return s;
}

int64_t local_numel_of(const Sharding& s) {
  int64_t n = 1;
  for (const auto& l : index_lists(s)) n *= static_cast<int64_t>(l.size());
  return n;
}

void fail(char* err, int errlen, const char* what) {
  if (err && errlen > 0) std::snprintf(err, static_cast<size_t>(errlen), "%s", what);
}

// The local elements a bulk call covers: [i_begin, i_end), where a negative
// i_end stands for "to the end of the shard".  Output buffers are always
// indexed by the absolute local index i.
struct Range {
  int64_t begin, end;
};
Range clip(const Sharding& s, int64_t i_begin, int64_t i_end) {
  const int64_t n = local_numel_of(s);
  if (i_end < 0 || i_end > n) i_end = n;
  if (i_begin < 0) i_begin = 0;
  return Range{i_begin, std::max(i_begin, i_end)};
}

// Runs body(b, e) over contiguous slices of the range on `threads` threads.
void sliced(Range r, int threads, const std::function<void(int64_t, int64_t)>& body) {
  const int64_t count = r.end - r.begin;
  if (threads < 1) threads = 1;
  if (threads == 1 || count < 4 * threads) {
    body(r.begin, r.end);
    return;
  }
  std::vector<std::thread> pool;
  const int64_t per = (count + threads - 1) / threads;
  for (int t = 0; t < threads; ++t) {
    const int64_t b = std::min<int64_t>(r.end, r.begin + per * t);
    const int64_t e = std::min<int64_t>(r.end, r.begin + per * (t + 1));
    if (b < e) pool.emplace_back(body, b, e);
  }
  for (auto& th : pool) th.join();
}

template <class F>
int guarded(char* err, int errlen, F&& f) {
  try {
    f();
    return 0;
  } catch (const std::exception& e) {
    fail(err, errlen, e.what());
    return -1;
  }
}

}  // namespace

extern "C" {

void oracle_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
  const Block b = philox4x32_10(ctr, key);
  std::memcpy(out, b.w, sizeof b.w);
}

uint32_t oracle_draw(uint64_t seed, uint64_t position) { return draw(seed, position); }

float oracle_uniform_f32(uint32_t x, float low, float high) { return uniform_f32(x, low, high); }
uint16_t oracle_uniform_bf16(uint32_t x, float low, float high) { return uniform_bf16(x, low, high); }
double oracle_normal_f64(uint32_t xa, uint32_t xb, int odd, double mean, double std) {
  return normal_f64(xa, xb, odd != 0, mean, std);
}
uint32_t oracle_dropout_threshold(double p) { return dropout_threshold(p); }
float oracle_dropout_scale(double p) { return dropout_scale(p); }
uint16_t oracle_bf16_from_double(double v) { return bf16_from_double(v); }
uint16_t oracle_bf16_from_float(float v) { return bf16_from_float(v); }
float oracle_float_from_bf16(uint16_t h) { return float_from_bf16(h); }
uint16_t oracle_uniform_f16(uint32_t x, float low, float high) { return uniform_16(kF16, x, low, high); }
uint16_t oracle_f16_from_double(double v) { return f16_from_double(v); }
double oracle_double_from_f16(uint16_t h) { return double_from_f16(h); }

// local_shape[ndim] and *local_numel of the rank's shard.
int oracle_local_shape(const FlatSharding* f, int64_t* local_shape, int64_t* local_numel, char* err,
                       int errlen) {
  return guarded(err, errlen, [&] {
    const auto lists = index_lists(unflatten(f));
    int64_t n = 1;
    for (size_t d = 0; d < lists.size(); ++d) {
      local_shape[d] = static_cast<int64_t>(lists[d].size());
      n *= local_shape[d];
    }
    *local_numel = n;
  });
}

// The global indices held along tensor dimension `dim`, in local order;
// `out` has room for local_shape[dim] entries.
int oracle_index_list(const FlatSharding* f, int32_t dim, int64_t* out, char* err, int errlen) {
  return guarded(err, errlen, [&] {
    const auto lists = index_lists(unflatten(f));
    const auto& l = lists.at(static_cast<size_t>(dim));
    std::copy(l.begin(), l.end(), out);
  });
}

// Global flat index j of every local element, in local order.
int oracle_global_indices(const FlatSharding* f, uint64_t* out, char* err, int errlen) {
  return guarded(err, errlen, [&] {
    const Sharding s = unflatten(f);
    for_each_local(s, 0, local_numel_of(s), [&](int64_t i, uint64_t j) { out[i] = j; });
  });
}

int oracle_raw_u32(const FlatSharding* f, uint64_t seed, uint64_t offset, uint32_t* out,
                   int64_t i_begin, int64_t i_end, int threads, char* err, int errlen) {
  return guarded(err, errlen, [&] {
    const Sharding s = unflatten(f);
    sliced(clip(s, i_begin, i_end), threads, [&](int64_t b, int64_t e) { raw_u32(s, seed, offset, b, e, out); });
  });
}

int oracle_uniform(const FlatSharding* f, int32_t dtype, double low, double high, uint64_t seed,
                   uint64_t offset, void* out, int64_t i_begin, int64_t i_end, int threads, char* err, int errlen) {
  return guarded(err, errlen, [&] {
    const Sharding s = unflatten(f);
    sliced(clip(s, i_begin, i_end), threads, [&](int64_t b, int64_t e) {
      uniform(s, static_cast<DType>(dtype), low, high, seed, offset, b, e, out);
    });
  });
}

int oracle_normal(const FlatSharding* f, int32_t dtype, double mean, double std, uint64_t seed,
                  uint64_t offset, void* out, int64_t i_begin, int64_t i_end, int threads, char* err, int errlen) {
  return guarded(err, errlen, [&] {
    const Sharding s = unflatten(f);
    sliced(clip(s, i_begin, i_end), threads, [&](int64_t b, int64_t e) {
      normal(s, static_cast<DType>(dtype), mean, std, seed, offset, b, e, out);
    });
  });
}

// The unrounded double-precision normals (what the tolerance is measured against).
int oracle_normal_f64_values(const FlatSharding* f, double mean, double std, uint64_t seed,
                             uint64_t offset, double* out, int64_t i_begin, int64_t i_end, int threads, char* err, int errlen) {
  return guarded(err, errlen, [&] {
    const Sharding s = unflatten(f);
    sliced(clip(s, i_begin, i_end), threads, [&](int64_t b, int64_t e) {
      normal_f64_values(s, mean, std, seed, offset, b, e, out);
    });
  });
}

int oracle_dropout(const FlatSharding* f, int32_t dtype, double p, uint64_t seed, uint64_t offset,
                   const void* x, void* y, uint8_t* mask, int64_t i_begin, int64_t i_end, int threads, char* err, int errlen) {
  return guarded(err, errlen, [&] {
    const Sharding s = unflatten(f);
    sliced(clip(s, i_begin, i_end), threads, [&](int64_t b, int64_t e) {
      dropout(s, static_cast<DType>(dtype), p, seed, offset, b, e, x, y, mask);
    });
  });
}

int oracle_dropout_add(const FlatSharding* f, int32_t dtype, double p, uint64_t seed, uint64_t offset,
                       const void* x, const void* residual, void* y, uint8_t* mask, int64_t i_begin, int64_t i_end,
                       int threads, char* err, int errlen) {
  return guarded(err, errlen, [&] {
    const Sharding s = unflatten(f);
    sliced(clip(s, i_begin, i_end), threads, [&](int64_t b, int64_t e) {
      dropout_add(s, static_cast<DType>(dtype), p, seed, offset, b, e, x, residual, y, mask);
    });
  });
}

int oracle_randint(const FlatSharding* f, int64_t low, int64_t high, uint64_t seed, uint64_t offset,
                   int64_t* out, int64_t i_begin, int64_t i_end, int threads, char* err, int errlen) {
  return guarded(err, errlen, [&] {
    if (high <= low || static_cast<uint64_t>(high - low) > (1ull << 32))
      throw std::invalid_argument("need 0 < high - low <= 2^32");
    const Sharding s = unflatten(f);
    sliced(clip(s, i_begin, i_end), threads, [&](int64_t b, int64_t e) {
      randint(s, low, high, seed, offset, b, e, out);
    });
  });
}

uint64_t oracle_advance_offset(const int64_t* global_shape, const int64_t* global_stride, int32_t ndim,
                               uint64_t offset, uint64_t virtual_threads) {
  std::vector<int64_t> stride;
  if (global_stride) stride.assign(global_stride, global_stride + ndim);
  return advance_offset(std::vector<int64_t>(global_shape, global_shape + ndim), stride, offset, virtual_threads);
}

}  // extern "C"
