// Measurement aids, not part of the method: the plain kernels whose rates bound the real ones
// (a fill can go no faster than bare 128-bit stores, fused dropout no faster than its own
// traffic pattern without arithmetic, and nothing faster than the generator alone).
// bench.py runs them next to the real kernels, in the same process.
#include <hip/hip_runtime.h>

#include "../../include/vesrng.h"
#include "philox.h"
#include "stream_store.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
constexpr int kThreads = 256;

// One 16-byte streaming store per thread (the kernels' own store form).
__global__ void __launch_bounds__(kThreads) store_probe(u32x4* out, uint64_t units) {
  const uint64_t t = static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (t >= units) return;
  const uint32_t v = static_cast<uint32_t>(t);
  const u32x4 q = {v, v + 1u, v + 2u, v + 3u};
  vesrng::stream_store(q, out + t);
}

// 16 bytes in, 16 bytes out per thread.
__global__ void __launch_bounds__(kThreads) copy_probe(const u32x4* in, u32x4* out, uint64_t units) {
  const uint64_t t = static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (t >= units) return;
  vesrng::stream_store(__builtin_nontemporal_load(in + t), out + t);
}

// The bf16 dropout kernel's accesses with no arithmetic: 16 bytes in, 16 + 8 bytes out per thread.
__global__ void __launch_bounds__(kThreads)
dropout_traffic_probe(const u32x4* in, u32x4* out, u32x2* mask, uint64_t units) {
  const uint64_t t = static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (t >= units) return;
  const u32x4 v = __builtin_nontemporal_load(in + t);
  const u32x2 m = {v[0] & 0x01010101u, v[1] & 0x01010101u};
  vesrng::stream_store(v, out + t);
  vesrng::stream_store(m, mask + t);
}

// Philox4x32-10 blocks and nothing else (the results are folded and, in practice, never stored).
__global__ void __launch_bounds__(kThreads) philox_probe(uint32_t* out, uint64_t blocks, uint32_t k0, uint32_t k1) {
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * kThreads;
  uint32_t acc = 0;
  for (uint64_t b = static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x; b < blocks; b += stride) {
    uint32_t w[4];
    vesrng::philox_block(b, k0, k1, w);
    acc ^= w[0] ^ w[1] ^ w[2] ^ w[3];
  }
  if (acc == 0x12345678u && k0 == 0x9ABCDEF0u) out[threadIdx.x] = acc;
}

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

}  // namespace

extern "C" vesrng_status vesrng_probe(vesrng_probe_kind kind, uint64_t units, const void* in, void* out, void* out2,
                                      void* hip_stream) {
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (units == 0) return VESRNG_OK;
  if (!out) return VESRNG_ERR_NULL;
  if (misaligned(in) || misaligned(out) || misaligned(out2)) return VESRNG_ERR_ALIGN;
  const uint64_t blocks = (units + kThreads - 1) / kThreads;
  if (blocks > 0x7FFFFFFFull) return VESRNG_ERR_BAD_PARAM;
  const dim3 grid(static_cast<uint32_t>(blocks)), block(kThreads);
  switch (kind) {
    case VESRNG_PROBE_STORE:
      hipLaunchKernelGGL(store_probe, grid, block, 0, stream, static_cast<u32x4*>(out), units);
      break;
    case VESRNG_PROBE_COPY:
      if (!in) return VESRNG_ERR_NULL;
      hipLaunchKernelGGL(copy_probe, grid, block, 0, stream, static_cast<const u32x4*>(in), static_cast<u32x4*>(out),
                         units);
      break;
    case VESRNG_PROBE_DROPOUT_TRAFFIC:
      if (!in || !out2) return VESRNG_ERR_NULL;
      hipLaunchKernelGGL(dropout_traffic_probe, grid, block, 0, stream, static_cast<const u32x4*>(in),
                         static_cast<u32x4*>(out), static_cast<u32x2*>(out2), units);
      break;
    case VESRNG_PROBE_PHILOX:
      // A grid-stride loop over `units` generator blocks on 16 workgroups per compute unit.
      hipLaunchKernelGGL(philox_probe, dim3(256 * 16), block, 0, stream, static_cast<uint32_t*>(out), units, 1234u,
                         0u);
      break;
    default:
      return VESRNG_ERR_BAD_PARAM;
  }
  return hipGetLastError() == hipSuccess ? VESRNG_OK : VESRNG_ERR_HIP;
}

extern "C" vesrng_status vesrng_device_info(int32_t* compute_units, int32_t* shader_clock_khz,
                                            int32_t* memory_clock_khz, int32_t* memory_bus_bits) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return VESRNG_ERR_HIP;
  const struct {
    int32_t* where;
    hipDeviceAttribute_t what;
  } wanted[] = {{compute_units, hipDeviceAttributeMultiprocessorCount},
                {shader_clock_khz, hipDeviceAttributeClockRate},
                {memory_clock_khz, hipDeviceAttributeMemoryClockRate},
                {memory_bus_bits, hipDeviceAttributeMemoryBusWidth}};
  for (const auto& w : wanted) {
    if (!w.where) continue;
    int value = 0;
    if (hipDeviceGetAttribute(&value, w.what, dev) != hipSuccess) return VESRNG_ERR_HIP;
    *w.where = value;
  }
  return VESRNG_OK;
}
