// Measurement aids, not part of the method: the plain kernels whose rates bound the real ones
// (a fill can go no faster than bare 128-bit stores, fused dropout no faster than its own
// traffic pattern without arithmetic, and nothing faster than the generator alone), the
// alternatives the kernels' design choices were measured against, and single-instruction loops
// that give the issue rate of each instruction class.  Built into libvesrng_bench.so, which only
// the benchmark and its test load; it shares the generator and the store helpers with the
// library's kernels so that a probe exercises exactly the kernels' own forms.
#include <hip/hip_runtime.h>

#include "../../include/vesrng_bench.h"
#include "build_id.h"
#include "philox.h"
#include "stream_store.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef u32x4 u32x4_align4 __attribute__((aligned(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
constexpr int kThreads = 256;

enum StoreForm { kStream, kNonTemporal, kPlain };

template <int FORM>
__device__ __forceinline__ void store16(u32x4 v, u32x4* p) {
  if constexpr (FORM == kStream) vesrng::stream_store(v, p);
  else if constexpr (FORM == kNonTemporal) __builtin_nontemporal_store(v, p);
  else *p = v;
}
template <int FORM>
__device__ __forceinline__ void store8(u32x2 v, u32x2* p) {
  if constexpr (FORM == kStream) vesrng::stream_store(v, p);
  else if constexpr (FORM == kNonTemporal) __builtin_nontemporal_store(v, p);
  else *p = v;
}

__device__ __forceinline__ u32x4 pattern(uint64_t t) {
  const uint32_t v = static_cast<uint32_t>(t);
  return u32x4{v, v + 1u, v + 2u, v + 3u};
}

// One 16-byte store per thread.
template <int FORM>
__global__ void __launch_bounds__(kThreads) store_probe(u32x4* out, uint64_t units) {
  const uint64_t t = static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (t >= units) return;
  store16<FORM>(pattern(t), out + t);
}

// The same bytes from a grid-stride loop.
__global__ void __launch_bounds__(kThreads) store_grid_stride_probe(u32x4* out, uint64_t units) {
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * kThreads;
  for (uint64_t t = static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x; t < units; t += stride)
    store16<kStream>(pattern(t), out + t);
}

// Four units per thread, a wave's stores of one round contiguous (unit = 4 * 256 * group + 256 * k + thread).
__global__ void __launch_bounds__(kThreads) store_4_per_thread_probe(u32x4* out, uint64_t units) {
  const uint64_t base = static_cast<uint64_t>(blockIdx.x) * (4 * kThreads) + threadIdx.x;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const uint64_t t = base + static_cast<uint64_t>(k) * kThreads;
    if (t < units) store16<kStream>(pattern(t), out + t);
  }
}

// 16-byte stores whose addresses are only 4-byte aligned: unit t goes to byte 16 t + 4.
__global__ void __launch_bounds__(kThreads) store_unaligned_probe(uint32_t* out, uint64_t units) {
  const uint64_t t = static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (t + 1 >= units) return;  // the last unit would pass the end of the buffer
  __builtin_nontemporal_store(pattern(t), reinterpret_cast<u32x4_align4*>(out + 4 * t + 1));
}

// 16 bytes in, 16 bytes out per thread.
__global__ void __launch_bounds__(kThreads) copy_probe(const u32x4* in, u32x4* out, uint64_t units) {
  const uint64_t t = static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (t >= units) return;
  vesrng::stream_store(__builtin_nontemporal_load(in + t), out + t);
}

// The bf16 dropout kernel's accesses with no arithmetic: 16 bytes in, 16 + 8 bytes out per thread.  WAVES only
// names the launch form in a profiler's trace: 8 = plain, 7 / 6 = launched with 21 / 26 KiB of untouched dynamic
// LDS per workgroup, so that a compute unit holds that many workgroups (of one wave per SIMD each).
template <int FORM, int WAVES = 8>
__global__ void __launch_bounds__(kThreads)
dropout_traffic_probe(const u32x4* in, u32x4* out, u32x2* mask, uint64_t units) {
  const uint64_t t = static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (t >= units) return;
  const u32x4 v = __builtin_nontemporal_load(in + t);
  const u32x2 m = {v[0] & 0x01010101u, v[1] & 0x01010101u};
  store16<FORM>(v, out + t);
  store8<FORM>(m, mask + t);
}

// Variants of the traffic pattern.  LOAD: 0 = non-temporal builtin, 1 = ordinary, 2 = sc1 nt, 3 = sc0 sc1.
template <int LOAD>
__device__ __forceinline__ u32x4 load16(const u32x4* p) {
  if constexpr (LOAD == 0) return __builtin_nontemporal_load(p);
  else if constexpr (LOAD == 1) return *p;
  else {
    u32x4 v;
    // The compiler does not count this load: the wait for its data is written out.
    if constexpr (LOAD == 2) asm volatile("global_load_dwordx4 %0, %1, off sc1 nt\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(p) : "memory");
    else asm volatile("global_load_dwordx4 %0, %1, off sc0 sc1\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(p) : "memory");
    return v;
  }
}
template <int LOAD>
__global__ void __launch_bounds__(kThreads)
dropout_traffic_load_probe(const u32x4* in, u32x4* out, u32x2* mask, uint64_t units) {
  const uint64_t t = static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (t >= units) return;
  const u32x4 v = load16<LOAD>(in + t);
  const u32x2 m = {v[0] & 0x01010101u, v[1] & 0x01010101u};
  vesrng::stream_store(v, out + t);
  vesrng::stream_store(m, mask + t);
}

// Two units per thread: a wave covers 2 KiB of x and y as two contiguous KiB (units base + lane and
// base + 64 + lane) and writes its 1 KiB of mask bytes with ONE 16-byte store per lane.  Only the traffic
// pattern is of interest: the mask bytes written are not the ones of the lane's own units.
__global__ void __launch_bounds__(kThreads)
dropout_traffic_wide_mask_probe(const u32x4* in, u32x4* out, u32x4* mask, uint64_t units) {
  const uint64_t t = static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x;
  const uint32_t lane = threadIdx.x & 63u;
  const uint64_t u0 = 2 * (t - lane) + lane, u1 = u0 + 64;
  if (u1 >= units) return;
  const u32x4 a = __builtin_nontemporal_load(in + u0), b = __builtin_nontemporal_load(in + u1);
  const u32x4 m = {a[0] & 0x01010101u, a[1] & 0x01010101u, b[0] & 0x01010101u, b[1] & 0x01010101u};
  vesrng::stream_store(a, out + u0);
  vesrng::stream_store(b, out + u1);
  vesrng::stream_store(m, mask + t);
}

// Philox4x32-10 blocks and nothing else (the results are folded and, in practice, never stored).
template <bool BITOP3>
__global__ void __launch_bounds__(kThreads) philox_probe(uint32_t* out, uint64_t blocks, uint32_t k0, uint32_t k1) {
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * kThreads;
  uint32_t acc = 0;
  for (uint64_t b = static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x; b < blocks; b += stride) {
    uint32_t w[4];
    vesrng::philox_block<BITOP3>(b, k0, k1, w);
    acc ^= w[0] ^ w[1] ^ w[2] ^ w[3];
  }
  if (acc == 0x12345678u && k0 == 0x9ABCDEF0u) out[threadIdx.x] = acc;
}

// ---- issue-rate loops -------------------------------------------------------------
// One instruction of class CLS on chain value x (and its 64-bit companion y); `u` is wave-uniform.
// The empty asm statements keep the compiler from merging or strength-reducing the chain.
template <int CLS>
__device__ __forceinline__ void alu_step(uint32_t& x, uint32_t& y, uint32_t u) {
  if constexpr (CLS == VESRNG_ALU_MAD_U64_U32) {
    const uint64_t p = static_cast<uint64_t>(u) * x + ((static_cast<uint64_t>(y) << 32) | x);
    x = static_cast<uint32_t>(p);
    y = static_cast<uint32_t>(p >> 32);
  } else if constexpr (CLS == VESRNG_ALU_BITOP3_B32) {
    x = __builtin_amdgcn_bitop3_b32(x, y, u, 0x96);
  } else if constexpr (CLS == VESRNG_ALU_ADD_U32) {
    x = x + u;
    asm volatile("" : "+v"(x));
  } else if constexpr (CLS == VESRNG_ALU_FMA_F32) {
    x = __float_as_uint(__fmaf_rn(__uint_as_float(x), __uint_as_float(u), __uint_as_float(y)));
  } else if constexpr (CLS == VESRNG_ALU_MUL_F32) {
    x = __float_as_uint(__fmul_rn(__uint_as_float(x), __uint_as_float(u)));
    asm volatile("" : "+v"(x));
  } else if constexpr (CLS == VESRNG_ALU_CVT_F32_U32) {
    x = __float_as_uint(static_cast<float>(x));
    asm volatile("" : "+v"(x));
  } else if constexpr (CLS == VESRNG_ALU_LOG_F32) {
    x = __float_as_uint(__builtin_amdgcn_logf(__uint_as_float(x)));
  } else if constexpr (CLS == VESRNG_ALU_SQRT_F32) {
    x = __float_as_uint(__builtin_amdgcn_sqrtf(__uint_as_float(x)));
  } else if constexpr (CLS == VESRNG_ALU_SIN_F32) {
    x = __float_as_uint(__builtin_amdgcn_sinf(__uint_as_float(x)));
  } else if constexpr (CLS == VESRNG_ALU_COS_F32) {
    x = __float_as_uint(__builtin_amdgcn_cosf(__uint_as_float(x)));
  } else if constexpr (CLS == VESRNG_ALU_CVT_PK_BF16_F32) {
    const f32x2 v = {__uint_as_float(x), __uint_as_float(y)};
    x = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    asm volatile("" : "+v"(x));
  } else if constexpr (CLS == VESRNG_ALU_LSHRREV_B32) {
    x = x >> (u & 31u);
    asm volatile("" : "+v"(x));
  } else if constexpr (CLS == VESRNG_ALU_MUL_LO_U32) {
    x = x * y;
    asm volatile("" : "+v"(x));
  } else {  // compare + select
    x = (x <= u) ? y : x;
    asm volatile("" : "+v"(x));
  }
}

template <int CLS>
__global__ void __launch_bounds__(kThreads) alu_probe(uint32_t* out, uint32_t iters, uint32_t u) {
  uint32_t x[8], y[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    x[c] = (threadIdx.x + 1u) * 0x9E3779B9u + static_cast<uint32_t>(c) * 0x01000193u + blockIdx.x;
    y[c] = x[c] ^ 0x3F800000u;
  }
#pragma unroll 1
  for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 8; ++r) {
#pragma unroll
      for (int c = 0; c < 8; ++c) alu_step<CLS>(x[c], y[c], u);
    }
  }
  uint32_t acc = 0;
#pragma unroll
  for (int c = 0; c < 8; ++c) acc ^= x[c] ^ y[c];
  if (acc == 0x12345678u && u == 0x9ABCDEF0u) out[threadIdx.x] = acc;
}

// Spins on dependent fused multiply-adds, then reports the two clocks' elapsed ticks.
__global__ void __launch_bounds__(kThreads) clock_probe(uint64_t* out, uint32_t iters, float u) {
  const uint64_t c0 = clock64(), w0 = wall_clock64();
  float a = static_cast<float>(threadIdx.x), b = a + 1.0f;
#pragma unroll 1
  for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 32; ++r) {
      a = __fmaf_rn(a, u, b);
      b = __fmaf_rn(b, u, a);
    }
  }
  const uint64_t c1 = clock64(), w1 = wall_clock64();
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    out[0] = c1 - c0;
    out[1] = w1 - w0;
    out[2] = static_cast<uint64_t>(__float_as_uint(a + b));  // keeps the loop alive
    out[3] = iters;
  }
}

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

vesrng_status launched() { return hipGetLastError() == hipSuccess ? VESRNG_OK : VESRNG_ERR_HIP; }

template <int CLS>
void launch_alu(uint32_t workgroups, uint32_t iters, uint32_t* out, hipStream_t stream) {
  hipLaunchKernelGGL(alu_probe<CLS>, dim3(workgroups), dim3(kThreads), 0, stream, out, iters, 0x3F7FFFF1u);
}

}  // namespace

extern "C" vesrng_status vesrng_bench_probe(vesrng_probe_kind kind, uint64_t units, const void* in, void* out,
                                            void* out2, void* hip_stream) {
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (units == 0) return VESRNG_OK;
  if (!out) return VESRNG_ERR_NULL;
  if (misaligned(in) || misaligned(out) || misaligned(out2)) return VESRNG_ERR_ALIGN;
  const uint64_t blocks = (units + kThreads - 1) / kThreads;
  if (blocks > 0x7FFFFFFFull) return VESRNG_ERR_BAD_PARAM;
  const dim3 grid(static_cast<uint32_t>(blocks)), block(kThreads);
  int cus = 256;
  u32x4* const o = static_cast<u32x4*>(out);
  const u32x4* const i = static_cast<const u32x4*>(in);
  switch (kind) {
    case VESRNG_PROBE_STORE:
      hipLaunchKernelGGL(store_probe<kStream>, grid, block, 0, stream, o, units);
      break;
    case VESRNG_PROBE_STORE_NT:
      hipLaunchKernelGGL(store_probe<kNonTemporal>, grid, block, 0, stream, o, units);
      break;
    case VESRNG_PROBE_STORE_PLAIN:
      hipLaunchKernelGGL(store_probe<kPlain>, grid, block, 0, stream, o, units);
      break;
    case VESRNG_PROBE_STORE_GRID_STRIDE: {
      int dev = 0;
      if (hipGetDevice(&dev) != hipSuccess ||
          hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return VESRNG_ERR_HIP;
      hipLaunchKernelGGL(store_grid_stride_probe, dim3(static_cast<uint32_t>(cus) * 8u), block, 0, stream, o, units);
      break;
    }
    case VESRNG_PROBE_STORE_4_PER_THREAD:
      hipLaunchKernelGGL(store_4_per_thread_probe, dim3(static_cast<uint32_t>((blocks + 3) / 4)), block, 0, stream, o,
                         units);
      break;
    case VESRNG_PROBE_STORE_UNALIGNED:
      hipLaunchKernelGGL(store_unaligned_probe, grid, block, 0, stream, static_cast<uint32_t*>(out), units);
      break;
    case VESRNG_PROBE_COPY:
      if (!in) return VESRNG_ERR_NULL;
      hipLaunchKernelGGL(copy_probe, grid, block, 0, stream, i, o, units);
      break;
    case VESRNG_PROBE_DROPOUT_TRAFFIC:
    case VESRNG_PROBE_DROPOUT_TRAFFIC_NT:
      if (!in || !out2) return VESRNG_ERR_NULL;
      if (kind == VESRNG_PROBE_DROPOUT_TRAFFIC)
        hipLaunchKernelGGL(dropout_traffic_probe<kStream>, grid, block, 0, stream, i, o, static_cast<u32x2*>(out2), units);
      else
        hipLaunchKernelGGL(dropout_traffic_probe<kNonTemporal>, grid, block, 0, stream, i, o, static_cast<u32x2*>(out2),
                           units);
      break;
    case VESRNG_PROBE_DROPOUT_TRAFFIC_7_WAVES:
    case VESRNG_PROBE_DROPOUT_TRAFFIC_6_WAVES:
      if (!in || !out2) return VESRNG_ERR_NULL;
      if (kind == VESRNG_PROBE_DROPOUT_TRAFFIC_7_WAVES)
        hipLaunchKernelGGL((dropout_traffic_probe<kStream, 7>), grid, block, 21u * 1024u, stream, i, o,
                           static_cast<u32x2*>(out2), units);
      else
        hipLaunchKernelGGL((dropout_traffic_probe<kStream, 6>), grid, block, 26u * 1024u, stream, i, o,
                           static_cast<u32x2*>(out2), units);
      break;
    case VESRNG_PROBE_DROPOUT_TRAFFIC_WIDE_MASK:
      if (!in || !out2) return VESRNG_ERR_NULL;
      hipLaunchKernelGGL(dropout_traffic_wide_mask_probe, dim3(static_cast<uint32_t>((blocks + 1) / 2)), block, 0, stream, i,
                         o, static_cast<u32x4*>(out2), units);
      break;
    case VESRNG_PROBE_DROPOUT_TRAFFIC_LOAD_PLAIN:
    case VESRNG_PROBE_DROPOUT_TRAFFIC_LOAD_SC1:
    case VESRNG_PROBE_DROPOUT_TRAFFIC_LOAD_SC0SC1:
      if (!in || !out2) return VESRNG_ERR_NULL;
      if (kind == VESRNG_PROBE_DROPOUT_TRAFFIC_LOAD_PLAIN)
        hipLaunchKernelGGL(dropout_traffic_load_probe<1>, grid, block, 0, stream, i, o, static_cast<u32x2*>(out2), units);
      else if (kind == VESRNG_PROBE_DROPOUT_TRAFFIC_LOAD_SC1)
        hipLaunchKernelGGL(dropout_traffic_load_probe<2>, grid, block, 0, stream, i, o, static_cast<u32x2*>(out2), units);
      else
        hipLaunchKernelGGL(dropout_traffic_load_probe<3>, grid, block, 0, stream, i, o, static_cast<u32x2*>(out2), units);
      break;
    case VESRNG_PROBE_PHILOX:
      // A grid-stride loop over `units` generator blocks on 16 workgroups per compute unit.
      hipLaunchKernelGGL(philox_probe<true>, dim3(256 * 16), block, 0, stream, static_cast<uint32_t*>(out), units, 1234u,
                         0u);
      break;
    case VESRNG_PROBE_PHILOX_TWO_XOR:
      hipLaunchKernelGGL(philox_probe<false>, dim3(256 * 16), block, 0, stream, static_cast<uint32_t*>(out), units,
                         1234u, 0u);
      break;
    default:
      return VESRNG_ERR_BAD_PARAM;
  }
  return launched();
}

extern "C" vesrng_status vesrng_bench_alu(vesrng_alu_class cls, uint32_t workgroups, uint32_t iters, void* out,
                                          void* hip_stream) {
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (workgroups == 0 || iters == 0) return VESRNG_OK;
  if (!out) return VESRNG_ERR_NULL;
  if (misaligned(out)) return VESRNG_ERR_ALIGN;
  if (workgroups > 0x7FFFFFFFu) return VESRNG_ERR_BAD_PARAM;
  uint32_t* const o = static_cast<uint32_t*>(out);
  switch (cls) {
    case VESRNG_ALU_MAD_U64_U32: launch_alu<VESRNG_ALU_MAD_U64_U32>(workgroups, iters, o, stream); break;
    case VESRNG_ALU_BITOP3_B32: launch_alu<VESRNG_ALU_BITOP3_B32>(workgroups, iters, o, stream); break;
    case VESRNG_ALU_ADD_U32: launch_alu<VESRNG_ALU_ADD_U32>(workgroups, iters, o, stream); break;
    case VESRNG_ALU_FMA_F32: launch_alu<VESRNG_ALU_FMA_F32>(workgroups, iters, o, stream); break;
    case VESRNG_ALU_MUL_F32: launch_alu<VESRNG_ALU_MUL_F32>(workgroups, iters, o, stream); break;
    case VESRNG_ALU_CVT_F32_U32: launch_alu<VESRNG_ALU_CVT_F32_U32>(workgroups, iters, o, stream); break;
    case VESRNG_ALU_LOG_F32: launch_alu<VESRNG_ALU_LOG_F32>(workgroups, iters, o, stream); break;
    case VESRNG_ALU_SQRT_F32: launch_alu<VESRNG_ALU_SQRT_F32>(workgroups, iters, o, stream); break;
    case VESRNG_ALU_SIN_F32: launch_alu<VESRNG_ALU_SIN_F32>(workgroups, iters, o, stream); break;
    case VESRNG_ALU_COS_F32: launch_alu<VESRNG_ALU_COS_F32>(workgroups, iters, o, stream); break;
    case VESRNG_ALU_CVT_PK_BF16_F32: launch_alu<VESRNG_ALU_CVT_PK_BF16_F32>(workgroups, iters, o, stream); break;
    case VESRNG_ALU_LSHRREV_B32: launch_alu<VESRNG_ALU_LSHRREV_B32>(workgroups, iters, o, stream); break;
    case VESRNG_ALU_MUL_LO_U32: launch_alu<VESRNG_ALU_MUL_LO_U32>(workgroups, iters, o, stream); break;
    case VESRNG_ALU_CNDMASK_B32: launch_alu<VESRNG_ALU_CNDMASK_B32>(workgroups, iters, o, stream); break;
    default: return VESRNG_ERR_BAD_PARAM;
  }
  return launched();
}

extern "C" vesrng_status vesrng_bench_clock(uint32_t iters, void* out, void* hip_stream) {
  if (!out) return VESRNG_ERR_NULL;
  if (misaligned(out)) return VESRNG_ERR_ALIGN;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
    return VESRNG_ERR_HIP;
  hipLaunchKernelGGL(clock_probe, dim3(static_cast<uint32_t>(cus)), dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<uint64_t*>(out), iters, 0.99999f);
  return launched();
}

extern "C" vesrng_status vesrng_bench_device_info(int32_t* compute_units, int32_t* shader_clock_khz,
                                                  int32_t* memory_clock_khz, int32_t* memory_bus_bits,
                                                  int32_t* wall_clock_khz) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return VESRNG_ERR_HIP;
  const struct {
    int32_t* where;
    hipDeviceAttribute_t what;
  } wanted[] = {{compute_units, hipDeviceAttributeMultiprocessorCount},
                {shader_clock_khz, hipDeviceAttributeClockRate},
                {memory_clock_khz, hipDeviceAttributeMemoryClockRate},
                {memory_bus_bits, hipDeviceAttributeMemoryBusWidth},
                {wall_clock_khz, hipDeviceAttributeWallClockRate}};
  for (const auto& w : wanted) {
    if (!w.where) continue;
    int value = 0;
    if (hipDeviceGetAttribute(&value, w.what, dev) != hipSuccess) return VESRNG_ERR_HIP;
    *w.where = value;
  }
  return VESRNG_OK;
}
