// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11) for gfx950: the value generator
// "lambda" of veScale's Algorithm 1.  Device code only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// 1 (always, in the library): three-way XORs as one v_bitop3_b32.  0 only in the measurement
// variant that times the plain a ^ b ^ c form.
#ifndef VESRNG_PHILOX_BITOP3
#define VESRNG_PHILOX_BITOP3 1
#endif

namespace vesrng {

// a ^ b ^ c in one instruction (v_bitop3_b32, truth table 0x96); the compiler emits two
// v_xor_b32 for the plain expression, and the XORs are half of Philox's instructions.
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
  return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// Philox4x32-10 on counter (c0, c1, c2, c3), key (k0, k1).  BITOP3 = false writes the XORs as
// a ^ b ^ c (only the measurement probe that compares the two forms does).
template <bool BITOP3 = (VESRNG_PHILOX_BITOP3 != 0)>
__device__ __forceinline__ void philox_rounds(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t (&w)[4]) {
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = static_cast<uint64_t>(0xD2511F53u) * c0;
    const uint64_t p1 = static_cast<uint64_t>(0xCD9E8D57u) * c2;
    const uint32_t h1 = static_cast<uint32_t>(p1 >> 32), h0 = static_cast<uint32_t>(p0 >> 32);
    const uint32_t n0 = BITOP3 ? xor3(h1, c1, k0) : (h1 ^ c1 ^ k0);
    const uint32_t n2 = BITOP3 ? xor3(h0, c3, k1) : (h0 ^ c3 ^ k1);
    c1 = static_cast<uint32_t>(p1);
    c3 = static_cast<uint32_t>(p0);
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;  // wave-uniform: lives in scalar registers
    k1 += 0xBB67AE85u;
  }
  w[0] = c0;
  w[1] = c1;
  w[2] = c2;
  w[3] = c3;
}

// Block b of the flat stream: counter (lo32 b, hi32 b, 0, 0).
template <bool BITOP3 = (VESRNG_PHILOX_BITOP3 != 0)>
__device__ __forceinline__ void philox_block(uint64_t b, uint32_t k0, uint32_t k1, uint32_t (&w)[4]) {
  philox_rounds<BITOP3>(static_cast<uint32_t>(b), static_cast<uint32_t>(b >> 32), 0u, 0u, k0, k1, w);
}

}  // namespace vesrng
