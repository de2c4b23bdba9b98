// Streaming stores shared by the kernels and the measurement probes (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// 1 (always, in the library): whole units leave with the cache-control bits sc1 nt.  0 only in the
// measurement variant that times the compiler's plain non-temporal store.
#ifndef VESRNG_STREAM_STORE_SC1
#define VESRNG_STREAM_STORE_SC1 1
#endif

namespace vesrng {

typedef uint32_t store_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t store_u32x2 __attribute__((ext_vector_type(2)));

// Streaming stores of whole units: write-through at agent scope with the non-temporal hint
// (cache-control bits sc1 nt).  Measured against the plain non-temporal store the compiler emits
// for __builtin_nontemporal_store (nt alone): fills 6.6-6.8 -> 6.9-7.1 TB/s, the dropout kernel
// 6.45 -> 6.55; system scope (sc0 sc1 nt) gains a little less.  The bits have no builtin, hence
// the inline assembly.  The compiler does not know these are memory instructions, so two things
// it would otherwise do are done by hand:
//  (a) a store of more than 64 bits reads its data registers late; on gfx940-class parts (gfx950
//      included) a vector-ALU write of those registers needs TWO wait states after the store (the
//      open-source compiler's hazard table for these targets; one on older parts).  The 16-byte
//      form therefore carries "s_nop 1" (two wait states); the 8-byte form has no such hazard.
//  (b) its s_waitcnt accounting does not count these stores, which only makes it conservative:
//      nothing here waits on a store, and vector memory operations complete in order.
__device__ __forceinline__ void stream_store(store_u32x4 v, store_u32x4* p) {
#if VESRNG_STREAM_STORE_SC1
  asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
#else
  __builtin_nontemporal_store(v, p);
#endif
}
__device__ __forceinline__ void stream_store(store_u32x2 v, store_u32x2* p) {
#if VESRNG_STREAM_STORE_SC1
  asm volatile("global_store_dwordx2 %0, %1, off sc1 nt" ::"v"(p), "v"(v) : "memory");
#else
  __builtin_nontemporal_store(v, p);
#endif
}
// Four mask bytes of an fp32 dropout unit.  A staging tile of these is not a whole number of
// 128-byte lines, and written through, the partial lines at tile borders cost the ragged fp32
// dropout 12 % (6.25 -> 5.5 TB/s); the plain non-temporal store lets the L2 merge them.
__device__ __forceinline__ void stream_store(uint32_t v, uint32_t* p) { __builtin_nontemporal_store(v, p); }

}  // namespace vesrng
