// Streaming stores shared by the kernels and the measurement probes (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vesrng {

typedef uint32_t store_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t store_u32x2 __attribute__((ext_vector_type(2)));

// Streaming stores of whole units: write-through at agent scope with the non-temporal hint
// (cache-control bits sc1 nt).  Measured against the plain non-temporal store the compiler emits
// for __builtin_nontemporal_store (nt alone): fills 6.6-6.8 -> 6.9-7.1 TB/s, the dropout kernel
// 6.45 -> 6.55; system scope (sc0 sc1 nt) gains a little less.  The bits have no builtin, hence
// the inline assembly; the compiler does not know these are memory instructions, so (a) the
// 16-byte form is followed by the one wait state the hardware needs before the registers that
// held its data may be rewritten, and (b) its own s_waitcnt accounting merely becomes
// conservative (vector memory operations complete in order on this architecture).
__device__ __forceinline__ void stream_store(store_u32x4 v, store_u32x4* p) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 0" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void stream_store(store_u32x2 v, store_u32x2* p) {
  asm volatile("global_store_dwordx2 %0, %1, off sc1 nt" ::"v"(p), "v"(v) : "memory");
}
// Four mask bytes of an fp32 dropout unit.  A staging tile of these is not a whole number of
// 128-byte lines, and written through, the partial lines at tile borders cost the ragged fp32
// dropout 12 % (6.25 -> 5.5 TB/s); the plain non-temporal store lets the L2 merge them.
__device__ __forceinline__ void stream_store(uint32_t v, uint32_t* p) { __builtin_nontemporal_store(v, p); }

}  // namespace vesrng
