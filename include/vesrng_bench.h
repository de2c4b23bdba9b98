/* vesrng_bench: measurement aids for the vesrng kernels on MI355X (gfx950).
 *
 * NOT part of the method and not part of libvesrng.so: these entry points live in their own
 * library, libvesrng_bench.so, which only the benchmark and its test load.  They launch plain
 * kernels whose rates bound the real ones - a fill can go no faster than bare 128-bit stores,
 * fused dropout no faster than its own traffic pattern without arithmetic, nothing faster than
 * the generator alone - and single-instruction loops that give the issue rate of each
 * instruction class the fill kernels are made of (the denominators of the ALU roofline).
 *
 * All pointers named `in`, `out`, `out2` are DEVICE pointers, 16-byte aligned, owned by the
 * caller; everything is enqueued on hip_stream (a hipStream_t as void*, NULL = default stream)
 * without synchronising.  Status codes are those of vesrng.h.
 */
#ifndef VESRNG_BENCH_H_
#define VESRNG_BENCH_H_

#include <stdint.h>

#include "vesrng.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Memory and generator probes.  `units` 16-byte units are touched, one per thread unless said
 * otherwise (STORE*: written to out; COPY: in -> out; DROPOUT_TRAFFIC*: 16 bytes in, 16 bytes to
 * out and 8 bytes to out2 per unit, the bf16 dropout kernel's accesses without its arithmetic),
 * or `units` Philox4x32-10 blocks are generated and discarded (PHILOX*; out must still be a
 * valid device pointer of at least 1 KiB). */
typedef enum {
  VESRNG_PROBE_STORE = 0,              /* the kernels' own store: global_store_dwordx4 sc1 nt */
  VESRNG_PROBE_COPY = 1,
  VESRNG_PROBE_DROPOUT_TRAFFIC = 2,
  VESRNG_PROBE_PHILOX = 3,             /* three-way XOR as one v_bitop3_b32 (the kernels' form) */
  /* The alternatives the kernels were measured against: */
  VESRNG_PROBE_STORE_NT = 4,           /* the compiler's plain non-temporal store (nt only) */
  VESRNG_PROBE_STORE_PLAIN = 5,        /* an ordinary store */
  VESRNG_PROBE_STORE_GRID_STRIDE = 6,  /* sc1 nt stores from a grid-stride loop, 8 workgroups per compute unit */
  VESRNG_PROBE_STORE_UNALIGNED = 7,    /* 16-byte nt stores at addresses that are only 4-byte aligned
                                          (out + 4 bytes): what a ragged run's whole blocks look like */
  VESRNG_PROBE_DROPOUT_TRAFFIC_NT = 8, /* the traffic pattern with plain non-temporal stores */
  VESRNG_PROBE_PHILOX_TWO_XOR = 9,     /* the generator written as a ^ b ^ c (two v_xor_b32) */
  VESRNG_PROBE_STORE_4_PER_THREAD = 10, /* sc1 nt stores, four consecutive units per thread */
  /* Alternatives of the dropout traffic pattern (all with sc1 nt stores): */
  VESRNG_PROBE_DROPOUT_TRAFFIC_WIDE_MASK = 11,  /* two units per thread (a wave covers two contiguous KiB), the 16 mask
                                                   bytes of the pair leave as ONE 16-byte store per thread */
  VESRNG_PROBE_DROPOUT_TRAFFIC_LOAD_PLAIN = 12, /* ordinary loads instead of non-temporal ones */
  VESRNG_PROBE_DROPOUT_TRAFFIC_LOAD_SC1 = 13,   /* loads with the cache-control bits sc1 nt */
  VESRNG_PROBE_DROPOUT_TRAFFIC_LOAD_SC0SC1 = 14, /* loads with sc0 sc1 (system scope) */
  /* Resident waves: the kept traffic pattern (kind 2) launched with 21 KiB / 26 KiB of untouched dynamic LDS per
     workgroup, so that a compute unit holds seven / six workgroups of four waves instead of eight.  The library's
     large dropout launches that write a mask run in the seven-wave form. */
  VESRNG_PROBE_DROPOUT_TRAFFIC_7_WAVES = 15,
  VESRNG_PROBE_DROPOUT_TRAFFIC_6_WAVES = 16
} vesrng_probe_kind;

VESRNG_API vesrng_status vesrng_bench_probe(vesrng_probe_kind kind, uint64_t units, const void* in, void* out,
                                            void* out2, void* hip_stream);

/* Issue-rate probes: every thread of `workgroups` groups of 256 executes `iters` loop iterations
 * of 64 instructions of ONE class (8 independent dependency chains, so latency is hidden and the
 * loop measures issue throughput), then folds the results into a store that in practice never
 * happens.  Wave-instructions issued = workgroups * 4 * iters * 64.  `out`: at least 1 KiB. */
typedef enum {
  VESRNG_ALU_MAD_U64_U32 = 0,   /* 32 x 32 -> 64-bit multiply-add: Philox's products */
  VESRNG_ALU_BITOP3_B32 = 1,    /* three-input bit operation: Philox's XORs */
  VESRNG_ALU_ADD_U32 = 2,       /* a simple 32-bit integer operation */
  VESRNG_ALU_FMA_F32 = 3,
  VESRNG_ALU_MUL_F32 = 4,
  VESRNG_ALU_CVT_F32_U32 = 5,
  VESRNG_ALU_LOG_F32 = 6,       /* the transcendental unit: v_log_f32 */
  VESRNG_ALU_SQRT_F32 = 7,
  VESRNG_ALU_SIN_F32 = 8,
  VESRNG_ALU_COS_F32 = 9,
  VESRNG_ALU_CVT_PK_BF16_F32 = 10,
  VESRNG_ALU_LSHRREV_B32 = 11,
  VESRNG_ALU_MUL_LO_U32 = 12,
  VESRNG_ALU_CNDMASK_B32 = 13,  /* compare + select: dropout's keep decision */
  VESRNG_ALU_CLASS_COUNT = 14
} vesrng_alu_class;

VESRNG_API vesrng_status vesrng_bench_alu(vesrng_alu_class cls, uint32_t workgroups, uint32_t iters, void* out,
                                          void* hip_stream);

/* Shader clock under load: one workgroup per compute unit spins on fused multiply-adds for
 * `iters` iterations; thread 0 of workgroup 0 then writes to out (device, 4 x uint64):
 * shader-clock ticks elapsed, constant-rate wall-clock ticks elapsed (the rate of the latter is
 * the device attribute wall_clock_khz below).  Asynchronous like the others. */
VESRNG_API vesrng_status vesrng_bench_clock(uint32_t iters, void* out, void* hip_stream);

/* What the HIP runtime reports for the current device, for the roofline's denominators.  Host
 * pointers; any may be NULL.  On MI355X the runtime reports a memory clock of 2,000,000 kHz and a
 * bus of 8192 bits: HBM3E's 8 Gb/s per pin is four transfers per reported clock, i.e.
 * 4 * clock * bus / 8 = 8.19 TB/s, the published 8 TB/s. */
VESRNG_API vesrng_status vesrng_bench_device_info(int32_t* compute_units, int32_t* shader_clock_khz,
                                                  int32_t* memory_clock_khz, int32_t* memory_bus_bits,
                                                  int32_t* wall_clock_khz);

#ifdef __cplusplus
}
#endif
#endif /* VESRNG_BENCH_H_ */
