/* vesrng: single-device-semantic random fills and fused dropout for sharded
 * tensors on AMD Instinct MI355X (gfx950).
 *
 * Method: veScale (arXiv 2509.07003), Section 5 "Consistent Semantics" and
 * Algorithm 1.  Every element of a sharded tensor receives exactly the random
 * value that a single device would give the element with the same global flat
 * index j: the value depends on (seed, offset, j) only, never on the mesh, the
 * placement, the rank or the launch shape.  The local flat index i of a rank's
 * shard is mapped to j through the sharding description (Section 2.2: device
 * mesh, one placement per mesh dimension; Appendix A: InterleavedShard), j is
 * mapped to a position in one global random stream, and a counter-based
 * generator (here Philox4x32-10, Salmon et al., SC'11) produces the value.
 *
 * Stream layout (this library's reading of Algorithm 1's "virtual thread and
 * offset"):  position p = offset + j;  generator block b = p / 4 with counter
 * (lo32 b, hi32 b, 0, 0) and key (lo32 seed, hi32 seed);  the element takes
 * output word p % 4.  `offset` counts draws and must be a multiple of 4.
 *
 * Conventions for every entry point
 *   - All descriptor arrays are HOST memory, read during the call only.
 *   - out / x / y / mask are DEVICE pointers owned by the caller: contiguous
 *     row-major buffers holding exactly the rank's local shard (local_numel
 *     elements), base address aligned to 16 bytes.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream).
 *     Kernels are enqueued and the call returns without synchronising.  The
 *     device that owns the buffers and the stream must be the calling thread's
 *     current HIP device.  The calls can be captured into a HIP graph.
 *   - The library allocates no device memory, keeps no RNG state (the state is
 *     the caller's (seed, offset)) and is re-entrant.
 *   - Errors: a vesrng_status is returned; on any error nothing is launched and
 *     no output is touched.  An empty shard is VESRNG_OK with no launch.
 */
#ifndef VESRNG_H_
#define VESRNG_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Exported from libvesrng.so (the library is built with hidden visibility). */
#define VESRNG_API __attribute__((visibility("default")))

typedef enum {
  VESRNG_OK = 0,
  VESRNG_ERR_NULL = 1,          /* a required pointer is NULL */
  VESRNG_ERR_BAD_SHAPE = 2,     /* ndim outside [0, 8], negative extent, numel >= 2^62 */
  VESRNG_ERR_BAD_MESH = 3,      /* mesh_ndim outside [0, 8] or a mesh extent < 1 */
  VESRNG_ERR_BAD_COORD = 4,     /* mesh coordinate outside its mesh extent */
  VESRNG_ERR_BAD_PLACEMENT = 5, /* Partial / unknown kind, tensor dim out of range,
                                   interleave < 1 or not dividing the dimension */
  VESRNG_ERR_OFFSET_ALIGN = 6,  /* offset is not a multiple of 4 */
  VESRNG_ERR_BAD_PARAM = 7,     /* p outside [0,1], std < 0, high < low, NaN, bad range */
  VESRNG_ERR_DTYPE = 8,         /* dtype not supported by this entry point */
  VESRNG_ERR_UNSUPPORTED = 9,   /* more than 8 sharding placements on one tensor dimension */
  VESRNG_ERR_OVERFLOW = 10,     /* offset + global numel does not fit 64 bits, or bad stride */
  VESRNG_ERR_HIP = 11,          /* the HIP runtime refused the launch */
  VESRNG_ERR_ALIGN = 12         /* a device pointer is not 16-byte aligned */
} vesrng_status;

/* Element type of out / x / y: IEEE binary32, bfloat16, IEEE binary16.  Every operator computes
 * in fp32 and rounds once (nearest even) to the 16-bit types. */
typedef enum { VESRNG_F32 = 0, VESRNG_BF16 = 1, VESRNG_F16 = 2 } vesrng_dtype;

/* Placement of the tensor on ONE mesh dimension (Section 2.2; Appendix A).
 * VESRNG_PARTIAL is listed so that callers can pass DTensor metadata through
 * unchanged; it is always rejected: a partial sum has no per-element value. */
typedef enum {
  VESRNG_REPLICATE = 0,
  VESRNG_SHARD = 1,
  VESRNG_INTERLEAVED_SHARD = 2,
  VESRNG_PARTIAL = 3
} vesrng_placement_kind;

typedef struct {
  int32_t kind;       /* vesrng_placement_kind */
  int32_t dim;        /* tensor dimension that is cut (SHARD, INTERLEAVED_SHARD) */
  int32_t interleave; /* INTERLEAVED_SHARD: number of groups the dimension is seen as */
} vesrng_placement;

/* Sharding description = the metadata Algorithm 1 takes "from DTensor".
 * Placements are applied mesh dimension 0 first.  SHARD cuts the (already cut)
 * dimension of length n into mesh_shape[m] consecutive chunks of ceil(n / P)
 * entries, the last non-empty one possibly shorter, later ones empty.
 * INTERLEAVED_SHARD views the dimension as `interleave` equal groups, cuts each
 * group like SHARD and keeps this rank's chunk of every group, in group order. */
typedef struct {
  int32_t ndim;
  const int64_t* global_shape;        /* [ndim] */
  const int64_t* global_stride;       /* [ndim] in elements, all > 0; NULL = row-major contiguous.
                                         This is Algorithm 1's global stride pi. */
  int32_t mesh_ndim;
  const int32_t* mesh_shape;          /* [mesh_ndim] */
  const vesrng_placement* placements; /* [mesh_ndim] */
  const int32_t* mesh_coord;          /* [mesh_ndim], coordinate of the rank to generate for */
  uint64_t virtual_threads;           /* Algorithm 1's global thread count Theta.  0 (default) = one flat
                                         stream, position offset + j.  Theta > 0 = the algorithm to the
                                         letter: virtual thread tau = j mod Theta, virtual offset
                                         beta = offset + j / Theta, generator counter (lo32 q, hi32 q,
                                         lo32 tau, hi32 tau) with q = beta / 4, output word beta mod 4;
                                         one generator call per element (slower: not the tuned path). */
} vesrng_sharding;

/* Host only.  Local shape (Algorithm 1's upsilon) and element count of the
 * rank's shard.  local_shape may be NULL. */
VESRNG_API vesrng_status vesrng_local_shape(const vesrng_sharding* s, int64_t* local_shape /* [ndim] */,
                                 int64_t* local_numel);

/* Host only.  The offset every rank must use for the next operator: one draw
 * per GLOBAL element, rounded up to a whole generator block
 * (new = offset + 4 * ceil(span / 4), span = largest global flat index + 1, i.e. the
 * element count of a contiguous tensor; with virtual_threads = Theta > 0, span =
 * ceil(that / Theta) steps per virtual thread); mesh, placements and coordinate
 * are ignored, so all ranks step together (Section 5, design (f)). */
VESRNG_API vesrng_status vesrng_advance_offset(const vesrng_sharding* s, uint64_t offset, uint64_t* new_offset);

/* Host only, test hook.  Algorithm 1's i -> j map evaluated on the host by the
 * same decode plan the kernels receive: global_index[k] = j(local_index[k]).
 * Both arrays are host memory of n entries; indices must be < local_numel. */
VESRNG_API vesrng_status vesrng_global_index(const vesrng_sharding* s, int64_t n, const int64_t* local_index,
                                  uint64_t* global_index);

/* Host only, test hook.  The same map evaluated by the general route (each coordinate is
 * mapped back through the placements one by one), which the library uses on the device for
 * shards that are not boxes, e.g. an interleaved dimension cut again across its groups. */
VESRNG_API vesrng_status vesrng_global_index_general(const vesrng_sharding* s, int64_t n,
                                                     const int64_t* local_index, uint64_t* global_index);

/* Raw 32-bit draws, Algorithm 1 with nothing after the generator call: "r <- lambda(alpha,
 * tau_virtual, beta_virtual); chi_i <- r".  out[i] = word (p % 4) of block (p / 4), p = offset + j(i)
 * (or the virtual-thread form when virtual_threads > 0); uint32, local_numel entries.  What the
 * other operators convert; also how a test sees the index map and the generator on their own. */
VESRNG_API vesrng_status vesrng_raw_u32(const vesrng_sharding* s, uint64_t seed, uint64_t offset,
                             uint32_t* out, void* hip_stream);

/* Uniform in [low, high).  u = (draw >> 8) * 2^-24, value = fl(fl(u * fl(high - low)) + low)
 * in fp32; a value that reaches high becomes the largest representable value
 * below high.  BF16 / F16: the fp32 value rounded to nearest even, same upper guard
 * (F16: low and high must lie within +-65504, else VESRNG_ERR_BAD_PARAM).
 * Covers Table 5's uniform_, rand_like and kaiming_uniform_ (pass +-bound). */
VESRNG_API vesrng_status vesrng_uniform(const vesrng_sharding* s, vesrng_dtype dtype, double low, double high,
                             uint64_t seed, uint64_t offset, void* out, void* hip_stream);

/* Normal(mean, std) by Box-Muller on the word pairs (0,1) and (2,3) of a block:
 * u1 = ((a >> 8) + 1) * 2^-24, u2 = (b >> 8) * 2^-24, r = sqrt(-2 ln u1); the
 * even stream position takes r cos(2 pi u2), the odd one r sin(2 pi u2).
 * Evaluated in fp32; agrees with the double-precision definition to
 * 1e-6 * max(|value|, std) (F32) or one ulp of the 16-bit type (BF16, F16).
 * Covers Table 5's normal_ and randn_like. */
VESRNG_API vesrng_status vesrng_normal(const vesrng_sharding* s, vesrng_dtype dtype, double mean, double std,
                            uint64_t seed, uint64_t offset, void* out, void* hip_stream);

/* Fused dropout (Table 5's nn.Dropout): keep = (draw >> 8) < round((1 - p) * 2^24);
 * y = keep ? round_to_dtype(fl32(x * fl32(1 / (1 - p)))) : +0;  mask = keep (0 / 1).
 * One pass: reads x once, writes y and (if non-NULL) the uint8 mask once.
 * y may alias x exactly (in place).  NaN payloads of kept NaN inputs are unspecified.
 * Mask-free use: pass mask = NULL (4 instead of 5 bytes per bf16 element).  Backward pass:
 * the same call on the incoming gradient with the forward's (seed, offset) regenerates the
 * keep decisions: grad_x = keep ? grad_y * scale : 0; no stored mask is read. */
VESRNG_API vesrng_status vesrng_dropout(const vesrng_sharding* s, vesrng_dtype dtype, double p, uint64_t seed,
                             uint64_t offset, const void* x, void* y, uint8_t* mask,
                             void* hip_stream);

/* Fused dropout + residual add (the step that follows dropout in a transformer block):
 * y = round_to_dtype(fl32(residual + (keep ? fl32(x * scale) : +0))), keep / scale / mask as in
 * vesrng_dropout.  One pass: reads x and residual once, writes y and (if non-NULL) mask once.
 * residual is a device pointer with the shape and dtype of x; y may alias x or residual. */
VESRNG_API vesrng_status vesrng_dropout_add(const vesrng_sharding* s, vesrng_dtype dtype, double p, uint64_t seed,
                                 uint64_t offset, const void* x, const void* residual, void* y,
                                 uint8_t* mask, void* hip_stream);

/* Integers in [low, high), 0 < high - low <= 2^32: out = low + draw mod (high - low),
 * stored as int64 (Table 5's randint_like). */
VESRNG_API vesrng_status vesrng_randint(const vesrng_sharding* s, int64_t low, int64_t high, uint64_t seed,
                             uint64_t offset, int64_t* out, void* hip_stream);

/* Text for a status code (a static string, never NULL): the error behaviour stated at the top of
 * this header - every entry point reports through vesrng_status - made printable. */
VESRNG_API const char* vesrng_status_string(vesrng_status st);

#ifdef __cplusplus
}
#endif
#endif /* VESRNG_H_ */
