/* daf.h -- C ABI of the MI355X (gfx950) DAF activation quantize/pack library.
 *
 * The library implements, on one GPU, the storage half of dynamic activation
 * quantization for training: an activation tensor computed by the forward pass is
 * quantized group by group to a per-group bit width, the codes are packed tightly
 * into 32-bit words, and before the backward pass the words are unpacked and
 * dequantized to the original precision (paper Sec. 2.2 "Quantization Calculation",
 * Eq. 1, and the paragraph after it; Sec. 3.1 overview; Sec. 3.3 "Bit Layout
 * Conversion"; Algorithm 2 for the order of codes inside a word).
 *
 * Conventions common to all calls
 *   - Pointers marked DEVICE are addresses in the current HIP device's memory; pointers
 *     marked HOST are ordinary process memory.  The library never takes ownership of a
 *     caller buffer and never writes to an input.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - The tensor is row-major contiguous; it is treated as a flat array of
 *     N = prod(shape) elements.  Group g covers flat indices
 *     [g*group_size, min((g+1)*group_size, N)); the last group may be short.
 *   - Every call returns a daf_status_t (0 = success, negative = error).  No exceptions,
 *     no logging, no abort.  Argument checks that do not need the GPU happen before any
 *     HIP call.
 *   - Packed layout (part of the ABI): group g owns words
 *     [off[g], off[g] + ceil(n_g*bits[g]/32)) of the packed buffer, where off is the
 *     exclusive prefix sum of those word counts.  Inside a group, code j occupies bits
 *     bits[g] wide at bit position j*bits[g] of the group's bit string, and the bit string
 *     fills each 32-bit word from its most significant bit downwards (Algorithm 2:
 *     value j of a word is (w << 4j) >> 28 for 4-bit codes).  Unused low bits of a short
 *     last group's final word are zero.
 *   - Random numbers: element i draws 8 bits from Philox4x32-10 with counter
 *     (lo32(i/16), hi32(i/16), 0, 0) and key (lo32(seed), hi32(seed)): byte i%16 of the
 *     128-bit output taken low word first, low byte first.  The draw depends on
 *     (seed, i) only, not on shape, grouping or launch configuration.
 */
#ifndef DAF_H_
#define DAF_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct daf_plan_s daf_plan_t;         /* opaque; created by daf_plan, freed by daf_plan_destroy */

typedef enum { DAF_F32 = 0, DAF_F16 = 1, DAF_BF16 = 2 } daf_dtype_t;

typedef enum {
  DAF_OK = 0,
  DAF_EINVAL = -1,        /* null pointer, bad shape, bad bits value, misaligned pointer, wrong count */
  DAF_EUNSUPPORTED = -2,  /* group_size not a multiple of 32, unknown dtype, packed size >= 2^32 words */
  DAF_ENOMEM = -3,        /* host or device allocation for the plan failed */
  DAF_EDEVICE = -4,       /* a HIP call or kernel launch failed */
  DAF_ETOOLARGE = -5      /* daf_quantize_pack_static: the tensor needs more scratch than the static buffer holds */
} daf_status_t;

/* Number of random bits spent per element by stochastic rounding (8). */
int daf_rand_bits(void);

/* Human-readable name of a status code; never NULL; static storage. */
const char* daf_status_string(int status);

/* daf_plan -- size and locate the packed representation of one activation tensor.
 *
 * Computes, per group, the number of 32-bit words ceil(n_g * bits[g] / 32) its codes
 * occupy (Sec. 3.3 packs eight 4-bit values per 32-bit word; generalised here to
 * 32/b codes per word) and the exclusive prefix sum of those counts, i.e. each group's
 * word offset in the packed buffer, with a device scan.
 *
 *   shape, ndim   HOST.  ndim >= 1, every dimension >= 1.  N = prod(shape).
 *   group_size    elements per group; a multiple of 32, >= 32.
 *   bits, n_bits  bit width of every group, each in {1,2,4,8}.
 *                 n_bits == 1: `bits` is a HOST pointer to the one width shared by all groups.
 *                 n_bits == G = ceil(N/group_size): `bits` is a DEVICE pointer to G bytes;
 *                 the plan keeps its own device copy.
 *   stream        stream the scan runs on; the call synchronizes it once before returning
 *                 (to read back the total and the validity flag).
 *   out_plan      HOST.  Receives the plan on success, NULL otherwise.
 *
 * Errors: DAF_EINVAL (null pointer, ndim < 1, dimension < 1, n_bits not in {1, G}, a width
 * outside {1,2,4,8}), DAF_EUNSUPPORTED (group_size % 32 != 0 or < 32, total >= 2^32 words),
 * DAF_ENOMEM, DAF_EDEVICE.
 */
int daf_plan(const int64_t* shape, int ndim, int32_t group_size,
             const uint8_t* bits, int64_t n_bits, void* stream, daf_plan_t** out_plan);

/* daf_plan_update / daf_plan_finish -- new widths for an existing per-group-width plan without
 * stopping the stream.  A controller that re-chooses the widths in every iteration (Sec. 3.2: the
 * importance of an activation is re-estimated while training runs; Sec. 3.4.1: the widths follow)
 * keeps one plan per saved tensor and runs
 *     statistics -> widths (e.g. daf_group_minmax, daf_select_bits) -> daf_plan_update -> daf_quantize_pack
 * on one stream, with no host round trip: daf_plan_update only enqueues the scan that rewrites
 * the plan's copy of the widths and its offset array.
 *
 *   plan     a plan created by daf_plan with n_bits == G (per-group widths).
 *   bits     DEVICE, G widths; read by the enqueued scan (keep it alive until the scan has run).
 *            A width outside {1,2,4,8} is replaced by 8 in the plan's copy, so every later call
 *            on the plan stays inside its buffers, and daf_plan_finish reports it.
 *   stream   the scan is enqueued here; calls that use the plan must be ordered after it (same
 *            stream, or an event).
 *
 * After daf_plan_update the exact packed size is not known to the host: daf_plan_packed_words
 * returns daf_plan_packed_words_bound (the size with 8 bits for every group; allocate out_words
 * for that) until daf_plan_finish, which synchronizes `stream` once, fetches the exact size and
 * returns DAF_EINVAL if the last update contained an invalid width.  Calling it is optional.
 *
 * Errors: DAF_EINVAL (null pointer, a one-width plan), DAF_EUNSUPPORTED (the bound reaches 2^32
 * words), DAF_EDEVICE. */
int daf_plan_update(daf_plan_t* plan, const uint8_t* bits, void* stream);
int daf_plan_finish(daf_plan_t* plan, void* stream);
int64_t daf_plan_packed_words_bound(const daf_plan_t* plan);

/* Plan queries (plain host reads, no HIP call). */
int64_t daf_plan_num_elements(const daf_plan_t* plan);   /* N */
int64_t daf_plan_num_groups(const daf_plan_t* plan);     /* G */
int64_t daf_plan_packed_words(const daf_plan_t* plan);   /* words the caller must allocate for out_words */
int32_t daf_plan_group_size(const daf_plan_t* plan);
int32_t daf_plan_uniform_bits(const daf_plan_t* plan);   /* the shared width, or 0 for per-group widths */

/* Which kernels daf_quantize_pack (and its fused variants) use for the whole groups of this plan
 * when the tensor has the given element format; the groups after the last whole tile and the
 * tensor's short last group always go one by one.  A host computation, for tuning and tests.
 *   DAF_ROUTE_TILE      group size a power of two up to 4096: one wave per 4096-element tile
 *   DAF_ROUTE_UNITS     other group sizes up to 4096: one wave per run of whole groups
 *   DAF_ROUTE_LONG      4128 ... 65536 elements: one workgroup per group
 *   DAF_ROUTE_TWO_PASS  longer groups of whole tiles, fewer than 256 groups of 8192 ... 65536, one
 *                       group for the tensor: statistics first, the activation is read twice
 *   DAF_ROUTE_GROUP     everything else: one wave or workgroup per group, element loads
 * Returns the route (>= 0), DAF_EINVAL for a NULL plan, DAF_EUNSUPPORTED for an unknown dtype. */
typedef enum {
  DAF_ROUTE_TILE = 0,
  DAF_ROUTE_UNITS = 1,
  DAF_ROUTE_LONG = 2,
  DAF_ROUTE_TWO_PASS = 3,
  DAF_ROUTE_GROUP = 4
} daf_route_t;
int daf_plan_quantize_route(const daf_plan_t* plan, daf_dtype_t dtype);

/* Copies the G group word offsets to HOST memory (synchronous; for inspection and tests).
 * Works for uniform plans too (offsets are then computed, not stored). */
int daf_plan_copy_offsets(const daf_plan_t* plan, uint32_t* out_off);

/* How daf_unpack_dequantize, daf_unpack_dequantize_batch and daf_unpack_relu_backward write
 * their output for this plan (unpacking next to the consumer, Sec. 3.3): the values are the
 * same either way, only the store instruction differs.
 *   cached = 0 (default)  streaming stores: the call alone is fastest (up to 16 % faster than
 *                         with cached stores); right when the consumer is compute-bound (a
 *                         matrix product), runs later, or the output is small or very large.
 *   cached = 1            ordinary stores: the call alone is slower, but a memory-bound kernel
 *                         that reads the output immediately afterwards finds part of it in
 *                         the caches.  Measured to pay only for outputs of roughly 80-200 MB
 *                         (the two kernels together 4-12 % faster); at 50 MB and at 700 MB and
 *                         more it is equal or slower than the default.
 * A plain host write: not to be changed while a call on the plan is being enqueued from
 * another thread.  Errors: DAF_EINVAL (NULL plan, cached not 0 or 1). */
int daf_plan_set_output_cached(daf_plan_t* plan, int cached);

/* Frees the plan and the device memory it owns.  NULL is allowed. */
void daf_plan_destroy(daf_plan_t* plan);

/* daf_quantize_pack -- forward-pass side: per-group min/max, scale, stochastic-rounding
 * quantization and bit packing, fused in one pass over x.
 *
 * For every group: min and max over the group (Eq. 1's min and max, taken per group), with
 * a zero result stored as +0; scale = (max-min)/(2^b-1) (Eq. 1, left); each element is
 * mapped to v = (x-min) * ((2^b-1)/(max-min)) and rounded to floor(v) or floor(v)+1, up
 * with probability equal to its fractional part quantised to 8 bits (Eq. 1, right, with
 * stochastic rounding in place of `round`; r + 1/2 < frac(v)*256 for the element's random
 * byte r), clamped to 2^b-1; the codes are packed as described at the top of this file.
 * A group whose max equals its min (or whose reciprocal range overflows) gets all-zero
 * codes and scale = range/(2^b-1).
 *
 *   plan       from daf_plan, for this tensor's shape, group size and widths.
 *   x          DEVICE, N elements of `dtype`, 16-byte aligned.  Finite values only, and every
 *              group's range max - min must be finite in binary32 as well (a group that spans
 *              more than 3.4e38, e.g. -3e38 and 3e38, has scale = inf and dequantizes to NaN).
 *   dtype      element type of x.  16-bit inputs are widened exactly to binary32 first.
 *   seed       key of the random stream.
 *   out_words  DEVICE, daf_plan_packed_words(plan) uint32, 4-byte aligned; fully overwritten.
 *   out_min    DEVICE, G floats; out_scale: DEVICE, G floats.  Always binary32.
 *   stream     the call only enqueues work on this stream; it does not synchronize.
 *
 * x is read once for every group size up to 65536 elements (any multiple of 32: a row of 768,
 * 3072 or 11008 elements is as good a group as a power of two); longer groups, fewer than 256
 * groups of 8192 ... 65536 elements (whole tiles), and one group for the whole tensor need the group's
 * statistics before any element can be quantized and read x twice.
 *
 * Concurrency.  Calls on different plans, or on a plan whose daf_plan_quantize_route is not
 * DAF_ROUTE_TWO_PASS, may overlap freely (different streams, several host threads): the plan is
 * only read.  A DAF_ROUTE_TWO_PASS plan owns scratch memory (the per-tile and per-group
 * statistics between its passes) that every call on it writes: calls on ONE such plan, from this
 * entry point, daf_quantize_pack_batch or daf_group_minmax, must not overlap in time -- keep them
 * on one stream, or create one plan per stream (plans are cheap: 8 bytes per 4096 elements).
 *
 * Errors: DAF_EINVAL (null or misaligned pointer), DAF_EUNSUPPORTED (dtype), DAF_EDEVICE.
 */
int daf_quantize_pack(const daf_plan_t* plan, const void* x, daf_dtype_t dtype, uint64_t seed,
                      uint32_t* out_words, float* out_min, float* out_scale, void* stream);

/* daf_quantize_pack_static -- daf_quantize_pack for callers that cannot allocate device memory
 * or hold allocations made for them: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same results, bit for bit.  The difference:
 * where daf_quantize_pack keeps the per-tile and per-group (min, max) pairs of its two-pass route
 * (groups longer than 65536 elements, fewer than 256 groups of 8192 ... 65536 elements, one group
 * for the whole tensor) in memory that daf_plan allocated for the plan, this call keeps them in
 * a buffer of DAF_STATIC_SCRATCH_BYTES that is part of the library's device image (one copy per
 * GPU, held until the process ends).  The call allocates and frees nothing and does not
 * synchronize; the first call on a device looks the buffer's address up once.
 *
 *   limit   the two-pass route needs 8 * (ceil(N / 4096) + G) bytes: at most
 *           DAF_STATIC_SCRATCH_BYTES, i.e. about 1.07e9 elements with one group per tensor;
 *           beyond that the call returns DAF_ETOOLARGE and launches nothing.  Plans on any other
 *           route use no scratch memory and have no limit.
 *   races   all calls on one GPU share the one buffer: two such calls for two-pass plans must not
 *           overlap in time (different streams, or graphs that replay concurrently).  The buffer
 *           keeps the previous call's contents; every entry a call reads it has written first.
 *
 * Errors: as daf_quantize_pack, plus DAF_ETOOLARGE.
 */
#define DAF_STATIC_SCRATCH_BYTES (2 << 20)
int daf_quantize_pack_static(const daf_plan_t* plan, const void* x, daf_dtype_t dtype, uint64_t seed,
                             uint32_t* out_words, float* out_min, float* out_scale, void* stream);

/* daf_unpack_dequantize -- backward-pass side: extract every code (Algorithm 2's rule,
 * for the group's width) and restore xhat = fma(code, scale, min) in binary32, then round
 * to `dtype` (nearest even): the stored activation returns to its original precision
 * before gradients are computed (Sec. 2.2).
 *
 *   words, min, scale   DEVICE, as produced by daf_quantize_pack for the same plan.
 *   bits                DEVICE pointer to G widths, or NULL to use the plan's own copy
 *                       (must be NULL for a uniform plan).
 *   out_x               DEVICE, N elements of `dtype`, 16-byte aligned; fully overwritten.
 *   stream              enqueue only; no synchronization.
 *
 * Errors: DAF_EINVAL, DAF_EUNSUPPORTED (dtype), DAF_EDEVICE.
 */
int daf_unpack_dequantize(const daf_plan_t* plan, const uint32_t* words,
                          const float* min, const float* scale, const uint8_t* bits,
                          void* out_x, daf_dtype_t dtype, void* stream);

/* ---- whole-tensor reduction -------------------------------------------------------------
 *
 * daf_minmax -- minimum and maximum over all N elements of a tensor: the collective reduction
 * that Sec. 3.2 identifies as the expensive part of dynamic quantization control, in the two
 * forms the section describes.
 *
 *   DAF_REDUCE_TWO_PASS  tree reduction inside each workgroup, one (min, max) pair per
 *                        workgroup written to memory, a second launch reduces the pairs
 *                        (Sec. 3.2.1, "parallel reduction").
 *   DAF_REDUCE_ATOMIC    tree reduction inside each workgroup, then the pair is merged into
 *                        one shared result with a float atomic minimum/maximum built from
 *                        integer compare-and-swap (Algorithm 1; Sec. 3.2.2, the hybrid of
 *                        tree and atomic reduction).  One launch.
 *
 *   x, dtype, n     DEVICE, n >= 1 elements, 16-byte aligned, finite values.
 *   method          one of the two above.
 *   workspace       DEVICE, daf_minmax_workspace_bytes() bytes, 16-byte aligned, prepared once
 *                   with daf_minmax_workspace_init (on the same stream or synchronized before
 *                   first use).  Calls that share a workspace must not overlap in time; the
 *                   workspace is left ready for the next call.
 *   out_minmax      DEVICE, 2 floats: min then max, as binary32; a zero result is +0.
 *   stream          enqueue only; no synchronization.
 *
 * Errors: DAF_EINVAL (null or misaligned pointer, n < 1, unknown method), DAF_EUNSUPPORTED
 * (dtype), DAF_EDEVICE.
 */
typedef enum { DAF_REDUCE_TWO_PASS = 0, DAF_REDUCE_ATOMIC = 1 } daf_reduce_method_t;

int64_t daf_minmax_workspace_bytes(void);
int daf_minmax_workspace_init(void* workspace, void* stream);
int daf_minmax(const void* x, daf_dtype_t dtype, int64_t n, int method, void* workspace,
               float* out_minmax, void* stream);

/* ---- statistics for a width controller, and a width rule on the device -------------------
 *
 * daf_group_minmax -- per-group minimum and maximum of x (the statistics of Eq. 1, per
 * group; the reductions a controller needs before it can choose widths, Sec. 3.2), each with
 * a zero stored as +0.  Same grouping, dtypes and alignment rules as daf_quantize_pack; the
 * plan supplies shape and group size (its widths are not used).
 *
 *   out_min, out_max   DEVICE, G floats each.
 *
 * daf_select_bits -- widths by rank quantiles of the range: groups are ranked by
 * (max - min in binary32, group index) ascending and rank r receives
 * classes[floor(r * n_classes / G)], so the smallest ranges get classes[0].  This is the rule
 * the benchmark workloads use in place of the paper's importance-driven controller
 * (Sec. 3.4.1); the result can be passed to daf_plan as its DEVICE bits array.
 *
 *   group_min, group_max   DEVICE, G floats each (e.g. from daf_group_minmax).
 *   classes, n_classes     HOST, 1..4 widths, each in {1,2,4,8}.
 *   out_bits               DEVICE, G bytes.
 *   workspace              DEVICE, daf_select_bits_workspace_bytes(G) bytes, 16-byte aligned;
 *                          contents need no preparation and are garbage afterwards; calls that
 *                          share a workspace must not overlap in time.
 *
 * Both calls only enqueue work on `stream`.
 * Errors: DAF_EINVAL (null/misaligned pointer, G < 1, bad class count or width),
 * DAF_EUNSUPPORTED (dtype; G >= 2^32), DAF_EDEVICE.
 */
int daf_group_minmax(const daf_plan_t* plan, const void* x, daf_dtype_t dtype,
                     float* out_min, float* out_max, void* stream);

/* daf_quantize_pack_metrics -- daf_quantize_pack that also returns, per group, the three
 * importance metrics Sec. 3.2 lists as reductions over the activation (quantization error,
 * quantization variance, magnitude), computed in the same pass (the reduction-fusion idea of
 * Sec. 3.2.3 applied to this pass):
 *   out_metrics[3g]   = sum over group g of (x - xhat)^2   (quantization error), where
 *                       xhat = fma(code, scale, min) in binary32, i.e. the dequantized value
 *                       before any narrowing to a 16-bit dtype;
 *   out_metrics[3g+1] = sum over group g of x^2            (magnitude);
 *   out_metrics[3g+2] = scale^2 * sum over group g of p (1 - p)   (quantization variance: the
 *                       variance of xhat under the stochastic rounding), p = the share of the
 *                       256 random bytes for which the element rounds up.
 * Sums are accumulated in binary32 (per lane, then across lanes, then across loads; the
 * variance as an exact integer per lane), so they agree with a double-precision evaluation to
 * a relative error of about n_g * 2^-24.  words, min and scale are identical to
 * daf_quantize_pack's.
 *
 *   out_metrics   DEVICE, 3*G floats, 4-byte aligned.
 *
 * Errors: as daf_quantize_pack; DAF_EUNSUPPORTED also for plans for which daf_quantize_pack reads
 * x twice (groups longer than 65536 elements, fewer than 256 groups of 8192 ... 65536
 * elements, one group for the tensor).
 */
int daf_quantize_pack_metrics(const daf_plan_t* plan, const void* x, daf_dtype_t dtype, uint64_t seed,
                              uint32_t* out_words, float* out_min, float* out_scale,
                              float* out_metrics, void* stream);

/* ---- several tensors per call ----------------------------------------------------------------
 *
 * A training step saves many activations (Sec. 3.1; e.g. 17 per ResNet-18 step).  These two
 * calls take a list of tensors of one dtype and produce exactly what one daf_quantize_pack /
 * daf_unpack_dequantize per item would, but merge the items into as few kernel launches as
 * their plans allow (consecutive items with the same group size and the same kind of width
 * share a launch, at most 32 per launch), so that the start-up and drain of a launch are paid
 * once per list instead of once per tensor.
 *
 *   items     HOST array; the pointers inside are DEVICE pointers with the alignment rules of
 *             the single-tensor calls; `bits` in a dequantize item may be NULL (the plan's).
 *
 * Errors: DAF_EINVAL (null array or pointer, n_items < 1, misaligned pointer),
 * DAF_EUNSUPPORTED (dtype), DAF_EDEVICE.  Argument checks cover the whole list before any
 * launch.
 */
typedef struct {
  const daf_plan_t* plan;
  const void* x;
  uint64_t seed;
  uint32_t* out_words;
  float* out_min;
  float* out_scale;
} daf_quantize_item_t;

typedef struct {
  const daf_plan_t* plan;
  const uint32_t* words;
  const float* min;
  const float* scale;
  const uint8_t* bits;
  void* out_x;
} daf_dequantize_item_t;

int daf_quantize_pack_batch(const daf_quantize_item_t* items, int32_t n_items, daf_dtype_t dtype, void* stream);
int daf_unpack_dequantize_batch(const daf_dequantize_item_t* items, int32_t n_items, daf_dtype_t dtype, void* stream);

/* ---- producer fusion: the activation function and the quantization in one pass -------------
 *
 * daf_relu_quantize_pack -- for a layer whose saved activation is y = max(z, 0): reads the
 * pre-activation z once, writes y (the forward pass needs it) and the quantized, packed y
 * exactly as daf_quantize_pack(plan, y, ...) would produce them (the element-wise fusion of
 * Sec. 3.2.3 applied to the producing operator; without it y is written by one kernel and
 * read back by the next).  Per element: y = z if z > 0, else +0 (so -0 becomes +0).
 *
 *   z        DEVICE, N elements of dtype, 16-byte aligned, finite.
 *   out_y    DEVICE, N elements of dtype, 16-byte aligned.  May be z itself (in place);
 *            otherwise must not overlap z.
 *   others   as daf_quantize_pack.
 *
 * Errors: as daf_quantize_pack; DAF_EINVAL also for out_y partially overlapping z;
 * DAF_EUNSUPPORTED also for plans for which daf_quantize_pack reads x twice (groups longer than
 * 65536 elements, fewer than 256 groups of 8192 ... 65536 elements, one group for the tensor).
 */
int daf_relu_quantize_pack(const daf_plan_t* plan, const void* z, daf_dtype_t dtype, uint64_t seed, void* out_y,
                           uint32_t* out_words, float* out_min, float* out_scale, void* stream);

/* ---- producer fusion into a matrix product ---------------------------------------------------
 *
 * daf_linear_quantize_pack -- the forward pass of a linear layer, y = x W^T, with the
 * quantization of y as the epilogue of the product's output tile: the kernel that produces the
 * activation also reduces it (per-group min/max), quantizes and packs it (Sec. 3.2.3: fuse the
 * reduction into the producing operator; Sec. 2.2 Eq. 1 and Sec. 3.3 for what is computed).
 * y is written once (the next layer needs it) and never read back for the quantization.
 *
 *   y[m, n] = round_to_dtype( sum_k x[m, k] * W[n, k] ), the products accumulated in binary32 on
 *   the matrix cores (the order of the additions is the kernel's own), rounded to nearest even;
 *   out_words / out_min / out_scale are exactly what daf_quantize_pack(plan, y, ...) gives for
 *   that y, bit for bit (same element map, same Philox bytes, same word layout).
 *
 *   plan     describes y: M * N elements, group size 32, 64 or 128 (a group is a run of
 *            consecutive elements of a row of y), one width or per-group widths.
 *   x        DEVICE, [M, K] row-major, dtype, 16-byte aligned.       M = elements / N.
 *   weight   DEVICE, [N, K] row-major, dtype, 16-byte aligned.
 *   N, K     N and M multiples of 256, K a multiple of 64.
 *   dtype    DAF_F16 or DAF_BF16.
 *   out_y    DEVICE, [M, N] row-major, dtype, 16-byte aligned.
 *   others   as daf_quantize_pack; or all three of out_words, out_min, out_scale null: the
 *            product alone (the same kernel without the quantization in its epilogue).
 *
 * Asynchronous on `stream`.  Errors: DAF_EINVAL (null or misaligned pointer, N or K < 1, N does
 * not divide the plan's element count), DAF_EUNSUPPORTED (binary32, another group size, shapes
 * that are not whole tiles), DAF_EDEVICE.
 */
int daf_linear_quantize_pack(const daf_plan_t* plan, const void* x, const void* weight, int64_t N, int64_t K,
                             daf_dtype_t dtype, uint64_t seed, void* out_y, uint32_t* out_words, float* out_min,
                             float* out_scale, void* stream);
/* The 256 x 256 output tile (row and column, in tiles) that workgroup `id` of a
 * daf_linear_quantize_pack launch over tiles_m x tiles_n tiles computes: the host copy of the map
 * the kernel uses, so that tests without a GPU can check that it visits every tile once.
 * Returns DAF_EINVAL for an id outside [0, tiles_m * tiles_n) or a null pointer. */
int daf_linear_tile_of_workgroup(int32_t id, int32_t tiles_m, int32_t tiles_n, int32_t* tile_m, int32_t* tile_n);

/* ---- consumer fusion for an element-wise consumer -------------------------------------------
 *
 * daf_unpack_relu_backward -- backward of y = max(z, 0) when y is the saved, quantized
 * activation: grad_z[i] = grad_y[i] if xhat[i] > 0, else +0, where xhat[i] is exactly the value
 * daf_unpack_dequantize would write (fma(code, scale, min) rounded to dtype).  The words are
 * unpacked and dequantized in registers and only the sign test leaves them; xhat is never
 * written to memory (the point of unpacking next to the consumer, Sec. 3.3 and Sec. 4.3.1).
 *
 *   words, min, scale, bits   as daf_unpack_dequantize.
 *   grad_y       DEVICE, N elements of dtype, 16-byte aligned.
 *   out_grad_z   DEVICE, N elements of dtype, 16-byte aligned.  May be grad_y itself (in place);
 *                otherwise must not overlap it.
 *
 * Errors: as daf_unpack_dequantize; DAF_EINVAL also for partially overlapping gradients.
 */
int daf_unpack_relu_backward(const daf_plan_t* plan, const uint32_t* words, const float* min, const float* scale,
                             const uint8_t* bits, const void* grad_y, void* out_grad_z, daf_dtype_t dtype,
                             void* stream);

/* ---- consumer fusion for a contraction ---------------------------------------------------------
 *
 * daf_unpack_matmul_grad_weight -- weight gradient of a linear layer y = x W^T whose input x
 * is the saved, quantized activation: with the plan's tensor read as x[M, K] (M = N_elements / K,
 * row-major, groups inside a row) and grad_y[M, N],
 *     out_grad_w[n, k] = sum_m grad_y[m, n] * xhat[m, k]        (binary32, [N, K] row-major)
 * where xhat[m, k] is exactly the value daf_unpack_dequantize would write in `dtype`.  The words
 * are unpacked and dequantized tile by tile inside the product (matrix cores: 16-bit formats
 * with binary32 accumulation, binary32 tensors with binary32 products) and xhat is never
 * written to memory (Sec. 3.3 / Sec. 4.3.1: unpack next to the consumer).  The order of the
 * additions differs from a plain loop, so the result agrees with a double-precision evaluation
 * to about M * 2^-24 relative to sum_m |grad_y| * |xhat|.  The result is deterministic: the
 * same call gives the same bits.
 *
 *   grad_y       DEVICE, M*N elements of dtype, 16-byte aligned.
 *   N, K         columns of grad_y; columns of x (must divide the plan's element count).
 *   out_grad_w   DEVICE, N*K floats, 16-byte aligned.
 *   workspace    DEVICE, daf_unpack_matmul_workspace_bytes(plan, N, K) bytes, 16-byte aligned
 *                (partial sums when m is split over several work-groups; may be NULL if 0; the
 *                size is the same for every element format).
 *
 * Errors: DAF_EINVAL (null or misaligned pointer, K not dividing the element count, missing
 * workspace); DAF_EUNSUPPORTED (M % 32, N % 64, K % 64 or K % group_size non-zero; N or K of
 * 2^24 or more; 2^30 or more packed words); DAF_EDEVICE.  daf_unpack_matmul_workspace_bytes
 * returns -1 for such shapes.
 */
int64_t daf_unpack_matmul_workspace_bytes(const daf_plan_t* plan, int64_t N, int64_t K);
int daf_unpack_matmul_grad_weight(const daf_plan_t* plan, const uint32_t* words, const float* min, const float* scale,
                                  const uint8_t* bits, const void* grad_y, int64_t N, int64_t K, daf_dtype_t dtype,
                                  float* out_grad_w, void* workspace, void* stream);

int64_t daf_select_bits_workspace_bytes(int64_t num_groups);
int daf_select_bits(const float* group_min, const float* group_max, int64_t num_groups,
                    const uint8_t* classes, int32_t n_classes, uint8_t* out_bits,
                    void* workspace, void* stream);

/* daf_select_bits_from_scale -- the same rule with the ranges taken from what an earlier
 * daf_quantize_pack of the tensor left behind, so that choosing the next iteration's widths
 * needs no pass over the activation at all (Sec. 3.4.1: the controller works from statistics
 * gathered while training runs): range_g = scale_g * (2^b_g - 1) in binary32, Eq. 1 (left)
 * turned round, where scale_g is that call's out_scale and b_g the width it used.  Groups are
 * ranked by (range_g, g) and classified exactly as in daf_select_bits.
 *
 *   group_scale    DEVICE, G floats (out_scale of the earlier call).
 *   group_bits     DEVICE, G widths the earlier call used, or NULL: then uniform_bits (1, 2, 4, 8)
 *                  is the width of every group.  May be out_bits itself (the widths are read
 *                  before any is written).
 *   others         as daf_select_bits.
 * Errors: as daf_select_bits; DAF_EINVAL also for group_bits NULL with an invalid uniform_bits.
 */
int daf_select_bits_from_scale(const float* group_scale, const uint8_t* group_bits, int32_t uniform_bits,
                               int64_t num_groups, const uint8_t* classes, int32_t n_classes,
                               uint8_t* out_bits, void* workspace, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DAF_H_ */
