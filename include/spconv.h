/*
 * spconv.h - C ABI of the MI355X (gfx950) sparse 3-D convolution library.
 *
 * The library computes the sparse convolution of the paper's Equation 1
 * (Section 2.1),
 *
 *     x_out[n] = sum over delta in Delta^3(K), sum over j of
 *                1[p_j = s*q_n + delta] * (x_in[j] . W[delta]),
 *
 * in the implicit-GEMM dataflow (Sections 2.2.3, 3.1): an output-stationary
 * kernel map M[n_out][K^3] is built first (M[n][k] = input row that is the
 * k-th neighbour of output n, or -1), then the feature kernels gather input
 * rows through M on their way into LDS and multiply them by the weight slice
 * of the offset on the matrix cores, accumulating in fp32 registers.  Output
 * rows can be visited in bitmask-sorted order and the loop over offsets can be
 * cut into several separately sorted splits whose partial sums are added by a
 * reduction kernel (Sections 2.2.3 and 4.1).  Forward and input gradient can
 * also run in the fetch-on-demand dataflow (Section 2.2.2: the weight-stationary
 * pair lists of the map, atomic scatter; spconv_config.kernel = 3), and the
 * tuners choose between the two.
 *
 * Conventions (the paper gives only the set Delta^3(K); these are fixed here):
 *   - a coordinate row is (b, x, y, z), int32; b is the batch index, never
 *     offset or strided; x, y, z in [-32768, 32767], b in [0, 65534];
 *   - offset index k = ((dx+r)*K + (dy+r))*K + (dz+r), r = (K-1)/2, i.e. x
 *     slowest, z fastest; K is 1 or 3, or 2 with offsets {0, 1}^3 (r = 0: the
 *     paper defines odd K only; with stride 2 this is the non-overlapping
 *     2x2x2 layer); bit k of a neighbour bitmask is 1u<<k.  K = 5 (the 125
 *     offsets of Section 2.1's neighbourhood) exists for submanifold maps
 *     (stride 1, not transposed, synchronous build): the library holds such
 *     a map as five planes of 25 offsets (dx = g - 2; offset k is offset
 *     k % 25 of plane k / 25), runs forward and dgrad plane by plane and sums
 *     the planes like the parts of a split, and sorts each plane by its own
 *     25-bit mask.  spconv_kmap_export_perm then counts parts over the
 *     planes (split = plane * n_split + part); the tuners, the paired
 *     transposed kmap, fetch-on-demand and spconv_fwd_noalloc refuse a K = 5
 *     kmap with SPCONV_EINVAL;
 *   - output q reads the input at s*q + delta with W[delta] (no kernel flip);
 *   - stride 1: P_out = P_in in input order; stride s > 1: P_out = unique
 *     floor(p / s), sorted ascending lexicographically in (b, x, y, z);
 *   - transposed: the caller passes the FINE set (the outputs of the
 *     transposed convolution); its inputs are the coarse set P_out(fine, s),
 *     in that sorted order, and y[j] = sum over (i, delta) with
 *     fine_j = s*coarse_i + delta of x[i] . W[delta].
 *
 * Memory: every pointer named "device" is a device pointer owned by the
 * caller (the library never frees caller memory); tensors are row-major and
 * contiguous, feature rows 16-byte aligned.  The opaque spconv_kmap owns all
 * of its buffers (hash table, maps, masks, permutations, cached reordered
 * maps, scratch) and releases them in spconv_kmap_destroy.  A kmap caches
 * derived data on first use, so concurrent calls on ONE kmap from several
 * host threads or several streams are not supported.
 *
 * Streams: `stream` is a hipStream_t passed as void* (NULL = the null
 * stream).  Calls are asynchronous with respect to the host except where
 * stated.  All work of one kmap must be issued on one stream (or the caller
 * orders the streams).
 *
 * Errors: every function returns 0 on success or a negative spconv_status.
 * Nothing is written to outputs on SPCONV_EINVAL / SPCONV_ESHAPE.
 */
#ifndef SPCONV_H
#define SPCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPCONV_API __attribute__((visibility("default")))

typedef enum spconv_status {
  SPCONV_OK = 0,
  SPCONV_EINVAL = -1,  /* null pointer, negative size, unsupported K / stride / dtype / channels / config */
  SPCONV_ERANGE = -2,  /* a coordinate lies outside the packable range */
  SPCONV_EDUP = -3,    /* two input rows carry the same coordinate (Section 2 assumes Unique was applied) */
  SPCONV_ENOMEM = -4,  /* device or host allocation failed */
  SPCONV_ESHAPE = -5,  /* channel counts or row counts do not fit the kmap */
  SPCONV_EHIP = -6,    /* a HIP call failed; see spconv_last_hip_error() */
  SPCONV_ENOPLAN = -7, /* spconv_fwd_noalloc: the plan of this configuration was not prepared */
  SPCONV_ELIMIT = -8   /* spconv_fwd_noalloc: partial sums exceed SPCONV_NOALLOC_SCRATCH_BYTES */
} spconv_status;

typedef enum spconv_dtype { SPCONV_F32 = 0, SPCONV_F16 = 1, SPCONV_BF16 = 2 } spconv_dtype;

typedef enum spconv_op { SPCONV_OP_FWD = 0, SPCONV_OP_DGRAD = 1, SPCONV_OP_WGRAD = 2 } spconv_op;

typedef struct spconv_kmap spconv_kmap; /* opaque */

/* Dataflow parameters (the design space of Section 4.1).  Zero-initialise for
 * the defaults.
 *   n_split     0: unsorted implicit GEMM, rows in map order, one pass.
 *               s >= 1 (at most 4 and at most K^3): the K^3 offsets are cut into s contiguous
 *               ranges [floor(i*V/s), floor((i+1)*V/s)); in each range the
 *               rows are visited in ascending order of that range's bitmask
 *               bits (stable), and for s > 1 the fp32 partial sums of the
 *               ranges are added by a reduction kernel.
 *   kernel      which fwd / dgrad kernel runs (F32 has one implicit-GEMM kernel,
 *               which runs for 0, 1 and 2, and one fetch-on-demand kernel with
 *               tiles of 64 pairs x 64 channels for 3):
 *               1: weights of a split resident in LDS, one wave per 16-row
 *                  block (needs reduced channels <= 128 and the split's
 *                  weight slices for tile_n channels to fit in LDS, else
 *                  SPCONV_EINVAL); tile_m is ignored;
 *               2: workgroup tiles of tile_m rows, weights streamed per offset;
 *               3: the fetch-on-demand dataflow of Section 2.2.2 instead of
 *                  implicit GEMM: the weight-stationary pair lists of the map
 *                  (the ones wgrad walks) in tiles of tile_m pairs of one
 *                  offset, products added to an fp32 accumulator with atomic
 *                  adds, rounded once to the output type.  No multiply is
 *                  spent on absent neighbours; results are the same up to
 *                  the order of the fp32 additions (which varies from call to
 *                  call).  Needs n_split = 0, else SPCONV_EINVAL;
 *               0: never 3; 1 where it fits and either the output is at most two
 *                  column tiles wide or (column tiles x reduced channels x
 *                  rows) is small, else 2.
 *   tile_m      output rows per workgroup of kernel 2: 64, 128 or 256 (0 = 64 or
 *               128, from the row count and the channel counts);
 *               pairs per workgroup of kernel 3: 64 or 128 (0 = 64; F32: 64 only).
 *   tile_n      output channels per workgroup: 16, 32, 64 (kernel 1) or 32, 64,
 *               128 (kernels 2 and 3); 0 = chosen from the channel counts (and,
 *               for kernel 2, from how many workgroups the rows give).
 *   wgrad_pairs target number of (output,input) pairs per wgrad workgroup
 *               (0 = chosen from the pair count); ignored by fwd / dgrad.
 *   flags       SPCONV_FLAG_SLABS: the sort key of every row of a sorted map (n_split >= 1)
 *               starts with the row's spatial slab (eight equal slabs along the longest axis
 *               of the coordinates), and the kernel with resident weights hands each of the
 *               chip's eight L2 domains a contiguous range of that order, so that its gathers
 *               stay within about one eighth of the input.  Any visiting order gives the same
 *               result; this one trades some lock-step redundancy for less traffic beyond
 *               L2.  Without the flag the library uses slabs from 2^20 rows on.
 */
typedef struct spconv_config {
  int32_t n_split;
  int32_t tile_m;
  int32_t tile_n;
  int32_t wgrad_pairs;
  int32_t kernel;
  int32_t flags;
  int32_t reserved[2];
} spconv_config;

/* spconv_config.flags */
#define SPCONV_FLAG_SLABS 1 /* sorted maps (n_split >= 1): see above */

/* Kernel-map construction ("mapping operations", Sections 3.1, 4.2, 6.2).
 *   coords      device, int32 [N][4] = (b, x, y, z), unique rows.
 *   N           number of rows, >= 0 (N = 0 gives an empty kmap).
 *   K           kernel size: 1, 3, 2 (K = 2 only together with stride 2), or 5 (stride 1, transposed = 0 only).
 *   stride      >= 1 (stride 1 with transposed = 0 is the submanifold case).
 *   transposed  0: coords are P_in.  1: coords are the fine output set.
 *   out         receives a new kmap; release with spconv_kmap_destroy.
 * Synchronises `stream` once (to read the error flags and, for stride > 1,
 * the number of coarse points).  Errors: EINVAL, ERANGE, EDUP, ENOMEM, EHIP;
 * on error *out is NULL. */
SPCONV_API int spconv_build_kmap(const int32_t* coords, int64_t N, int K, int stride, int transposed,
                      void* stream, spconv_kmap** out);

/* The same build without the synchronisation, for pipelines that must not stall: for K = 3,
 * stride 1, transposed 0 the call only enqueues work and returns a usable kmap at once; range
 * and duplicate errors stay on the device until spconv_kmap_status is called (any time later,
 * typically one iteration behind).  Until then the pair count is unknown: wgrad sizes its work
 * list from the bound n_out * K^3 (surplus workgroups exit immediately).  A kmap built from
 * invalid rows is safe to run (all indices stay in range) but its results are meaningless.
 * Other map kinds are built synchronously, exactly as by spconv_build_kmap. */
SPCONV_API int spconv_build_kmap_async(const int32_t* coords, int64_t N, int K, int stride, int transposed,
                                       void* stream, spconv_kmap** out);

/* Stride-1 convolution whose output set is not the input set (Equation 1, Section 2.1, with
 * P_out != P_in): P_out = every point that has at least one input in its K^3 neighbourhood,
 * { q : q + delta in P_in for some delta }, sorted ascending lexicographically in (b, x, y, z); the
 * map is M[n][k] = j with p_j = q_n + delta_k as always.  K is 1 or 3.  A layer on this kmap grows
 * the occupied set by one voxel in every direction (the "dilating" convolution of dense-output
 * heads); forward, dgrad and wgrad run on it like on any other kmap.  Synchronises `stream` once
 * (size of P_out, error flags).  Errors: EINVAL, ERANGE (also when an output would lie outside the
 * packable coordinate range), EDUP, ENOMEM, EHIP.  spconv_kmap_transpose refuses such a kmap. */
SPCONV_API int spconv_build_kmap_dilated(const int32_t* coords, int64_t N, int K, void* stream, spconv_kmap** out);

/* The kmap of the transposed convolution that pairs with km: the same (input, output) pairs with
 * the two roles exchanged, i.e. exactly what spconv_build_kmap returns for the same rows with
 * `transposed` flipped, without building a table or probing again (one scatter pass over km's
 * map, unless km's dgrad has made it already; nothing is copied).  An encoder-decoder network derives each up-convolution's kmap from its
 * down-convolution this way.  *out shares km's tables and coordinate sets (reference-counted: destroy both
 * kmaps, in either order) and the plans cached on them, so the rule against concurrent calls on one kmap
 * covers the pair.  `stream` must be ordered after the work that built km; an unresolved asynchronous build is resolved
 * first (one synchronisation) and its error, if any, is returned.  Errors: EINVAL, ENOMEM,
 * EHIP, ERANGE / EDUP of a pending build; on error *out is NULL. */
SPCONV_API int spconv_kmap_transpose(spconv_kmap* km, void* stream, spconv_kmap** out);

/* The K = 1, stride 1 kmap over one of km's row sets: its input rows (on_outputs = 0) or its
 * output rows (on_outputs = 1).  A 1x1x1 convolution (Eq. 1 with the single offset 0) pairs every
 * row with itself, so nothing is hashed or probed: the rows were validated when km was built, and
 * the call writes an identity map and copies the coordinates (exactly what spconv_build_kmap
 * returns for those rows with K = 1, at a fraction of its cost: the projection shortcuts of a
 * residual network take their kmaps from the level's 3x3x3 kmap this way).  *out is independent
 * of km.  `stream` must be ordered after the work that built km; an unresolved asynchronous build
 * is resolved first and its error, if any, is returned.  Errors: EINVAL (null arguments,
 * on_outputs other than 0 or 1), ENOMEM, EHIP, ERANGE / EDUP of a pending build; on error *out
 * is NULL. */
SPCONV_API int spconv_kmap_pointwise(spconv_kmap* km, int on_outputs, void* stream, spconv_kmap** out);

/* Resolves an asynchronous build: waits until the build's last kernel has published its result
 * (a word in pinned host memory that the host reads: nothing is recorded on the stream, and no
 * wait at all once that kernel has finished), returns SPCONV_OK, SPCONV_ERANGE or SPCONV_EDUP, and
 * makes the pair count available.  The verdict stays with the kmap: every later call returns it
 * again, also when another call (spconv_kmap_sizes asking for the pair count,
 * spconv_kmap_mac_units, a tuner) was the one that waited for the build.  SPCONV_OK at once for
 * kmaps built synchronously (their errors were returned by the build).  `stream` is unused for
 * kmaps built asynchronously (the build's own stream is waited for if the result is late). */
SPCONV_API int spconv_kmap_status(spconv_kmap* km, void* stream);

/* Row counts of the two sides of the map and the number of present pairs
 * sum_k |M_k| (the "effective MACs" of Section 2.2.3 in units of
 * C_in*C_out).  Any pointer may be NULL.  Asking for n_pairs the first time
 * runs a small reduction on the kmap's build stream and synchronises it. */
SPCONV_API int spconv_kmap_sizes(const spconv_kmap* km, int64_t* n_in, int64_t* n_out, int64_t* n_pairs);

/* Copies P_out, the output coordinates q_n of Equation 1 (Section 2.1), int32 [n_out][4], to dst
 * (device): the caller's rows for stride 1, the sorted unique floor(p / s) otherwise. */
SPCONV_API int spconv_kmap_out_coords(const spconv_kmap* km, int32_t* dst, void* stream);

/* Copies P_in, the input coordinates p_j of Equation 1 (Section 2.1), int32 [n_in][4], to dst
 * (device): the caller's rows for transposed = 0, the sorted coarse set for transposed = 1. */
SPCONV_API int spconv_kmap_in_coords(const spconv_kmap* km, int32_t* dst, void* stream);

/* Copies the output-stationary map of Section 3.1 to dst (device): int32 [n_out][K^3],
 * M[n][k] = j where p_j = s*q_n + delta_k (the pairs that Equation 1 sums over), -1 = absent. */
SPCONV_API int spconv_kmap_export(const spconv_kmap* km, int32_t* dst, void* stream);

/* Copies the neighbour bitmasks (uint32 [n_out], Section 2.2.3) to dst (device).  K = 5: uint32
 * [n_out][4], bit k of a row's 125-bit mask in bit k % 32 of word k / 32; dst 16-byte aligned. */
SPCONV_API int spconv_kmap_export_mask(const spconv_kmap* km, uint32_t* dst, void* stream);

/* Builds (and caches in the kmap) everything op needs under cfg before the
 * first compute call: the input-side map for dgrad of strided / transposed
 * maps, per-split bitmask argsort, reordered and padded maps and per-tile
 * masks (Sections 2.2.3, 3.2, 4.1), the offset-major map and work list of
 * wgrad.  The compute calls do this themselves on first use; calling it
 * explicitly lets the mapping cost be timed apart from the kernels
 * (Section 6.1 separates them the same way).  May synchronise the stream. */
SPCONV_API int spconv_kmap_prepare(spconv_kmap* km, spconv_op op, const spconv_config* cfg_or_null, void* stream);

/* Drops every cached plan (not the map itself), so that mapping can be timed again: the sorted
 * and reordered maps of both tables, the pair lists, and the input-side table unless a transposed
 * partner (spconv_kmap_transpose) uses it as its map.  Plans cached on tables shared with a partner
 * are dropped for both.  Synchronises the device. */
SPCONV_API int spconv_kmap_drop_plans(spconv_kmap* km);

/* Permutation of split `split` of the cached plan of (op, cfg): int32
 * [n_rows] with row r of the sorted order = original row perm[r] (identity
 * for n_split = 0).  For tests of the sort invariants. */
SPCONV_API int spconv_kmap_export_perm(spconv_kmap* km, spconv_op op, const spconv_config* cfg_or_null,
                            int split, int32_t* dst, void* stream);

/* Executed and effective MAC units (units of C_in*C_out MACs) of op under cfg
 * in this library's lock-step model: a block of 16 consecutive rows of the
 * visiting order (one MFMA block) pays for offset k whenever one of them has
 * neighbour k (the quantity plotted in Section 4.1).  Synchronises the stream. */
SPCONV_API int spconv_kmap_mac_units(spconv_kmap* km, spconv_op op, const spconv_config* cfg_or_null,
                          int64_t* executed, int64_t* effective, void* stream);

SPCONV_API void spconv_kmap_destroy(spconv_kmap* km);

/* Forward, Equation 1:  out[n] = sum_k feats[M[n][k]] . W[k].
 *   feats   device [n_in][C_in]   weights device [K^3][C_in][C_out]
 *   out     device [n_out][C_out], fully overwritten.
 * dtype applies to feats, weights and out; accumulation is fp32 with one
 * rounding (to nearest even) at the end.  C_in and C_out must be multiples
 * of 8 (F16/BF16) or 4 (F32), else SPCONV_EINVAL.  km is not const because plans are cached. */
SPCONV_API int spconv_fwd(const void* feats, const void* weights, spconv_kmap* km, int C_in, int C_out,
               spconv_dtype dtype, const spconv_config* cfg_or_null, void* out, void* stream);

/* spconv_fwd for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and same result as
 * spconv_fwd, but the call makes no allocation of any kind (no hipMalloc / hipFree, no allocator
 * callback, no pool):
 *   - the plan of cfg must exist already, made by spconv_kmap_prepare(km, SPCONV_OP_FWD, cfg) or by
 *     an earlier spconv_fwd with the same cfg; otherwise SPCONV_ENOPLAN.  kernel = 3 (fetch on
 *     demand) is refused with SPCONV_EINVAL;
 *   - the fp32 partial sums of n_split >= 2 (n_split * n_out * C_out * 4 bytes) go to a fixed
 *     array of SPCONV_NOALLOC_SCRATCH_BYTES that every GPU the library runs on holds until the
 *     process ends; a larger need is refused with SPCONV_ELIMIT and nothing is launched.
 * All calls on one GPU share that array and it keeps the previous call's contents (every element a
 * call reads it has written before, so nothing needs clearing); two calls that overlap on one GPU -
 * different streams, or several host threads - race on it and must be ordered by the caller. */
#define SPCONV_NOALLOC_SCRATCH_BYTES (64u << 20)
SPCONV_API int spconv_fwd_noalloc(const void* feats, const void* weights, spconv_kmap* km, int C_in, int C_out,
                       spconv_dtype dtype, const spconv_config* cfg_or_null, void* out, void* stream);

/* Input gradient of Equation 1 (the dgrad kernel of Section 4.2):
 *   din[j] = sum over (n, k) with M[n][k] = j of dout[n] . W[k]^T.
 *   dout device [n_out][C_out]   weights as in spconv_fwd
 *   din  device [n_in][C_in], fully overwritten. */
SPCONV_API int spconv_dgrad(const void* dout, const void* weights, spconv_kmap* km, int C_in, int C_out,
                 spconv_dtype dtype, const spconv_config* cfg_or_null, void* din, void* stream);

/* Weight gradient of Equation 1 (the wgrad kernel of Sections 4.2, 6.2):
 *   dweights[k] = sum over n with M[n][k] >= 0 of feats[M[n][k]]^T . dout[n].
 *   dweights device fp32 [K^3][C_in][C_out] whatever dtype is, fully overwritten. */
SPCONV_API int spconv_wgrad(const void* feats, const void* dout, spconv_kmap* km, int C_in, int C_out,
                 spconv_dtype dtype, const spconv_config* cfg_or_null, float* dweights, void* stream);

/* Picks the configuration of the design space of Section 4.1 (dataflow: implicit
 * GEMM or fetch-on-demand; number of splits, sorted or not; tile sizes) with the
 * lowest measured time for op on
 * this kmap and these channel counts, where time = kernel time + mapping time
 * / layers_sharing_kmap (layers that use the same maps form a group and share
 * the mapping cost, Section 4.2).  Blocking: allocates scratch tensors, runs
 * and times every candidate on `stream`.  best receives the winner;
 * best_us (may be NULL) its time in microseconds. */
SPCONV_API int spconv_tune(spconv_kmap* km, int C_in, int C_out, spconv_dtype dtype, spconv_op op,
                int layers_sharing_kmap, spconv_config* best, float* best_us, void* stream);

/* One layer of a group: the layers of a network that use the same kmap (Section 4.2). */
typedef struct spconv_layer_shape {
  int32_t c_in, c_out;
} spconv_layer_shape;

/* Group-based tuning (Section 4.2).  All n_layers layers run on `km`, so they share one map
 * structure and one dataflow: the tuner tries every structure of the design space (implicit GEMM
 * on the unsorted map or on 1..min(4, K^3) sorted splits; fetch-on-demand on the pair lists),
 * gives each layer the fastest kernel and tile shape for that structure, adds the time to build
 * every plan those choices need - paid once per group, not once per layer - and keeps the
 * structure with the lowest measured total.
 *   training = 0: forward only; fwd[n_layers] receives the configurations (dgrad, wgrad unused).
 *   training = 1: dgrad[n_layers] and wgrad[n_layers] are filled as well.  bind_fwd_dgrad = 1
 *     gives forward and dgrad the same structure (the paper's workload-pattern oriented binding:
 *     the two kernels have the same shape); 0 tunes them apart.  wgrad is always tuned apart, and
 *     with one value for the whole group: it walks weight-stationary pair lists whose only
 *     parameter is the number of pairs per work item (in this library the maps that dgrad and
 *     wgrad could share under the paper's sparse-mapping oriented binding are different objects).
 * group_us (may be NULL): the winning total in microseconds, every layer once, mapping included.
 * Blocking; allocates scratch tensors; leaves the winning plans to be rebuilt on first use. */
SPCONV_API int spconv_tune_group(spconv_kmap* km, const spconv_layer_shape* layers, int n_layers,
                                 spconv_dtype dtype, int training, int bind_fwd_dgrad, spconv_config* fwd,
                                 spconv_config* dgrad, spconv_config* wgrad, float* group_us, void* stream);

/* Element-wise glue between layers of a network (not part of the paper's method: activation,
 * residual add and their gradients), so that a whole network can run on this library's kernels.
 *   op 0: out = max(a, 0)            (b ignored, may be NULL)
 *   op 1: out = a + b
 *   op 2: out = max(a + b, 0)
 *   op 3: out = b > 0 ? a : 0        (gradient a through a ReLU whose output was b)
 * a, b, out: device, n elements of dtype; out may alias a or b. */
SPCONV_API int spconv_ew(int op, const void* a, const void* b, void* out, int64_t n, spconv_dtype dtype, void* stream);

/* dst[r][dst_off + c] = src[r][src_off + c] for r < rows, c < cols: channel concat / split of
 * row-major tensors with row lengths src_ld / dst_ld (elements). */
SPCONV_API int spconv_copy_cols(const void* src, int src_ld, int src_off, void* dst, int dst_ld, int dst_off, int cols,
                                int64_t rows, spconv_dtype dtype, void* stream);

/* Device allocations made by the library go through these callbacks when set
 * (so that a framework's caching allocator can back them); NULL, NULL restores
 * the library's own pool over hipMalloc.  alloc returns a device pointer aligned
 * to 256 bytes, or NULL when out of memory; both run on the calling host thread,
 * inside library calls.  `stream` is the hipStream_t (as void*) of the library
 * call in progress: the block is first used by work enqueued on that stream, and
 * a block is handed back while work of that stream may still be using it, so a
 * stream-ordered allocator must order its reuse behind that stream (exactly what
 * hipFreeAsync(ptr, stream), or a caching allocator keyed by stream, does).
 * spconv_kmap_destroy and spconv_kmap_drop_plans pass the stream of the last
 * call that used the kmap.  Switch allocators only while no kmap is alive: a block
 * goes back to whatever is installed when it is released. */
SPCONV_API int spconv_set_allocator(void* (*alloc)(size_t bytes, void* stream, void* user),
                         void (*free_)(void* ptr, void* stream, void* user), void* user);

/* What spconv_fwd / spconv_dgrad would launch for one side of a map: host arithmetic only (no GPU
 * is touched, none is needed), for tests and tools.  The library's run functions take every
 * launch dimension, LDS size and table size from the same functions that fill this structure.
 *   K        kernel size of the map (K^3 offsets)
 *   rows     rows of the side that is walked (outputs for forward, inputs for dgrad)
 *   rows_src rows of the tensor that is gathered from
 *   C_red    reduced channels (C_in for forward, C_out for dgrad), C_cols the produced ones
 *   dgrad    0 / 1 (the tiled kernel's LDS layout differs)
 * Returns SPCONV_EINVAL for every shape or configuration the compute calls refuse, SPCONV_OK with
 * an all-zero structure for rows = 0 (nothing is launched). */
typedef struct spconv_launch_info {
  int32_t kernel;         /* 1: weights resident in LDS, 16-row blocks; 2: workgroup tiles */
  int32_t parts;          /* max(1, n_split) */
  int32_t sorted;         /* n_split >= 1: rows are visited through a permutation */
  int32_t tile_m, tile_n; /* rows per block / tile, output channels per workgroup */
  int32_t k_steps;        /* kernel 1: 32-channel steps per offset; kernel 2: channels per LDS stage */
  int32_t waves, threads; /* per workgroup */
  int32_t grid[3];        /* kernel 1: workgroups per slice, column tiles, parts; kernel 2: tiles, column tiles, parts */
  int32_t xcd_ranges;     /* kernel 1: blocks are dealt to the XCDs as eight contiguous ranges */
  int32_t lo[4], width[4];      /* offset range of each part */
  int64_t lds_bytes;            /* dynamic LDS of the launch */
  int64_t slab_bytes, slab_map_bytes; /* kernel 1: per-wave LDS slab and its map part */
  int64_t rows_pad, n_tiles;    /* padded rows of the map; 16-row blocks (kernel 1) or tiles (kernel 2) */
  int64_t map_elems[4];         /* int32 elements of the table each part's kernel indexes */
} spconv_launch_info;
SPCONV_API int spconv_describe_launch(int K, int64_t rows, int64_t rows_src, int C_red, int C_cols,
                                      spconv_dtype dtype, const spconv_config* cfg_or_null, int dgrad,
                                      spconv_launch_info* out);

/* Measures, on the current device, what roofline reports quote beside the published peaks:
 * the rate of a plain streaming copy of 1 GiB (bytes read + bytes written per second, in GB/s:
 * what HBM delivers to a kernel with perfect access patterns) and the rate of back-to-back
 * 16x16x32 fp16 matrix instructions on every SIMD (dense TFLOP/s).  Either pointer may be NULL.
 * Blocking; allocates 2 GiB for the copy; takes about 10 ms. */
SPCONV_API int spconv_measure_peaks(double* hbm_copy_gbs, double* mfma_f16_tflops, void* stream);

SPCONV_API const char* spconv_strerror(int status);
/* Text of the last failing HIP call on this host thread ("" if none). */
SPCONV_API const char* spconv_last_hip_error(void);
/* Library version as major*10000 + minor*100 + patch. */
SPCONV_API int spconv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPCONV_H */
