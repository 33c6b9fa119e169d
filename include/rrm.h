/*
 * rrm.h - C ABI of the MI355X (gfx950) Recurrent Residual Module library.
 *
 * The library keeps, for one linear layer (convolution or fully connected) of a CNN that runs
 * on video, the previous frame's input I_{t-1} and projection P_{t-1} = W (*) I_{t-1} + b on
 * the device and advances them with the paper's delta update (Eq. 5; Algorithm 1, inner loop)
 *
 *      P_t = P_{t-1} + W (*) (I_t - I_{t-1}),
 *
 * doing work only where the input changed.  Everything is asynchronous on the HIP stream the
 * caller passes; no call in the per-frame path synchronises with the host or allocates.
 *
 * Layouts (all row-major, innermost index last)
 *   activations  x  [n][h][w][c_in]            (FC: [n][c_in])
 *   conv weights    [c_out][kh][kw][c_in/groups]   cross-correlation, no kernel flip
 *   FC weights      [c_out][c_in]
 *   outputs      y  [n][h_out][w_out][c_out]   (FC: [n][c_out])
 *   n is the number of independent video streams (chunks of a video processed in parallel,
 *   Sec. 3.2 last paragraph); each has its own snapshots, weights are shared.
 *
 * Element types (rrm_dtype)
 *   RRM_I8_I32    x, weights int8; bias, y int32.  Exact.  The difference of two inputs must
 *                 fit int8 (true whenever inputs are post-ReLU values in [0,127]); a violation
 *                 raises the sticky RRM_ERR_RANGE reported by rrm_get_stats.
 *   RRM_BF16_F32  x, weights bfloat16 (16-bit patterns); bias, y float32.  Inputs must be
 *                 finite.
 *   RRM_BIN_I32   x, weights are +1/-1 values bit-packed along the channel axis into 32-bit
 *                 words, LSB first, bit 1 = +1 (c_in must be a multiple of 32; x is
 *                 [n][h][w][c_in/32] words, weights [c_out][kh][kw][c_in/groups/32] words);
 *                 bias, y int32.  Exact.  Convolution only; taps outside the image contribute 0.
 *
 * Pointers: `weights` and `bias` given to rrm_layer_create may be host or device memory and are
 * copied (the caller may free them on return).  x / y arguments of rrm_step and rrm_dense are
 * DEVICE pointers, 16-byte aligned, borrowed until the work enqueued on `hip_stream` has run.
 * `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).
 *
 * Errors: every call returns an rrm_status (never throws, never aborts).  rrm_last_error()
 * gives a human-readable description of the last failure on the calling thread.
 *
 * Threading: one handle is used from one stream at a time; distinct handles are independent.
 */
#ifndef RRM_H
#define RRM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rrm_layer rrm_layer; /* opaque: device copies of W, b, snapshots, scratch */

typedef enum {
    RRM_OK = 0,
    RRM_ERR_NULL = -1,   /* a required pointer is NULL */
    RRM_ERR_SHAPE = -2,  /* shape not representable / not supported */
    RRM_ERR_DTYPE = -3,  /* unknown dtype, or dtype not valid for this kind */
    RRM_ERR_ALLOC = -4,  /* device or host allocation failed */
    RRM_ERR_HIP = -5,    /* a HIP runtime call failed */
    RRM_ERR_STATE = -6,  /* call not valid in the handle's current state */
    RRM_ERR_RANGE = -7,  /* an int8 difference did not fit int8 (sticky, see rrm_get_stats) */
    RRM_ERR_OPTION = -8, /* unknown option key or value */
    RRM_ERR_ALIGN = -9   /* a device pointer is not 16-byte aligned */
} rrm_status;

typedef enum { RRM_CONV = 0, RRM_FC = 1 } rrm_kind;
typedef enum { RRM_I8_I32 = 0, RRM_BF16_F32 = 1, RRM_BIN_I32 = 2 } rrm_dtype;

/* Layer description.  FC layers use n, c_in, c_out (h = w = kh = kw = stride = groups = 1,
 * pad = 0).  h_out = (h + 2*pad - kh)/stride + 1, likewise w_out. */
typedef struct {
    int kind; /* rrm_kind */
    int n, h, w, c_in, c_out, kh, kw, stride, pad, groups;
} rrm_shape;

/* Counters of a handle.  All are totals since creation or the last rrm_reset.  `steps` is counted by the host
 * when a call is enqueued (a captured graph that is replayed does not advance it); every other counter is kept
 * on the device by the kernels themselves and also advances under graph replay. */
typedef struct {
    uint64_t steps;           /* rrm_step calls enqueued by the host */
    uint64_t delta_steps;     /* steps executed on the sparse delta path */
    uint64_t changed_elems;   /* input elements (binary: bits) that differed from the snapshot */
    uint64_t changed_units;   /* 16-byte input units with any difference (FC: = changed_elems) */
    uint64_t active_tiles;    /* int8 / bf16 conv: output blocks recomputed (4x4 positions for the window-tile
                                 kernel, single positions for the position-gather kernel); binary conv: output
                                 positions updated (8x8 tiles where a layer's bands do not fit LDS); FC: columns
                                 streamed */
    uint64_t total_tiles;     /* the same unit, counted as a dense step would, summed over delta steps
                                 (FC: c_in per step) */
    int32_t range_error;      /* non-zero once an int8 difference overflowed */
    int32_t tile_positions;   /* output positions per tile of active_tiles / total_tiles: 16, 1, 64; FC: 0 */
    uint64_t truncated_elems; /* BF16 with a threshold: differences below it (neither applied nor committed) */
    double truncated_sumsq;   /* and the sum of their squares: sum over steps of l2(u)^2 of Eq. 7's truncated maps */
} rrm_stats;

/* Create a layer handle (Eq. 3 defines the layer; Sec. 3.2 the state it keeps).
 *   weights  layout and element type as above; host or device; copied and repacked.
 *   bias     c_out values (int32 or float32), host or device, may be NULL (= 0); copied.
 *   shape    validated; unsupported combinations give RRM_ERR_SHAPE.  A convolution keeps the input window of
 *            a 4 x 4 output sub-tile (3*stride + kh rows, 3*stride + kw columns, one 16-byte channel chunk or
 *            more) and that chunk's weights of every filter tap in on-chip memory.  Of the windows up to
 *            11 x 11 at strides up to 4, all fit except BF16 11 x 11 at stride 4 with 16 or more channels per
 *            group; a layer that does not fit is refused here, with a message.  BIN layers keep the window of
 *            an 8 x 8 output tile (7*stride + kh rows) twice: 152 KB bounds it.
 *   out      receives the handle.  The initial state is I_0 = 0 (Algorithm 1, first line) and
 *            P_0 = b, so the first rrm_step yields the dense result of its frame. */
rrm_status rrm_layer_create(const void* weights, const void* bias, const rrm_shape* shape, int dtype,
                            rrm_layer** out);

/* One (layer, frame) iteration of Algorithm 1: difference with the stored input, weights times
 * the non-zero part of the difference, sum into the stored projection, snapshot of the input.
 *   x_t    device, this frame's input for all n streams.
 *   y_out  device, may be NULL; when given it receives a full copy of P_t (n*h_out*w_out*c_out
 *          values).  Without it, read the projection through rrm_snapshot.
 * After the enqueued work has run: y_snap == b + W (*) x_t (exactly for I8/BIN; to fp32
 * accumulation accuracy for BF16) and x_snap == x_t bitwise. */
rrm_status rrm_step(rrm_layer* layer, const void* x_t, void* y_out, void* hip_stream);

/* The standard (dense) layer of Eq. 3: y = b + W (*) x.  Stateless: snapshots are untouched. */
rrm_status rrm_dense(rrm_layer* layer, const void* x, void* y, void* hip_stream);

/* rrm_dense for callers that cannot allocate device memory while they run (code under HIP-graph capture, tight
 * serving loops, harnesses that forbid it): FC layers only; the partial sums of the row splits, which rrm_dense
 * keeps in a buffer the handle allocated at create, live in a static device array of 4 MiB that exists once per
 * GPU.  The call allocates and frees nothing.  Same arguments and result as rrm_dense.  A layer whose partial
 * sums (n x row splits x c_out x 4 bytes) exceed the array gives RRM_ERR_SHAPE.  Every call on a GPU shares that
 * GPU's array: calls that overlap in time on one GPU (different streams, different handles) race.
 * Errors: RRM_ERR_NULL, RRM_ERR_ALIGN, RRM_ERR_SHAPE (not an FC layer, or too large), RRM_ERR_HIP. */
rrm_status rrm_dense_noalloc(rrm_layer* layer, const void* x, void* y, void* hip_stream);

/* Forget the stream history: I <- 0, P <- b, counters cleared (the "new precise inference"
 * of Sec. 3.4 starts from here: the next rrm_step recomputes its frame in full). */
rrm_status rrm_reset(rrm_layer* layer, void* hip_stream);

/* Borrowed device pointers to the stored input and projection (valid until destroy). */
rrm_status rrm_snapshot(rrm_layer* layer, const void** x_snap, const void** y_snap);

/* Copy the stored input and/or projection into caller-owned device buffers (either may be NULL),
 * enqueued on hip_stream: x_dst receives the bytes of x_snap (same format as x_t), y_dst the
 * n*h_out*w_out*c_out values of y_snap. */
rrm_status rrm_read_snapshot(rrm_layer* layer, void* x_dst, void* y_dst, void* hip_stream);

/* Options: how a step is carried out, never what it computes (every setting yields the P_t of Eq. 5 / Algorithm 1,
 * within the layer's tolerance).  Value semantics per key:
 *   "path"        0 auto, 1 sparse delta path always (scan + tile kernel, no switch to recomputation), 2 recompute
 *                 densely every step, 3 INT8 / BF16 conv: the single-launch scatter path always (one kernel compares,
 *                 multiplies the changed input positions and adds the products into the stored projection with
 *                 atomic adds: work proportional to the changed input positions; fp32 results then depend on the
 *                 order of the adds within the layer's tolerance).  Automatic mode takes path 3 for layers with few
 *                 positions in all (one stream of a small map), where two dependent launches cost more than the work.
 *   "fc_splits"   FC, dense path: number of row splits of the weight matrix, in [1, the default chosen at
 *                 create] (the partial-sum scratch is sized for the default)
 *   "fc_batched"  FC with 16 to 4096 streams (c_out a multiple of 16, rows of whole 64-byte steps): 1 (default) =
 *                 dense layer and step run as one product on the matrix cores with W read once for all streams:
 *                 an I8 step multiplies the difference of all streams (one pass over W whatever the density), a
 *                 BF16 step commits x_t and recomputes b + W x_t (its difference would need two bf16 terms, two
 *                 products); 0 = one column walk per stream as at batch 1.  Layers with a truncation threshold
 *                 or "fc_sparse_weights" take the walk.
 *   "fc_sparse_weights"  FC, delta step: 1 = walk the non-zero weights of the changed columns only (pruned
 *                 models, Sec. 4.3; the (row, value) lists exist when at most half of W is non-zero at create,
 *                 else RRM_ERR_OPTION), 0 = walk whole columns (default).  fp32 sums of the sparse walk
 *                 depend on the order of its atomic adds, within the layer's tolerance; integers are exact.
 *   "bf16_terms"  BF16 conv: 2 = difference carried as hi+lo bf16 pair (default), 1 = hi only
 *   "dense_switch_pct"  INT8 / BF16 conv: a delta step whose changes touch more than this percentage of the
 *                 4x4 output blocks recomputes the whole projection (same result; cheaper than reading and
 *                 re-writing most of it); 1..100, 100 = never; defaults 75 (int8) / 40 (bf16) for the window-tile
 *                 kernel, which decides per launch, and 90 / 50 for the position-gather kernel, which decides per
 *                 work unit
 *   "conv_kernel" INT8 / BF16 conv: 0 = automatic (the window-tile kernel), 1 = window-tile kernel (4x4 output
 *                 blocks with their input windows gathered into LDS; any stride), 2 = position-gather kernel
 *                 (single active output positions as columns of the product; stride 1 and channel runs of
 *                 16-byte multiples; faster where every stream changes sparsely and alike).  Set it before the
 *                 first rrm_step, or follow it with rrm_reset: the two kernels keep their change flags differently.
 *   "bin_single_launch"  binary conv, delta step: 1 (default) = the whole step in one launch where the layer allows
 *                 it (compare, popcount products of the changed positions and commit in the band kernel), 0 = a
 *                 difference kernel followed by the band kernel.  Change it only right after create or rrm_reset
 *                 (the two forms keep the flip buffer differently).
 *   "bin_cout_per_wave"  binary conv: output channels per wavefront, 8 / 16 (0 = heuristic)
 *   "profile"     1 = bracket every kernel of the following rrm_step calls with HIP events on the
 *                 caller's stream (see rrm_get_kernel_times; not for use under graph capture), 0 = off */
rrm_status rrm_set_option(rrm_layer* layer, const char* key, long value);

/* Read the counters: how many inputs changed and how much of the projection a step touched, the measured
 * counterpart of the density rho in the cost model of Sec. 3.3 (Table 1, Eq. 6), and the truncated differences
 * of Sec. 3.4 (Eq. 7).  Synchronises with the device (copies a small block back); call it after
 * the stream has been synchronised, outside timed regions.  Returns RRM_ERR_RANGE (with *out
 * filled) if the sticky range flag is set. */
rrm_status rrm_get_stats(rrm_layer* layer, rrm_stats* out);

/* rrm_step for a layer whose input is f(P) of the layer before it, without materialising that input
 * (Algorithm 1: the non-linear map f is applied to the projection and the result is the next layer's
 * input I).  f is the benchmark's int8 map of rrm_aux_relu_requant_pool_i8: ReLU, arithmetic right shift, clamp
 * to 127, optional 3x3 / stride-2 max pooling.  Equivalent to rrm_step(layer, f(producer's y_snap), ...), but
 * an input entry is computed and compared only under the 4x4 blocks of the projection that the producer's last
 * step wrote: elsewhere neither P nor f(P) changed.  Both layers INT8 convolutions with equal n, layer's c_in ==
 * producer's c_out (a multiple of 16), layer's (h, w) == the mapped size of the producer's (h_out, w_out).
 * Call it once after every step of the producer, on the same stream, and feed `layer` through this call
 * only (its stored input must be the mapped projection of the producer's previous step; a freshly created or
 * reset `layer` compares everything).  Not available with "path" = 2.
 * Errors: RRM_ERR_NULL, RRM_ERR_DTYPE, RRM_ERR_SHAPE, RRM_ERR_STATE, RRM_ERR_ALIGN, RRM_ERR_HIP. */
rrm_status rrm_step_from_projection(rrm_layer* layer, rrm_layer* producer, int shift, int pool, void* y_out,
                                    void* hip_stream);

/* One frame through a stack of INT8 convolution layers: Algorithm 1's inner loop over the layers, with the
 * non-linear map f between them (ReLU, right shift, clamp to 127, optional 3x3 / 2 max pooling; see
 * rrm_step_from_projection) fused into the next layer's difference kernel, so that no layer input but the frame is
 * ever written to memory:
 *     layer 0                      rrm_step(entries[0].layer, x_t)
 *     layer i > 0                  rrm_step_from_projection(entries[i].layer, entries[i-1].layer,
 *                                                           entries[i-1].shift, entries[i-1].pool)
 *     f_out (may be NULL)          f of the last layer's stored projection, recomputed only where its last step
 *                                  wrote (rrm_aux_relu_requant_pool_changed_i8 with entries[n-1].shift / .pool);
 *                                  device, int8, must hold the previous call's result
 * The shape conditions are those of the calls above.  Everything is enqueued on hip_stream; nothing synchronises.
 * Errors: RRM_ERR_NULL, or the first error of a constituent call. */
typedef struct {
    rrm_layer* layer;
    int shift; /* right shift of f applied to this layer's projection */
    int pool;  /* non-zero: 3x3 / stride-2 max pooling in f */
} rrm_stack_entry;
rrm_status rrm_stack_step(const rrm_stack_entry* entries, int n_layers, const void* x_t, void* f_out, void* hip_stream);

/* Truncation threshold of a BF16 layer (Sec. 3.4, "Improving sparsity": small values of the difference are
 * truncated to zero to gain sparsity; the experiments use 1e-2).  An entry with |x_t - x_snap| < epsilon
 * (difference formed in fp32) is not applied to the stored projection and not committed to the stored input,
 * so y_snap == b + W (*) x_snap stays true and the entry is still pending at the next frame; x_snap then
 * differs from x_t by less than epsilon per entry.  epsilon = 0 (the default) is the exact method.  Takes
 * effect at the next rrm_step; steps with "path" = 2 ignore it.
 * Errors: RRM_ERR_NULL, RRM_ERR_DTYPE (not BF16), RRM_ERR_OPTION (negative or not finite). */
rrm_status rrm_set_threshold(rrm_layer* layer, float epsilon);

/* Kernel times of the rrm_step calls made since "profile" was switched on (or since the last call
 * of this function): sums, in microseconds, of the event-bracketed durations of the scan kernel
 * (delta + change map) and of the compute kernel (tile conv / column scatter / popcount conv), and
 * the number of steps summed.  Synchronises with the recorded events.  At most 1024 steps are kept. */
rrm_status rrm_get_kernel_times(rrm_layer* layer, double* scan_us, double* compute_us, int* steps);

void rrm_layer_destroy(rrm_layer* layer);

const char* rrm_status_string(int status);
const char* rrm_last_error(void);

/* Harness helper, NOT part of the paper's linear-layer path: the nonlinear map f that the int8
 * conv-stack benchmark places between layers.  out = maxpool3x3/2( min(127, max(0, y) >> shift) )
 * (pooling only if pool != 0), y NHWC int32 -> out NHWC int8, both device pointers. */
rrm_status rrm_aux_relu_requant_pool_i8(const void* y, void* out, int n, int h, int w, int c, int shift,
                                        int pool, void* hip_stream);

/* The same map applied to the stored projection of an int8 convolution layer (c_out a multiple of 4),
 * recomputing only the outputs whose window touches a 4x4 block of output positions that the layer's last
 * rrm_step wrote (Algorithm 1 applies f to all of P; where P did not change, f(P) did not either).  `out`
 * ([n][ho'][wo'][c_out] int8, 4-byte aligned, device, caller-owned) must hold the result of the previous call
 * for this layer: entries that are not recomputed keep it.  Call it once after every rrm_step, on the same
 * stream; after rrm_layer_create, rrm_reset or a dense step everything is recomputed.
 * Errors: RRM_ERR_NULL, RRM_ERR_SHAPE (not an int8 conv layer, c_out % 4 != 0, bad shift / pool),
 * RRM_ERR_ALIGN, RRM_ERR_HIP. */
rrm_status rrm_aux_relu_requant_pool_changed_i8(rrm_layer* layer, void* out, int shift, int pool, void* hip_stream);

/* Measurement probes for the benchmark, NOT part of the method: what the device sustains, to price the
 * library's kernels against measured as well as published peaks.
 * rrm_aux_probe_mfma: `workgroups` workgroups of four wavefronts, each wavefront issuing 4 * iters
 *   matrix-core products of register-resident operands (dtype RRM_I8_I32: 32x32x32 int8 tiles, 65536
 *   operations each; RRM_BF16_F32: 32x32x16 bf16 tiles, 32768 each).  `sink` is a device word that the
 *   kernel practically never writes.  1 <= iters <= 1 << 20, 1 <= workgroups <= 1 << 16.
 * rrm_aux_probe_copy: copies bytes / 16 sixteen-byte vectors from src to dst (device pointers, 16-byte
 *   aligned, not overlapping): `bytes` read and `bytes` written.
 * Errors: RRM_ERR_NULL, RRM_ERR_DTYPE, RRM_ERR_SHAPE (counts out of range), RRM_ERR_ALIGN, RRM_ERR_HIP. */
rrm_status rrm_aux_probe_mfma(int dtype, void* sink, int iters, int workgroups, void* hip_stream);
rrm_status rrm_aux_probe_copy(void* dst, const void* src, size_t bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* RRM_H */
