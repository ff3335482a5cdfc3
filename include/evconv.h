/* evconv.h - C ABI of the MI355X (gfx950) incremental-CNN library.
 *
 * Incremental CNN inference on event-camera inputs: each step runs the network on the sparse
 * increment x_inc(n) = x(n) - x(n-1) (Eq.1) only where it is nonzero, adds the result into
 * cached per-layer pre-activations (the x_acc of Eq.12-14) and returns the output together
 * with its increment (Eq.2).  Every step of that path runs in HIP kernels of this library;
 * the caller supplies device memory (one workspace) and a HIP stream, nothing else.
 *
 * Plain C: no C++ types, no exceptions cross this boundary.  Pointers are marked HOST or
 * DEVICE.  One handle must be used from one host thread at a time.
 *
 * Mask tile: the paper's mask marks h x w sections of a tensor that are entirely zero
 * ("Implementation of Increment Layers"; 6 x 6 in "Comparison to prior works") and a mask may only
 * skip zeros, so no value depends on the section size.  This library fixes it at 8 x 8 sites over
 * all channels: 64 sites are one gfx950 wavefront, so one ballot instruction yields a tile's 64-bit
 * occupancy word, and every kernel's mask arithmetic is written on such words.  The section size is
 * therefore not a parameter of the description.
 *
 * Data layout: public tensors are C x H x W fp32 (row-major, W fastest).  Site index means
 * y*W + x.  Inside the workspace activations are H x W x C ("channels last", the notation of
 * "Implementation of Increment Layers"); evconv_get_state returns that internal layout.
 *
 * Semantics of one node (input increment x_inc on active set S_in -> output increment y_inc on
 * active set S_out); T is the touched set, the input mask pushed through the op's footprint:
 *   CONV2D / LINEAR  y_lin = theta_L(x_inc) at T (Eq.10), no bias (bias enters in reset only).
 *                    T = outputs with at least one tap on an active, in-bounds input site.
 *   ADD              y_lin = a_inc + b_inc, T = S_a | S_b (Eq.11).
 *   CONCAT           channel concatenation, T = S_a | S_b.
 *   UPSAMPLE_BILINEAR2X  half-pixel centres, weights {0.25, 0.75}, clamped borders; T = outputs
 *                    with an active source site.  Linear, so Eq.10 applies.
 *   ACT              y_lin = x_inc, T = S_in (the activation increment layer, Eq.12-14).
 *   GLOBAL_AVGPOOL   y_lin = mean over sites of x_inc (1 x 1 x C), T = {0} if S_in nonempty.
 *   SPARSIFY         the sparsification layer with error feedback (Eq.3-8): residual delta (kept
 *                    as this node's accumulated tensor, zero after reset), x_corr = delta + x_inc,
 *                    y_inc = k * floor(0.5 + x_corr / k), delta = x_corr - y_inc, at the elements
 *                    of S_in whose x_inc is nonzero (the others emit 0 and keep delta: the same
 *                    formulas give that for |delta| <= k/2, so no value depends on the mask); S_out =
 *                    sites with a nonzero y_inc.  k = sparsify_tp * RMS(node input at the last
 *                    reset), kept to 8 fraction bits, or the fp32 value at weight_off when
 *                    weight_off >= 0; k == 0 is the identity.  In reset and in dense-recompute
 *                    mode the node is the identity.  Lossy: y no longer equals the forward pass.
 *   MUL              elementwise product of two nodes of equal shape (Eq.15-17): keeps the
 *                    accumulated values of both factors (states Z and Z2); y_inc = (x1acc + x1_inc)
 *                    * x2_inc + x2acc * x1_inc with the accumulators of the previous step, each
 *                    operation rounded once (no fused multiply-add); then both accumulators
 *                    advance (Eq.17).  T = S_out = S_a | S_b (Eq.16).  act must be NONE.
 *   DELAY            recurrent state (the paper's evaluation networks are recurrent; how the state
 *                    is carried is this library's reading): the value of a LATER node X at the
 *                    previous step.  in0 = X (in0 > this node's index), in1 = an earlier node or
 *                    -1 that has X's height and width, c_out = X's channels; act must be NONE.
 *                    y_inc(n) = X's y_inc(n-1) and T = S_out = X's S_out(n-1); the state before
 *                    the first frame is zero, so the first step after a reset emits X's whole
 *                    value at every site.  State Z = the value emitted so far.  A regular forward
 *                    pass in mid-stream (refresh, dense-recompute mode) keeps the state: the node
 *                    then holds X's value of the previous step; the step after it emits
 *                    X's value minus Z at every site.
 *   MAXPOOL          state a += x_inc; y_inc = max(window of a_new) - max(window of a_old) at
 *                    windows containing an active site; padding value -inf; act must be NONE.
 * A node keeps an accumulated tensor z (+= y_lin at T) if it is CONV2D, LINEAR,
 * GLOBAL_AVGPOOL, ACT, or has an activation.  With an activation theta_a the output is
 * y_inc = theta_a(z_new) - theta_a(z_old) (Eq.12), else y_inc = y_lin.
 * S_out is T for ADD / CONCAT / UPSAMPLE / GLOBAL_AVGPOOL / MUL / DELAY without activation (Eq.11b), otherwise
 * the sites of T where some channel of y_inc is != 0 (-0 counts as zero, NaN as nonzero).
 * Output nodes additionally keep y += y_inc on S_out (Eq.2).
 */
#ifndef EVCONV_H
#define EVCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EVCONV_ABI_VERSION 2

typedef struct evconv_net evconv_net; /* opaque, library-owned; freed by evconv_destroy */

typedef enum {
  EVCONV_OK = 0,
  EVCONV_ERR_INVALID_ARG = 1, /* null pointer, bad enum value */
  EVCONV_ERR_BAD_DESC = 2,    /* graph not topologically ordered, bad offsets, abi mismatch */
  EVCONV_ERR_SHAPE = 3,       /* channel / spatial sizes of a node's inputs do not fit */
  EVCONV_ERR_STATE = 4,       /* step before reset */
  EVCONV_ERR_WORKSPACE = 5,   /* workspace too small or misaligned (256 bytes) */
  EVCONV_ERR_HIP = 6,         /* a HIP call failed; text in evconv_last_error */
  EVCONV_ERR_UNSUPPORTED = 7  /* valid request this build does not implement */
} evconv_status;

typedef enum {
  EVCONV_OP_CONV2D = 0,
  EVCONV_OP_ADD = 1,
  EVCONV_OP_CONCAT = 2,
  EVCONV_OP_UPSAMPLE_BILINEAR2X = 3,
  EVCONV_OP_MAXPOOL = 4,
  EVCONV_OP_GLOBAL_AVGPOOL = 5,
  EVCONV_OP_LINEAR = 6,
  EVCONV_OP_ACT = 7,
  EVCONV_OP_SPARSIFY = 8,
  EVCONV_OP_MUL = 9,
  EVCONV_OP_DELAY = 10
} evconv_op;

/* ONE_MINUS: theta(z) = 1 - z (the "1 - update gate" of a gated recurrent unit); as every
 * activation it acts on the accumulated tensor, so its increment is -x_inc. */
typedef enum {
  EVCONV_ACT_NONE = 0, EVCONV_ACT_RELU = 1, EVCONV_ACT_SIGMOID = 2, EVCONV_ACT_TANH = 3, EVCONV_ACT_ONE_MINUS = 4
} evconv_act;

/* dtype of the weights and of the increments inside the channel contraction; accumulation and
 * every cached tensor are always fp32.
 *   EVCONV_F32        fp32 operands on the fp32 matrix-core (or vector) path.
 *   EVCONV_BF16       weights rounded to bf16 at create, increments rounded to bf16 inside the
 *                     contraction: relative error of a product about 2^-8.
 *   EVCONV_F32_SPLIT  fp32 weights and increments, each written as bf16 high part + bf16 low part
 *                     (16 significant bits together); a product is lo*hi + hi*lo + hi*hi on the bf16
 *                     matrix cores with fp32 accumulation: relative error of a product about 2^-16.
 *                     Meets the fp32 parity bar of this library's tests at several times the speed
 *                     of EVCONV_F32; layers the matrix-core kernel does not take run as EVCONV_F32. */
typedef enum { EVCONV_F32 = 0, EVCONV_BF16 = 1, EVCONV_F32_SPLIT = 2 } evconv_dtype;

typedef enum {
  EVCONV_MODE_INCREMENTAL = 0,     /* the paper's method */
  EVCONV_MODE_DENSE_RECOMPUTE = 1, /* regular forward pass of x(n) with the same kernels (the
                                      refresh of "Drift Errors", used as the dense comparator) */
  EVCONV_MODE_AUTO = 2             /* whichever of the two is faster on the current stream; see
                                      evconv_set_mode */
} evconv_mode;

/* evconv_net_desc.flags: planner switches for tests and comparisons (0 = everything on). */
#define EVCONV_FLAG_NO_FUSION 1u  /* no node is computed by another node's kernel */
#define EVCONV_FLAG_NO_FOLD 2u    /* an up-sampling is never folded into the consuming conv's weights */
#define EVCONV_FLAG_FORCE_VALU 4u /* no matrix-core kernels */

/* One node.  Inputs are earlier node ids; -1 is the network input; in1 is ignored by one-input
 * ops.  The activation is fused after the op. */
typedef struct {
  int32_t op;          /* evconv_op */
  int32_t act;         /* evconv_act */
  int32_t in0, in1;
  int32_t c_in, c_out; /* CONV2D / LINEAR; other ops derive their channels */
  int32_t kh, kw;      /* CONV2D, MAXPOOL; must be equal, 1..7 */
  int32_t stride;      /* 1 or 2 */
  int32_t pad;         /* zero padding (-inf for MAXPOOL), < kh */
  int32_t wdtype;      /* evconv_dtype */
  int32_t is_output;   /* nonzero: y and y_inc of this node are returned by reset / step */
  int64_t weight_off;  /* byte offset into `weights`: fp32 [c_out][c_in][kh][kw]; -1 if none */
  int64_t bias_off;    /* byte offset of fp32 [c_out]; -1 = no bias */
} evconv_node_desc;

typedef struct {
  int32_t abi_version; /* EVCONV_ABI_VERSION */
  int32_t n_nodes;
  const evconv_node_desc* nodes; /* HOST, n_nodes entries, topological order */
  int32_t in_c, in_h, in_w;
  uint32_t flags;         /* EVCONV_FLAG_* */
  float sparsify_tp;      /* threshold parameter t_p of the SPARSIFY nodes (>= 0; 0 = lossless) */
  int32_t n_streams;      /* independent event streams (cameras) stepped together and sharing the
                           * weights, 1..256 (0 = 1).  Every stream owns a copy of the whole state;
                           * inputs are contiguous [n_streams][C][H][W]; the pointers in evconv_out
                           * are stream 0's, stream s lies s * evconv_stream_stride bytes further. */
} evconv_net_desc;

/* Result of one output node.  All pointers are DEVICE memory inside the workspace, valid until
 * the next reset / step / destroy on the same net, and written asynchronously on the net's
 * stream: synchronise the stream before reading them. */
typedef struct {
  int32_t node, c, h, w;
  const float* y;          /* C x H x W: y(n), the running sum of Eq.2 */
  const float* dy;         /* C x H x W: y_inc(n), zero outside the active set */
  const int32_t* dy_idx;   /* ascending active output sites (h*w entries allocated) */
  const int32_t* dy_count; /* one int32: number of valid entries of dy_idx */
} evconv_out;

typedef struct {
  int32_t n_sites, n_tiles;      /* of the node's output grid */
  int32_t n_touched, n_active;   /* sites in T and in S_out after the last step */
  int32_t n_touched_tiles;       /* tiles with at least one touched site */
  double flops_executed;         /* 2 * k*k*c_in*c_out * 64 * n_touched_tiles */
  double flops_dense;            /* 2 * k*k*c_in*c_out * n_sites */
} evconv_layer_stats;

typedef enum {
  EVCONV_STATE_Z = 0,           /* fp32 H x W x C accumulated tensor (nodes that keep one) */
  EVCONV_STATE_DY = 1,          /* fp32 H x W x C increment buffer; meaningful on T only */
  EVCONV_STATE_IDX = 2,         /* int32 ascending site list of S_out */
  EVCONV_STATE_COUNT = 3,       /* int32 */
  EVCONV_STATE_BITMAP = 4,      /* uint64 words, bit t%64 of word t/64 = tile t non-empty */
  EVCONV_STATE_OCC = 5,         /* uint64 per tile: S_out, bit (y%8)*8 + x%8, tiles row-major */
  EVCONV_STATE_OCC_TOUCHED = 6, /* uint64 per tile: T */
  EVCONV_STATE_X_PREV = 7,      /* node -1 only: fp32 C x H x W cached previous frame */
  EVCONV_STATE_STEP = 8,        /* SPARSIFY nodes: one fp32, the rounding step k */
  EVCONV_STATE_Z2 = 9           /* MUL nodes: fp32 H x W x C accumulated second factor (Z: the first) */
} evconv_state_kind;

/* Bytes of device workspace a net of this description needs.  No GPU work.  The workspace holds
 * the state that "Implementation of Increment Layers" asks an increment layer to keep between
 * inferences - the accumulated input x_acc of every nonlinear operator (Eq.12-14; both factors
 * for a product, Eq.15-17; the residual delta of a sparsification layer, Eq.4-8), the previous
 * input x(n-1) of Eq.1, the output sum of Eq.2 - plus, per node, the increment tensor, its masks
 * (per-tile occupancy words of the active and of the touched set), the ascending site list and
 * the re-laid weights. */
evconv_status evconv_query_workspace(const evconv_net_desc* desc, size_t* bytes);

/* Builds a net: one increment layer beside every forward layer of the description ("Increment
 * tensors and increment layers").  `weights` is HOST memory (copied and re-laid out; the caller may free it on
 * return).  `workspace` is DEVICE memory, 256-byte aligned, at least the queried size, owned by
 * the caller and used exclusively by this net until evconv_destroy.  `hip_stream` is a
 * hipStream_t (NULL = the default stream); all later work of this net is enqueued on it.
 * Synchronous.  On error *out is untouched. */
evconv_status evconv_create(const evconv_net_desc* desc, const void* weights, size_t weight_bytes,
                            void* workspace, size_t workspace_bytes, void* hip_stream,
                            evconv_net** out);

/* For callers that cannot allocate device memory (code under HIP graph capture set-up, tight
 * serving loops, harnesses that forbid hipMalloc): evconv_create with the workspace taken from an
 * array that is part of the library's code object, EVCONV_STATIC_WORKSPACE_BYTES per GPU, held
 * from the library's load to the end of the process.  Neither this call nor any later call on
 * the net allocates or frees device memory.  The net is built on the current device.
 * EVCONV_ERR_WORKSPACE if the description needs more than the array holds (the text of
 * evconv_last_error(NULL) gives both sizes); EVCONV_ERR_STATE while another net created by this
 * call on the same device has not been destroyed: the array is one per GPU, two nets in it
 * would overwrite each other.  The array keeps the previous net's contents; the part a new net
 * uses is cleared by this call.  The pointers in evconv_out point into the array.  Otherwise as
 * evconv_create. */
#define EVCONV_STATIC_WORKSPACE_BYTES (32u << 20)
evconv_status evconv_create_static(const evconv_net_desc* desc, const void* weights, size_t weight_bytes,
                                   void* hip_stream, evconv_net** out);

/* Number of output nodes (entries written to the `out` arrays below). */
int32_t evconv_num_outputs(const evconv_net* net);

/* In the three calls below the input tensor holds one C x H x W fp32 frame (or increment) per
 * stream, contiguous [n_streams][C][H][W]; all streams advance together.
 *
 * Reset: regular forward pass of x0 (DEVICE, C x H x W fp32) that fills the previous-frame
 * cache, every accumulated tensor and y(0), from a zero recurrent state (DELAY nodes).  `out`
 * (HOST array of evconv_num_outputs entries, may be NULL) receives the pointers; dy is zero,
 * count 0.  Asynchronous on the net's stream.  For a net without DELAY nodes this is also the
 * refresh of the "Drift Errors" section; a recurrent net is refreshed through
 * evconv_set_refresh_period, which keeps the state. */
evconv_status evconv_reset(evconv_net* net, const float* x0, evconv_out* out);

/* One inference step with increment layers ("Increment tensors and increment layers") on a
 * caller-supplied increment tensor x_inc(n) (DEVICE, dense C x H x W fp32, zeros where nothing
 * changed): the mask of the input is formed, then every
 * node runs its increment operator in topological order - linear operators on the increment alone
 * at the touched sites (Eq.9-10, "Convolution on Sparse Inputs"), additions with OR-ed masks
 * (Eq.11), activations through their accumulated input (Eq.12-14), products (Eq.15-17),
 * sparsification layers (Eq.3-8) - and the outputs are summed, y(n) = y(n-1) + y_inc(n) (Eq.2).
 * `out` as in evconv_reset, with dy / dy_idx / dy_count describing y_inc(n).
 * Asynchronous.  EVCONV_ERR_STATE before the first reset.
 *
 * A step only enqueues kernels (no allocation, no synchronisation, no memset), so the caller may
 * capture it into a HIP graph and replay that.  What a replay cannot see is host-side state:
 * the refresh period counts calls, not replays, and a net with DELAY nodes passes "the previous
 * pass was a regular forward pass" to its kernels as an argument.  Capture such a net's step
 * after an incremental step (not directly after evconv_reset), and run refreshes outside the
 * graph, followed by one un-captured step. */
evconv_status evconv_step(evconv_net* net, const float* increment, evconv_out* out);

/* One incremental step on the next frame x(n) (DEVICE, C x H x W fp32): the increment is
 * formed against the cached previous frame with one fp32 subtraction per element (Eq.1). */
evconv_status evconv_step_frame(evconv_net* net, const float* x_t, evconv_out* out);

/* NULL is accepted.  Never frees the workspace.  Synchronises the net's stream first. */
evconv_status evconv_destroy(evconv_net* net);

/* INCREMENTAL (default): every step is the paper's incremental inference.  DENSE_RECOMPUTE: every
 * step is a regular forward pass of x(n) through the same kernels (all sites, accumulated tensors
 * overwritten); y is the forward pass value, dy = y(n) - y(n-1) at every site.  Both leave the
 * same state up to fp32 rounding (Eq.2), so the mode may be changed between any two steps.
 * AUTO: the library times a few consecutive steps in each of the two modes with HIP events on the
 * net's stream (without synchronising: the result is picked up by a later call, once the events
 * have completed), runs the faster one for the next 256 steps, then measures again.  Incremental
 * inference only pays while the increments stay sparse through the layers ("Mitigating Reduced
 * Sparsity on Upsampling"; a recurrent state densifies everything behind it), and where that
 * ends depends on the stream, not on the description.  The choice depends on measured time, so
 * AUTO is not run-to-run bit-reproducible (results agree within fp32 rounding).  A net with
 * active SPARSIFY nodes (sparsify_tp > 0 or a fixed step) stays incremental in AUTO mode, because
 * a regular pass does not sparsify; so does a step that is being captured into a HIP graph.
 * EVCONV_ERR_INVALID_ARG for another value. */
evconv_status evconv_set_mode(evconv_net* net, int32_t mode /* evconv_mode */);

/* The mode the next step would run in (AUTO resolves to INCREMENTAL or DENSE_RECOMPUTE). */
int32_t evconv_current_mode(const evconv_net* net);

/* Refresh policy of "Drift Errors": with period N > 0 every N-th call of evconv_step /
 * evconv_step_frame after a reset runs as a regular forward pass of x(n) that re-initialises
 * every accumulated tensor (for a supplied increment, x(n) = cached frame + increment), which
 * removes the rounding drift of the fp32 running sums (and the sparsification residuals).  The
 * internal increments and lists of such a step are empty; y is the forward pass value and
 * dy = y(n) - y(n-1) at every site, listed in dy_idx, so that Eq.2 also holds across a refresh for
 * a consumer that sums the returned increments.  0 (the default) never refreshes; the count restarts at every reset and at every call of this
 * function.  EVCONV_ERR_INVALID_ARG for a negative period. */
evconv_status evconv_set_refresh_period(evconv_net* net, int32_t period);

/* Shape (c, h, w) of a node's output; node -1 is the network input. */
evconv_status evconv_node_shape(const evconv_net* net, int32_t node, int32_t* chw /* HOST[3] */);

/* Synchronous copy of internal state to HOST memory (parity checks, checkpoints): the tensors
 * an increment layer is defined by in "Implementation of Increment Layers" - its increment, its
 * mask (as occupancy words, list, count, tile bitmap) and its accumulated input x_acc (Eq.14;
 * Eq.17 for a product; the residual of Eq.8 for a sparsification layer).  `bytes` must be the
 * exact size; node -1 addresses the input increment stage (Eq.1). */
evconv_status evconv_get_state(evconv_net* net, int32_t node, int32_t kind, void* dst, size_t bytes);

/* The same for stream `stream` of a net created with n_streams > 1 (evconv_get_state reads
 * stream 0).  EVCONV_ERR_INVALID_ARG for a stream outside [0, n_streams). */
evconv_status evconv_get_state_stream(evconv_net* net, int32_t stream, int32_t node, int32_t kind, void* dst,
                                      size_t bytes);

/* Bytes between the copies of any state or output pointer of consecutive streams, and the number
 * of streams (n_streams may be NULL).  The workspace holds n_streams such copies back to back. */
evconv_status evconv_stream_stride(const evconv_net* net, size_t* bytes /* HOST */, int32_t* n_streams /* HOST */);

/* Sparsity and work of a node in the last step (stream 0): sizes of its touched and active sets
 * (the per-layer sparsity of the "Sparsification layer" section's figure) and, for CONV2D / LINEAR,
 * the floating-point operations of the step against those of a regular forward pass - the
 * "MFLOPs" columns of the paper's result tables under this counting rule: 2 * k * k * c_in * c_out
 * per output site, a mask tile with at least one touched site counted in full (64 sites), padding
 * taps included on both sides.  Synchronous. */
evconv_status evconv_get_stats(evconv_net* net, int32_t node, evconv_layer_stats* out);

/* Per-node kernel timing with HIP events recorded on the net's stream around each node's
 * launches.  profile_begin allocates `max_records` event pairs and arms recording for the
 * following reset / step calls (recording stops silently when the pairs run out);
 * profile_end synchronises the stream and accumulates the elapsed times; get_node_time returns
 * the accumulated milliseconds and number of timed launches of a node since profile_begin; node -1
 * is the increment builder (Eq.1 and the input mask), node n_nodes the compaction of all masks
 * into site lists at the end of a step. */
evconv_status evconv_profile_begin(evconv_net* net, int32_t max_records);
evconv_status evconv_profile_end(evconv_net* net);
evconv_status evconv_get_node_time(const evconv_net* net, int32_t node, double* ms_total /* HOST */,
                                   int64_t* launches /* HOST */);

/* Measurement aid, not part of the method: where the time of a matrix-core convolution workgroup
 * goes ("Convolution on Sparse Inputs": mask test, conditioned fetch, contraction, write-back are
 * the phases of the paper's kernel as well).  In a library built with -DEVCONV_PHASE_STAMPS
 * (python -m paper_2303_04670_amd.build --phase-stamps; the regular build has none of this and
 * returns EVCONV_ERR_UNSUPPORTED) one lane of every such workgroup writes a 100 MHz wall-clock stamp
 * at each phase boundary.  Copies the records of the kernels of one operand mode (evconv_dtype)
 * written since the last reset to out (HOST, max_records records of 32 x uint64; field meanings:
 * PhaseField in csrc/conv_mfma_impl.h), stores the number written in n_records (it may exceed
 * max_records and the 32768 the library keeps) and, if reset != 0, starts a new collection.
 * Synchronises the device. */
evconv_status evconv_debug_phase_stamps(int32_t operand_mode, uint64_t* out /* HOST */, int32_t max_records,
                                        int32_t reset, int32_t* n_records /* HOST */);

/* Measurement aid, not part of the method: small timing probes of the properties of the chip that
 * the matrix-core kernels are designed around ("Convolution on Sparse Inputs" leaves the kernel
 * design to the hardware at hand).  Runs on hip_stream in `scratch` (DEVICE, at least
 * EVCONV_CHIP_PROBE_SCRATCH_BYTES, overwritten) and writes EVCONV_CHIP_PROBE_VALUES floats to out
 * (HOST):
 *   [0..3]   cycles per iteration (at 2.4 GHz) of one wave per SIMD issuing one fp32 MFMA plus 0, 4,
 *            16, 32 independent vector instructions
 *   [4..7]   us, one wave each on every SIMD: vector loop alone, fp32 MFMA chain alone, the loop
 *            beside the chain, the chain beside the loop
 *   [8..10]  us: bf16 MFMA chain alone, the vector loop beside it, the chain beside the loop
 *   [11..14] us: a chain of dependent global loads alone / beside three fp32 MFMA chain waves per
 *            SIMD; a chain of dependent LDS reads alone / beside them
 *   [15..16] ns per LDS atomic instruction whose 64 lanes hit one word / 64 different words
 *   [17..19] us: a loop of 16-byte LDS reads alone / beside another wave's one-word atomics /
 *            beside its 64-word atomics
 *   [20..22] us: the fp32 MFMA chain with a 16-cycle s_nop after every MFMA, alone; the global-load
 *            chain and the LDS chain beside three such waves per SIMD
 * Synchronous (a few milliseconds).  EVCONV_ERR_INVALID_ARG for a null pointer or too little
 * room, EVCONV_ERR_HIP if a launch or copy fails. */
#define EVCONV_CHIP_PROBE_VALUES 23
#define EVCONV_CHIP_PROBE_SCRATCH_BYTES (1u << 20)
evconv_status evconv_debug_chip_probes(void* scratch /* DEVICE */, size_t scratch_bytes, void* hip_stream,
                                       float* out /* HOST */, int32_t n_out);

/* Name of the kernel family that executes a node ("conv_valu_f32", "conv_mfma_f32", ...).  A node
 * that another node's kernel computes reports where it went: "fused_into_conv_epilogue" (an ADD
 * applied by the producing convolution; its buffers are still written), "fused_into_conv_gather",
 * "fused_into_conv_weights", "fused_into_concat_gather" (an up-sampling that exists only inside
 * its consumer: such a node keeps no state and evconv_get_state fails for it).  The planner
 * switches EVCONV_FLAG_* of the description turn these off for tests and comparisons. */
const char* evconv_node_kernel(const evconv_net* net, int32_t node);

/* Text of the last error on this net (or of the last failed create when net is NULL). */
const char* evconv_last_error(const evconv_net* net);

#ifdef __cplusplus
}
#endif
#endif /* EVCONV_H */
