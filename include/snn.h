/*
 * snn.h - C ABI of the MI355X (gfx950) library for surrogate-gradient BPTT
 * training of layered leaky-integrate-and-fire (LIF) spiking networks.
 *
 * The network is the stack of the paper's Section 2.1.2 network listing:
 *     Linear(no bias) -> LIF -> ... -> Linear(no bias) -> LI readout
 * Layers l = 1..L-1 are spiking (LIF, optionally recurrent), layer L is the
 * non-spiking leaky readout with C = sizes[L] classes.  One training step is
 * snn_forward + snn_backward + snn_sgd_step.
 *
 * Conventions
 *   - Every tensor with a time axis is time-major [T][B][N], N fastest.
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are ordinary
 *     host memory.  The library never allocates device memory: the caller
 *     hands over one workspace (snn_workspace_bytes) and keeps it, the input
 *     raster and the labels alive until the calls that use them have finished
 *     on the stream.
 *   - All kernels are enqueued on the HIP stream given to snn_init.  Calls
 *     return after enqueueing unless stated otherwise.
 *   - Every function returns an snn_status; nothing throws or exits.  After
 *     a non-zero status snn_last_error(ctx) describes it.
 *   - There is no CPU fallback: without a usable HIP device snn_init fails
 *     with SNN_ERR_HIP.
 *   - Size limit (hard): the kernels address a tensor with 32-bit byte offsets, so
 *     every [T][B][N_l] tensor must stay below 2 GiB at 4 bytes per element
 *     (T * B * (N_l + 8) * 4 < 2^31 for every l); larger configurations are
 *     refused by snn_workspace_bytes / snn_init with SNN_ERR_ARG, not tiled.
 *     At most SNN_MAX_LAYERS weight matrices.
 *   - The library reads no environment variable.  Which kernels a context uses
 *     for a step is decided from its shapes; snn_set_option overrides that
 *     choice per context (for tests and tuning).
 */
#ifndef SNN_H_
#define SNN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct snn_ctx snn_ctx;          /* opaque, host side */

#define SNN_MAX_LAYERS 12                /* weight matrices per network (spiking layers + readout) */

typedef enum {
  SNN_OK = 0,
  SNN_ERR_NULL = 1,          /* a required pointer was NULL                          */
  SNN_ERR_ARG = 2,           /* value out of range (T,B,N <= 0, beta outside [0,1],
                                theta <= 0, slope <= 0, unknown enum, bad label)    */
  SNN_ERR_SHAPE = 3,         /* byte count does not match the tensor asked for      */
  SNN_ERR_WORKSPACE = 4,     /* workspace too small or not 256-byte aligned         */
  SNN_ERR_STATE = 5,         /* call order: backward needs forward, sgd needs backward */
  SNN_ERR_HIP = 6,           /* a HIP call failed; text in snn_last_error           */
  SNN_ERR_UNSUPPORTED = 7
} snn_status;

/* Backward function of the spiking activation (Section 2.1.1), x = V - theta, k = slope:
 *   SUPERSPIKE  1 / (1 + k|x|)^2                  (surrogate listing, k = 25 in the paper)
 *   ARCTAN      (k/2) / (1 + (pi k x / 2)^2)      (named by the paper; this is the derivative
 *                                                  of (1/pi) atan(pi k x / 2) + 1/2)
 *   SIGMOID     k s (1 - s), s = 1/(1+exp(-k x))
 *   TRIANGULAR  max(0, 1 - |k x|)                 (surrogate listing)
 *   BOXCAR      1/2 where |k x| <= 1, else 0      (named by the paper; width 2/k, height 1/2)
 *   STE         1                                 (straight-through estimator, the default the
 *                                                  paper states for its activation builder)
 * The forward function is always the Heaviside step with no spike at x == 0. */
typedef enum {
  SNN_SURR_SUPERSPIKE = 0,
  SNN_SURR_ARCTAN = 1,
  SNN_SURR_SIGMOID = 2,
  SNN_SURR_TRIANGULAR = 3,
  SNN_SURR_BOXCAR = 4,
  SNN_SURR_STE = 5
} snn_surrogate;

/* Arithmetic of the matrix products.  State, surrogate, loss and accumulation are fp32 in
 * both modes; spikes are exact 0/1 in both.
 *   FP32       real operands are split into three bfloat16 pieces (hi+mid+lo = the fp32
 *              value) and every needed piece product is accumulated in fp32 on the MFMA
 *              units: products with a 0/1 operand are exact.
 *   BF16_GEMM  the weights W and R are rounded once to bfloat16 (round to nearest even)
 *              wherever they enter a product, forward and backward; the current gradients
 *              enter their products as a hi+lo pair of bfloat16 (error below 2^-16
 *              relative), so the result is the gradient of the rounded-weight network. */
typedef enum { SNN_PREC_FP32 = 0, SNN_PREC_BF16_GEMM = 1 } snn_precision;

/* How the readout trace y_t is reduced over time before the softmax cross-entropy (mean over
 * the batch):
 *   MAX_OVER_TIME  z = max_t y_t; the gradient goes to the first maximising step
 *   INTEGRAL       z = sum_t y_t (the integral cross-entropy Section 2.1.3 names for
 *                  rate-coded objectives; no label smoothing) */
typedef enum {
  SNN_LOSS_MAX_OVER_TIME = 0,
  SNN_LOSS_INTEGRAL = 1
} snn_loss;

typedef struct {
  int32_t T;                 /* time steps                                              */
  int32_t B;                 /* batch                                                   */
  int32_t n_layers;          /* L = number of weight matrices = spiking layers + readout */
  const int32_t *sizes;      /* host, L+1 entries: N_0 (input) .. N_L (classes)         */
  const uint8_t *recurrent;  /* host, L-1 flags (may be NULL = none): 1 = recurrent LIF */
  const float *beta;         /* host, L entries in [0,1]; last one is the readout's     */
  float threshold;           /* theta > 0                                               */
  int32_t surrogate;         /* snn_surrogate                                           */
  float slope;               /* k > 0                                                   */
  int32_t precision;         /* snn_precision                                           */
  int32_t loss;              /* snn_loss                                                */
  int32_t learn_beta;        /* 0: decays fixed.  1: the per-neuron decays are trained as in
                                the LIF listing (Section 2.1.2): snn_backward also yields
                                dL/dbeta, snn_sgd_step also does beta <- clip(beta - lr
                                dbeta, 0, 1).  Either way every neuron (and readout class)
                                has its own decay, initialised from `beta` and settable   */
  const float *adapt_decay;  /* host, L-1 entries in [0,1], or NULL                      */
  const float *adapt_step;   /* host, L-1 entries >= 0, or NULL (both NULL: no layer adapts).
                                Neurons with an adaptive firing threshold (named in Section
                                2.1.2, which gives no equations; this is the reading built
                                here): a spiking layer with adapt_step > 0 carries a second
                                state A_t >= 0, A_0 = 0, and Eq. 1-2 take the threshold in
                                force theta_t = theta + A_t:
                                  S_t = H(V_t - theta_t), V_{t+1} = beta V_t + X_t - theta_t S_t,
                                  A_{t+1} = adapt_decay A_t + adapt_step S_t.
                                The reverse sweep runs through both states.  adapt_step = 0:
                                plain LIF.  Feed-forward layers only: a layer that is both
                                recurrent and adaptive is refused with SNN_ERR_UNSUPPORTED.  */
} snn_config;

/* Tensors that snn_get_tensor / snn_set_tensor move.  `layer` is 1-based as in the text:
 * weights 1..L, spiking-layer tensors 1..L-1, readout tensors ignore it.  Element type on
 * the host side is float unless noted; shapes are dense (no padding). */
typedef enum {
  SNN_T_WEIGHT = 0,      /* [N_{l-1}][N_l]  fp32 master weights (settable)                 */
  SNN_T_RWEIGHT = 1,     /* [N_l][N_l] (from,to), recurrent layers only (settable)         */
  SNN_T_GRAD_W = 2,      /* [N_{l-1}][N_l]                                                 */
  SNN_T_GRAD_R = 3,      /* [N_l][N_l]                                                     */
  SNN_T_CURRENT = 4,     /* I^l [T][B][N_l] (settable)                                     */
  SNN_T_MEMBRANE = 5,    /* V^l [T][B][N_l]: potential the spike decision used (settable)  */
  SNN_T_SPIKES = 6,      /* S^l [T][B][N_l], uint8 0/1 (settable)                          */
  SNN_T_D_SPIKES = 7,    /* dL/dS^l [T][B][N_l] (settable)                                 */
  SNN_T_D_CURRENT = 8,   /* dL/dI^l [T][B][N_l] (settable)                                 */
  SNN_T_READOUT_CURRENT = 9,  /* J [T][B][C] (settable)                                    */
  SNN_T_READOUT_TRACE = 10,   /* Y [T][B][C]                                               */
  SNN_T_LOGITS = 11,     /* z [B][C] = max_t Y                                             */
  SNN_T_ARGMAX_T = 12,   /* t* [B][C], int32: first maximising step (settable)             */
  SNN_T_D_LOGITS = 13,   /* dL/dz [B][C] (settable)                                        */
  SNN_T_D_READOUT_CURRENT = 14, /* dL/dJ [T][B][C] (settable)                                */
  SNN_T_LOSS = 15,       /* 1 float                                                        */
  SNN_T_LOSS_PER_SAMPLE = 16, /* [B]                                                       */
  SNN_T_BETA = 17,       /* [N_l] decays of layer l (1..L, L = readout), in [0,1] (settable)   */
  SNN_T_GRAD_BETA = 18,  /* [N_l] dL/dbeta of layer l; needs learn_beta (else SNN_ERR_STATE)   */
  SNN_T_ADAPTATION = 19  /* A^l [T][B][N_l]: threshold adaptation in force at each step, layers
                            with adapt_step > 0 only (else SNN_ERR_ARG) (settable)            */
} snn_tensor;

/* Single steps of the path, for kernel-level tests on imposed inputs (snn_run_step). */
typedef enum {
  SNN_STEP_CURRENT_GEMM = 0,   /* I^l = S^{l-1} W^l (layer L: J = S^{L-1} W^L)             */
  SNN_STEP_LIF_FORWARD = 1,    /* I^l -> V^l, S^l (recurrent layers: includes S R; adaptive: A^l) */
  SNN_STEP_READOUT_FORWARD = 2,/* J -> Y, z, t*, loss, dz                                  */
  SNN_STEP_READOUT_REVERSE = 3,/* dz, t* -> dJ                                             */
  SNN_STEP_LIF_REVERSE = 4,    /* dS^l, V^l (adaptive layers: and A^l) -> dI^l             */
  SNN_STEP_WEIGHT_GRAD = 5,    /* dW^l = S^{l-1}^T dI^l (and dR^l); layer L uses dJ        */
  SNN_STEP_INPUT_GRAD = 6      /* dS^{l-1} = dI^l W^l^T, l >= 2                            */
} snn_step;

/* Kernel classes for the built-in event timer (snn_profile_*). */
typedef enum {
  SNN_K_NONE = -1,
  SNN_K_CURRENT_GEMM = 0, SNN_K_LIF_FORWARD = 1, SNN_K_RLIF_FORWARD = 2,
  SNN_K_READOUT_FORWARD = 3, SNN_K_READOUT_REVERSE = 4, SNN_K_LIF_REVERSE = 5,
  SNN_K_RLIF_REVERSE = 6, SNN_K_WEIGHT_GRAD = 7, SNN_K_INPUT_GRAD = 8, SNN_K_SGD = 9,
  SNN_K_CALIBRATE = 10,        /* once per snn_backward, between two launches: a bracket around a
                                  one-wavefront kernel that waits SNN_CALIBRATE_US on the device
                                  clock; elapsed - SNN_CALIBRATE_US is what a bracket adds to the
                                  kernel it times (launched only while this class is selected) */
  SNN_K_GRAD_REDUCE = 11,      /* the launch that adds the per-split partial sums of the weight
                                  gradients (SNN_K_WEIGHT_GRAD covers the products alone)      */
  SNN_K_EVENT_PAIR = 12,       /* once per snn_backward: a bracket around nothing.  Its elapsed time is
                                  what an event pair itself adds to the stream; a bracketed kernel's
                                  elapsed time minus this is the kernel's own duration             */
  SNN_K_COUNT = 13
} snn_kernel_class;
#define SNN_CALIBRATE_US 10

/* Kernel-selection options of a context (snn_set_option).  Every choice computes the same step
 * of the path; results differ only in the order floating-point sums are taken.  The defaults
 * are the measured best; the tests use the options to reach each kernel on small shapes.
 *   LAYER_FORWARD     feed-forward spiking layers of 64..LAYER_MAX_NEURONS padded neurons on
 *                     rounded weights run product and scan as ONE launch (Eq. 1-2 with the
 *                     preceding Linear layer): 0 never; 1 all but the last spiking layer;
 *                     2 every such layer; 3 the last one also forms the readout's currents
 *                     (128 padded neurons, at most 32 padded classes); 4 (default) and runs the
 *                     readout scan, the loss and the readout's current gradients
 *   LAYER_PAIR        1 (default): two consecutive one-launch layers of exactly 128 padded
 *                     neurons share a launch; 0: one launch each; 2: they share a launch with a
 *                     workgroup per layer and sample, the upper layer's following the lower
 *                     layer's through memory 64 steps at a time (measured slower: 32.9 against
 *                     27.7 us at 700-128-128-20, T = 128, B = 256; the upper layer's chain per 64
 *                     steps is longer than the lower layer's scan of them, and starts only once the
 *                     lower layer's whole product is done)
 *   LAYER_REVERSE     1 (default): the reverse pass of a layer of 64..256 neurons below a layer of
 *                     at most 128 columns runs as one launch (dS product, surrogate, scan; dS is
 *                     not stored); 2: so does that of a layer that is a multiple of 128 wide below a
 *                     wider layer (measured slower than product + scan, hence not the default);
 *                     0: off
 *   TOP_SCANS         1 (default): the scans of a layer below at most 128 columns form the
 *                     narrow products themselves (readout currents forward, dS reverse); 0: off
 *   DEFER_REDUCE      1 (default): snn_backward leaves the per-split partial sums of the weight
 *                     gradients to snn_sgd_step (or the first reader); 0: it adds them itself
 *   LAYER_MIN_BATCH   smallest batch for the one-launch layers; 0 (default) = 1 for rasters of up
 *                     to 256 steps, else 64
 *   LAYER_NEURONS     neurons per workgroup of the one-launch forward layers: 128 (default) or 64
 *   LAYER_MAX_NEURONS widest layer (and fan-in) that runs as one launch: 64..1024 (default 1024)
 *   STREAM_MIN_MB     tensors of at least this many MiB count as streaming past the caches
 *                     (non-temporal accesses, the streamed current product); default 128
 *   STREAM_GEMM       1 (default): such current products use the streamed kernel; 0: the general one
 *   TILE_ROWS         rows per workgroup tile of the general products: 0 (default) = by shape,
 *                     or 32, 64, 128
 *   LAYER_TIME_SPLIT  0 (default): one workgroup per sample, blocks of 128 steps; 1: a one-launch
 *                     forward layer of 128 neurons per workgroup gives each sample to two workgroups
 *                     that take its blocks of 64 steps in turn (the product of the next block runs
 *                     while this one is scanned; the state is handed over through memory).  Measured
 *                     no faster at 700-128-128-20, T = 128, B = 256 (each workgroup still loads all of
 *                     W per block, and the loads are what bounds the product): on request only
 *   WGRAD_TR          1 (default): weight-gradient products wider than 64 columns on rounded weights use
 *                     the kernel that brings both operand tiles into LDS as they lie in memory and
 *                     reads the MFMA fragments through the transposing LDS reads; 0: the general
 *                     product kernel, which transposes in registers
 *   RLIF_PERSIST      1 (default): the forward time loop of a recurrent layer wider than 128 neurons on rounded
 *                     weights runs as ONE launch when its grid of 32 x 32 tiles fits the compute units at a
 *                     workgroup each and its padded width is a multiple of 256 up to 2048 (weights resident
 *                     in LDS, spikes exchanged as bits through memory, a counter per sample tile; a wait that
 *                     times out after about a second is reported as SNN_ERR_HIP); 0: a launch per step
 *                     (LAYER_TIME_SPLIT = 1 and LAYER_PAIR = 2 tell one launch from the next by a count that the
 *                     host passes as a kernel argument: do not replay calls made under them from a captured
 *                     graph.  Everything else enqueues kernels only - no host read-back unless a loss pointer
 *                     is given, no allocation, fill kernels instead of memsets - and can be captured.)
 *   WAIT_LIMIT_LOG2   a workgroup of that launch polls at most 2^value times for another one's words:
 *                     4..20 (default 18, about a second)
 *   WAIT_FAULT        0 (default); 1: every such wait expects words that nobody writes, so it times out and
 *                     the launch ends the way it would if a workgroup were missing (the grid drains, the next
 *                     call that reads the error word returns SNN_ERR_HIP).  For tests of that path. */
typedef enum {
  SNN_OPT_LAYER_FORWARD = 0,
  SNN_OPT_LAYER_PAIR = 1,
  SNN_OPT_LAYER_REVERSE = 2,
  SNN_OPT_TOP_SCANS = 3,
  SNN_OPT_DEFER_REDUCE = 4,
  SNN_OPT_LAYER_MIN_BATCH = 5,
  SNN_OPT_LAYER_NEURONS = 6,
  SNN_OPT_LAYER_MAX_NEURONS = 7,
  SNN_OPT_STREAM_MIN_MB = 8,
  SNN_OPT_STREAM_GEMM = 9,
  SNN_OPT_TILE_ROWS = 10,
  SNN_OPT_LAYER_TIME_SPLIT = 11,
  SNN_OPT_WGRAD_TR = 12,
  SNN_OPT_RLIF_PERSIST = 13,
  SNN_OPT_WAIT_LIMIT_LOG2 = 14,
  SNN_OPT_WAIT_FAULT = 15,
  SNN_OPT_COUNT = 16
} snn_option;

/* Validate `cfg` and report the device bytes snn_init needs (a multiple of 256).
 * Pure host code.  Errors: SNN_ERR_NULL, SNN_ERR_ARG. */
int32_t snn_workspace_bytes(const snn_config *cfg, size_t *bytes);

/* Build a network: the stack Linear(no bias) -> LIF -> ... -> Linear(no bias) -> LI of the
 * network listing in Section 2.1.2 (initial potentials zero, as its initial_state does),
 * optionally with recurrent LIF layers.  `workspace_dev`: device memory, 256-byte aligned, at least
 * snn_workspace_bytes(cfg) bytes, owned by the caller, used exclusively by this context
 * until snn_destroy.  `W_host`: L host pointers, W_host[l] row-major [N_l][N_{l+1}]
 * (in, out), i.e. I = S W as in the paper's Linear layers without bias.  `R_host`: L-1
 * host pointers ([N][N], (from, to)), entries for non-recurrent layers ignored; may be
 * NULL when no layer is recurrent.  Weights are copied; the host arrays may be freed on
 * return.  `hip_stream`: a hipStream_t (NULL = the default stream).  Synchronises the
 * stream before returning.  Errors: NULL/ARG/WORKSPACE/HIP. */
int32_t snn_init(const snn_config *cfg, void *workspace_dev, size_t workspace_bytes,
                 const float *const *W_host, const float *const *R_host,
                 void *hip_stream, snn_ctx **out);

/* Forward pass (Eq. 1-2 per spiking layer, LI readout, softmax cross-entropy on the
 * max-over-time readout, mean over the batch).
 *   x_dev       device, uint8 [T][B][N_0], values 0 or 1 (anything non-zero counts as 1
 *               is NOT promised: other values are a caller error)
 *   labels_dev  device, int32 [B], each in [0, C)
 *   loss_host   host float, may be NULL.  If given, the call waits for the stream and
 *               stores the loss; a label outside [0,C) then yields SNN_ERR_ARG.
 * x_dev and labels_dev must stay valid until the following snn_backward has finished. */
int32_t snn_forward(snn_ctx *ctx, const uint8_t *x_dev, const int32_t *labels_dev,
                    float *loss_host);

/* The same with the input raster packed along time, eight spikes per byte, as the paper
 * keeps its datasets on the device (Section 2.1.4, numpy.packbits along the temporal axis)
 * and decompresses them batch by batch inside the training step:
 *   x_packed_dev  device, uint8 [ceil(T/8)][B][N_0]; bit 7-(t%8) of byte [t/8][b][n] is
 *                 the spike at step t (the first step in the most significant bit; bits
 *                 of steps >= T are ignored)
 * Where layer 1 runs as one launch (feed-forward, a multiple of 64 neurons wide, rounded
 * weights, at most 1024 input channels in rows of a multiple of 4 bytes) that launch reads the
 * packed raster itself and unpacks between its LDS read and the MFMA, and so does the weight-
 * gradient product of layer 1 in snn_backward when B is a multiple of 8; nothing is unpacked in
 * memory then.  Other shapes are unpacked into the workspace by a pre-pass.  x_packed_dev must
 * stay valid until the following snn_backward has finished.  Everything else as for
 * snn_forward. */
int32_t snn_forward_packed(snn_ctx *ctx, const uint8_t *x_packed_dev, const int32_t *labels_dev,
                           float *loss_host);

/* Reverse sweep: what reverse-mode differentiation of the unrolled forward loop computes
 * (Section 2.1.3 takes the gradient of the loss with jax.value_and_grad), with the derivative
 * of the Heaviside step replaced by the surrogate's backward function (Section 2.1.1): readout
 * gradient, per spiking layer the reverse-time scan with the fused
 * surrogate derivative, the weight-gradient products dW^l = S^{l-1}^T dI^l (dR^l =
 * S^l^T dI^l) and the input-gradient products dS^{l-1} = dI^l W^l^T.  Needs a preceding
 * snn_forward on the current weights (else SNN_ERR_STATE).
 * The weight-gradient products are split along the T*B rows; the sum of the splits' partial
 * results may be left to the next call that needs it (snn_sgd_step, or snn_get_tensor /
 * snn_run_step, which add them first): the gradients a caller sees are the same either way. */
int32_t snn_backward(snn_ctx *ctx);

/* The optimiser update that the training-loop listing of Section 2.1.4 fuses with the gradient
 * computation into one compiled step; the paper names no optimiser, this is plain SGD:
 * W <- W - lr dW, R <- R - lr dR on the fp32 masters, then refresh the bfloat16 operand
 * copies the products read.  Needs a preceding snn_backward (else SNN_ERR_STATE). */
int32_t snn_sgd_step(snn_ctx *ctx, float lr);

/* Copy a tensor to / from dense host memory.  `bytes` must equal the tensor's dense size
 * (else SNN_ERR_SHAPE).  Both wait for the stream.  snn_set_tensor accepts the tensors
 * marked settable; setting a weight also refreshes its bfloat16 copies, and setting a weight or
 * the decays invalidates a previous forward (snn_backward then needs a new one).
 * snn_get_tensor reports a pending bad-label flag as SNN_ERR_ARG. */
int32_t snn_get_tensor(snn_ctx *ctx, int32_t tensor, int32_t layer, void *dst_host, size_t bytes);
int32_t snn_set_tensor(snn_ctx *ctx, int32_t tensor, int32_t layer, const void *src_host,
                       size_t bytes);

/* Run one step of the path for one layer on whatever the context's buffers hold (for
 * tests that impose a step's inputs with snn_set_tensor).  `x_dev` is needed when the step
 * reads the input raster (CURRENT_GEMM and WEIGHT_GRAD of layer 1), `labels_dev` for
 * READOUT_FORWARD; otherwise they may be NULL.  Does not change the forward/backward
 * call-order state. */
int32_t snn_run_step(snn_ctx *ctx, int32_t step, int32_t layer, const uint8_t *x_dev,
                     const int32_t *labels_dev);

/* Set / read a kernel-selection option (snn_option) of this context.  Takes effect from the
 * next call on.  Errors: SNN_ERR_NULL; SNN_ERR_ARG for an unknown option or a value outside the
 * range listed with the option (the option keeps its value). */
int32_t snn_set_option(snn_ctx *ctx, int32_t option, int32_t value);
int32_t snn_get_option(const snn_ctx *ctx, int32_t option, int32_t *value);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc) and have no workspace to hand over: the weight-gradient
 * product of one layer, the step snn_run_step(SNN_STEP_WEIGHT_GRAD) runs inside a context, with
 * the per-split partial sums in a static device array of SNN_STATIC_SCRATCH_BYTES that every GPU
 * the library runs on holds until the process ends.  Allocates nothing, on the device or through
 * any library.
 *   S_dev   device, uint8 [M][K], values 0 or 1: the spikes below the layer, M = T*B rows
 *   G_dev   device, float [M][N]: the layer's current gradients dL/dI
 *   dW_dev  device, float [K][N]: receives S^T G (every element written; fp32-exact products,
 *           fixed summation order, so the result is bit-repeatable)
 * K and N multiples of 4; S_dev 4-byte aligned, G_dev and dW_dev 16-byte aligned (else
 * SNN_ERR_ARG).  Sizes beyond the scratch are refused with SNN_ERR_UNSUPPORTED: M <=
 * SNN_STATIC_MAX_ROWS, K*N <= SNN_STATIC_MAX_WEIGHTS, M*K < 2^31, M*N*4 < 2^31.  Enqueues on
 * `hip_stream` (NULL = the default stream) and returns; runs on the current device.  All calls on
 * one GPU share that GPU's array: calls that may overlap on one GPU (different streams, several
 * threads) race and must be ordered by the caller.  Error text: snn_last_error(NULL). */
#define SNN_STATIC_SCRATCH_BYTES (16u << 20)
#define SNN_STATIC_MAX_ROWS (1 << 24)
#define SNN_STATIC_MAX_WEIGHTS (1 << 21)
int32_t snn_weight_grad_static(const uint8_t *S_dev, const float *G_dev, float *dW_dev, int64_t M,
                               int32_t K, int32_t N, void *hip_stream);

/* Event timer.  snn_profile_select(ctx, k, layer) brackets every later launch of kernel
 * class k (layer = 0: all layers, else that layer only) with a pair of HIP events on the
 * library's stream; k = SNN_K_NONE switches it off and clears the totals.
 * snn_profile_read waits for the stream and returns the summed elapsed milliseconds and
 * the number of bracketed launches since the last select. */
int32_t snn_profile_select(snn_ctx *ctx, int32_t kernel_class, int32_t layer);
/* Bracket only every n-th matching launch (n >= 1, default 1; counted from the next select on):
 * an event pair costs a few microseconds on the stream, which a timed loop that wants the
 * kernel's average duration, not every sample of it, need not pay at every step.  For
 * callers that time whole steps while the timer is on (the bench). */
int32_t snn_profile_every(snn_ctx *ctx, int32_t n);
int32_t snn_profile_read(snn_ctx *ctx, double *total_ms, int64_t *launches);

/* Free the host-side context (the workspace stays the caller's).  Waits for the stream. */
int32_t snn_destroy(snn_ctx *ctx);

/* Text of the last error of this context (ctx == NULL: of the last failed call that had no
 * context, e.g. snn_init).  Owned by the library, valid until the next call. */
const char *snn_last_error(const snn_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* SNN_H_ */
